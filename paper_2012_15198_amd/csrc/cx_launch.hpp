// Host side of the device half (internal header): launch shapes, the row-order table's slots, the two
// launchers and the argument checks shared by the entry points.  Each cx_api_*.hip includes this header and
// defines its entry points, so the operators compile in parallel; everything has internal linkage (each
// translation unit carries its own row-order table).
#ifndef CX_LAUNCH_HPP
#define CX_LAUNCH_HPP
#include "cx_kernels.hpp"

namespace {

// ---------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------
struct Launch {
    int U, D, waves, nt, lockstep, wgs_per_cu;
};

Launch pick_launch(const WalkShape &dflt)
{
    Launch l;
    l.U = cx_get_tuning(0);
    if (l.U != 1 && l.U != 2 && l.U != 4) l.U = dflt.U;
    l.lockstep = cx_get_tuning(4) == 0 ? 0 : 1;
    l.waves = cx_get_tuning(1);
    if (l.waves < 1 || l.waves > kMaxWavesPerBlock) l.waves = dflt.waves;
    l.nt = cx_get_tuning(2);
    if (l.nt != 0 && l.nt != 1) l.nt = 1;
    l.D = cx_get_tuning(3);
    if (l.D != 2 && l.D != 4 && l.D != 8) l.D = dflt.D;
    l.wgs_per_cu = cx_get_tuning(9);
    if (l.wgs_per_cu < 0 || l.wgs_per_cu > 16) l.wgs_per_cu = dflt.wgs_per_cu;
    return l;
}

[[maybe_unused]] bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// true if the byte ranges [a, a+bytes) and [b, b+bytes) overlap without being identical
[[maybe_unused]] bool partial_overlap(const void *a, const void *b, uint64_t bytes)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    if (x == y) return false;
    return x < y ? (y - x) < bytes : (x - y) < bytes;
}
[[maybe_unused]] bool any_overlap(const void *a, const void *b, uint64_t bytes)
{
    return a == b || partial_overlap(a, b, bytes);
}

struct MixArgs {
    int n;
    int64_t P;
    int S;
    const int64_t *seg_off;
    const int32_t *peers;
    int shift, skip_mix;
    hipStream_t stream;
    bool out_of_place;          // every output buffer is distinct from its input buffer
    int rows_per_gossip_row;    // G: matrix rows behind one gossiping row (cluster footprint)
    // Row-order table supplied by the entry point instead of one of the library's per-stream
    // slots: its capacity in words and where to get its device address once the workload is known
    // to fit (the call fails with CX_ERR_SHAPE rather than run without a table when it does not).
    unsigned *(*order_provider)() = nullptr;
    int64_t order_entries = 0;
};

// Dynamic LDS a workgroup reserves so that at most `wgs_per_cu` of them are resident on a CU
// (0 = no cap).  Fewer resident workgroups keep fewer bytes in flight per CU, which this
// memory system rewards for the row-wandering walk (+3 to +8 %) and for the fused gather
// (+2 %).  A CU has 160 KB of LDS; a workgroup may take up to 64 KB.
[[maybe_unused]] size_t lds_reservation(int wgs_per_cu)
{
    if (wgs_per_cu <= 0) return 0;
    const size_t reserve = (160u << 10) / static_cast<unsigned>(wgs_per_cu);
    return reserve > (64u << 10) ? (64u << 10) : reserve;
}

// A (slices, depth) pair is built for an operator only if its ring of in-flight rows stays
// within the register file without spilling (at least two waves per SIMD stay resident).
template <class Op, class = void>
struct MaxSlices {
    static constexpr int value = 4;
};
template <class Op>
struct MaxSlices<Op, std::void_t<decltype(Op::kMaxU)>> {
    static constexpr int value = Op::kMaxU;                // an operator may build fewer shapes
};

template <class Op, int U, int D>
constexpr bool fits()
{
    // registers of the ring of rows in flight plus the four working tiles of the walk: a
    // workgroup of eight waves leaves each wave 256 registers
    return U <= MaxSlices<Op>::value &&
           Op::kRawPerSlice * U * D * 4 + 4 * Op::template Work<U>::kN * Op::template Work<U>::kRegs <= 224 &&
           Op::kRawPerSlice * U * D * 4 <= 144 && !(U == 4 && Op::kRawPerSlice * D >= 8);
}

template <class Op, int U, int D>
bool try_launch(const Op &op, const Launch &l, const MixArgs &a)
{
    if (l.U != U || l.D != D) return false;
    if constexpr (!fits<Op, U, D>()) {
        return false;
    } else {
        const int64_t tile_cols = static_cast<int64_t>(kWave) * Op::kElems * U;
        const int64_t ntiles = (a.P + tile_cols - 1) / tile_cols;
        int waves = l.waves;
        while (waves > 1 && (sizeof(int) * kScheduleWords(a.n) + StageBytes<Op>::value) * waves > 48 * 1024) --waves;
        const int64_t nblocks = (ntiles + waves - 1) / waves;
        const dim3 grid(static_cast<unsigned>(nblocks)), block(kWave * waves);
        const size_t schedules = (sizeof(int) * kScheduleWords(a.n) * waves + 15) / 16 * 16;
        size_t lds = schedules + static_cast<size_t>(StageBytes<Op>::value) * waves;
        if (lds < lds_reservation(l.wgs_per_cu)) lds = lds_reservation(l.wgs_per_cu);
        const Op staged = with_stage_base(op, schedules);
        if (l.nt)
            hipLaunchKernelGGL((mix_kernel<Op, U, D, true>), grid, block, lds, a.stream, staged, a.n, a.P,
                               a.S, a.seg_off, a.peers, a.shift, a.skip_mix, ntiles, l.lockstep);
        else
            hipLaunchKernelGGL((mix_kernel<Op, U, D, false>), grid, block, lds, a.stream, staged, a.n, a.P,
                               a.S, a.seg_off, a.peers, a.shift, a.skip_mix, ntiles, l.lockstep);
        return true;
    }
}

// Device address of this translation unit's g_order on the current device.  In host code the
// array's name is only a handle: the address comes from hipGetSymbolAddress, once per device.
constexpr int kMaxDevices = 64;
unsigned *order_tables_base(int *device_out)
{
    static std::mutex mu;
    static unsigned *base[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    *device_out = dev;
    std::lock_guard<std::mutex> lock(mu);
    if (!base[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_order)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        base[dev] = static_cast<unsigned *>(p);
    }
    return base[dev];
}

// Serialises "order_kernel, then gather_kernel" of one call against other host threads, so
// that two threads enqueueing on one stream cannot interleave their pairs.
std::mutex &enqueue_mutex()
{
    static std::mutex mu;
    return mu;
}

// The order table `stream` may write on the current device, or nullptr (run without one).
// A stream keeps the slot it used last.  When every slot belongs to another stream, a slot
// whose owner has no work in flight (or no longer exists) changes hands.  Calls recorded under
// stream capture get a slot of their own, apart from the one the same stream uses for eager
// calls, and keep it for good: the captured graph names it, and may be replayed on any stream
// while eager calls go on.  (Graphs captured on ONE stream share that slot: replay them in
// one stream's order.)
unsigned *order_table_for(hipStream_t stream)
{
    struct Slot {
        hipStream_t owner;
        bool used, for_capture;
    };
    static Slot slots[kMaxDevices][kOrderSlots];
    int dev = 0;
    unsigned *base = order_tables_base(&dev);
    if (!base) return nullptr;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    const bool capturing = hipStreamIsCapturing(stream, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone;
    Slot *mine = slots[dev];
    int slot = -1;
    for (int i = 0; i < kOrderSlots && slot < 0; ++i)
        if (mine[i].used && mine[i].owner == stream && mine[i].for_capture == capturing) slot = i;
    for (int i = 0; i < kOrderSlots && slot < 0; ++i)
        if (!mine[i].used) slot = i;
    // (no questions about other streams while this one records: a capture forbids them)
    for (int i = 0; i < kOrderSlots && slot < 0 && !capturing; ++i) {
        if (mine[i].for_capture) continue;                                        // a graph names it
        hipStreamCaptureStatus ocs = hipStreamCaptureStatusNone;
        const hipError_t q = hipStreamIsCapturing(mine[i].owner, &ocs);
        if (q == hipSuccess && ocs != hipStreamCaptureStatusNone) continue;       // recording: leave it
        const hipError_t busy = q == hipSuccess ? hipStreamQuery(mine[i].owner) : q;
        if (busy == hipErrorNotReady) continue;                                   // work in flight
        if (busy != hipSuccess) (void)hipGetLastError();                          // the stream is gone
        slot = i;
    }
    if (slot < 0) return nullptr;
    mine[slot] = Slot{stream, true, capturing};
    return base + static_cast<int64_t>(slot) * kOrderEntries;
}

// Out-of-place launch: one workgroup per (gossiping row, chunk of waves * 64 * U slices).
template <class Op, int U>
bool try_gather(const Op &op, int want_u, int waves, int nt, int cl_req, int xcd_aware, const MixArgs &a,
                int *status)
{
    if (want_u != U) return false;
    if constexpr (U > MaxSlices<Op>::value) {
        return false;
    } else {
    const int64_t chunk_cols = static_cast<int64_t>(kWave) * Op::kElems * U * waves;
    const int64_t nchunks = (a.P + chunk_cols - 1) / chunk_cols;
    const int nxcd = xcd_aware ? 8 : 1;
    // Rows in cycle order pay when the partner's fetch has to be kept out of HBM; a matrix that
    // the last-level cache holds whole gains nothing from the extra launch.
    const int64_t matrix_bytes = static_cast<int64_t>(a.n) * a.rows_per_gossip_row * a.P * (16 / Op::kElems);
    const bool own_table = a.order_provider != nullptr;
    bool ordered = a.n > 1 && a.S <= 4096 &&
                   (own_table || cx_get_tuning(8) == 1 || (cx_get_tuning(8) != 0 && matrix_bytes > (64LL << 20)));
    if (own_table && !ordered) { *status = CX_ERR_SHAPE; return true; }
    std::lock_guard<std::mutex> enqueue_lock(enqueue_mutex());
    unsigned *order = nullptr;
    const int64_t order_entries = own_table ? a.order_entries : kOrderEntries;
    if (ordered && !own_table) {
        order = order_table_for(a.stream);
        if (!order) ordered = false;
    }
    int64_t cl = cl_req;
    if (cl < 1) {
        // ordered rows: the operator's visit length per XCD (shorter visits lose DRAM row
        // locality, longer ones push the previous visit out of L2);
        // natural row order: the whole cluster (all rows) should fit one XCD's 4 MB L2
        const int64_t row_bytes = chunk_cols * (16 / Op::kElems) * a.rows_per_gossip_row;
        cl = ordered ? (static_cast<int64_t>(VisitKb<Op>::of(a.n)) << 10) / row_bytes : (4 << 20) / (row_bytes * a.n);
        if (cl < 1) cl = 1;
    }
    if (ordered) {                                // the order table must fit its slot
        const int64_t max_clusters = order_entries / a.n - nxcd;
        if (max_clusters < 1) { if (own_table) { *status = CX_ERR_SHAPE; return true; } ordered = false; }
        else {
            const int64_t min_cl = (nchunks + max_clusters - 1) / max_clusters;
            if (cl < min_cl) {
                if (own_table) { *status = CX_ERR_SHAPE; return true; }       // beyond the stated maximum
                cl = min_cl;
            }
        }
    }
    if (cl > 4096) cl = 4096;
    int64_t clusters = (nchunks + cl * nxcd - 1) / (cl * nxcd);
    if (clusters > 65535) {                       // grid.z limit: widen the clusters
        cl = (nchunks + 65535LL * nxcd - 1) / (65535LL * nxcd);
        clusters = (nchunks + cl * nxcd - 1) / (cl * nxcd);
    }
    if (cl * nxcd > 0x7fffffffLL || clusters > 65535 || a.n > 65535) { *status = CX_ERR_SHAPE; return true; }
    // the kernel numbers chunks and tiles, the grid's padding included, in 32 bits
    if ((clusters * nxcd * cl + 1) * waves > 0x7fffffffLL) { *status = CX_ERR_SHAPE; return true; }
    if (ordered && clusters * nxcd * a.n > order_entries) {        // table too large: natural row order
        if (own_table) { *status = CX_ERR_SHAPE; return true; }
        ordered = false;
    }
    const dim3 grid(static_cast<unsigned>(cl * nxcd), static_cast<unsigned>(a.n),
                    static_cast<unsigned>(clusters));
    const dim3 block(kWave * waves);
    const int xcd_shift = xcd_aware ? 3 : 0;
    if (!ordered) order = nullptr;
    if (ordered && own_table) {
        order = a.order_provider();
        if (!order) { *status = CX_ERR_HIP; return true; }
    }
    if (ordered) {
        const int64_t nclusters = clusters * nxcd;
        hipLaunchKernelGGL(order_kernel, dim3(a.S), dim3(256), sizeof(int) * kScheduleWords(a.n), a.stream, a.n,
                           a.P, a.S, a.seg_off, a.peers, a.shift, cl * chunk_cols, static_cast<int>(nclusters),
                           order);
        if (hipGetLastError() != hipSuccess) { *status = CX_ERR_HIP; return true; }
    }
    int cap = cx_get_tuning(9);
    if (cap < 0 || cap > 16) cap = Op::kGather.wgs_per_cu;
    size_t glds = lds_reservation(cap);
    if (LdsStaged<Op>::value && glds < LdsStaged<Op>::bytes) glds = LdsStaged<Op>::bytes;
    if (glds < static_cast<size_t>(StageBytes<Op>::value) * waves) glds = static_cast<size_t>(StageBytes<Op>::value) * waves;
    const Op staged = with_stage_base(op, 0);
    if (nt)
        hipLaunchKernelGGL((gather_kernel<Op, U, true>), grid, block, glds, a.stream, staged, a.n, a.P, a.S,
                           a.seg_off, a.peers, a.shift, a.skip_mix, static_cast<unsigned>(nchunks),
                           static_cast<unsigned>(cl), static_cast<unsigned>(waves), xcd_shift, order);
    else
        hipLaunchKernelGGL((gather_kernel<Op, U, false>), grid, block, glds, a.stream, staged, a.n, a.P, a.S,
                           a.seg_off, a.peers, a.shift, a.skip_mix, static_cast<unsigned>(nchunks),
                           static_cast<unsigned>(cl), static_cast<unsigned>(waves), xcd_shift, order);
    *status = hipGetLastError() == hipSuccess ? CX_OK : CX_ERR_HIP;
    return true;
    }
}

template <class Op>
int launch_mix(const Op &op, const MixArgs &a)
{
    constexpr int U0 = Op::kWalk.U, D0 = Op::kWalk.D;
    static_assert(fits<Op, U0, D0>(), "default launch shape must fit");
    if ((a.P + 255) / 256 > 0x7fffffffLL) return CX_ERR_SHAPE;
    if (a.out_of_place && cx_get_tuning(5) != 1) {
        int u = cx_get_tuning(0);
        if (u != 1 && u != 2 && u != 4) u = Op::kGather.U;
        while (u > 1 && Op::kRawPerSlice * u > 8) u >>= 1;   // the rows in flight must fit the registers
        if (Op::kRawPerSlice >= 8 || u > MaxSlices<Op>::value) u = 1;
        int waves = cx_get_tuning(1);
        if (waves < 1 || waves > kMaxWavesPerBlock) waves = Op::kGather.waves;
        const int nt = cx_get_tuning(2) == 0 ? 0 : 1;
        const int cl = cx_get_tuning(6);
        const int xcd_aware = cx_get_tuning(7) == 0 ? 0 : 1;
        int status = CX_OK;
        if (try_gather<Op, 1>(op, u, waves, nt, cl, xcd_aware, a, &status) ||
            try_gather<Op, 2>(op, u, waves, nt, cl, xcd_aware, a, &status) ||
            try_gather<Op, 4>(op, u, waves, nt, cl, xcd_aware, a, &status))
            return status;
    }
    Launch l = pick_launch(Op::kWalk);
    const bool done =
        try_launch<Op, 1, 2>(op, l, a) || try_launch<Op, 1, 4>(op, l, a) || try_launch<Op, 1, 8>(op, l, a) ||
        try_launch<Op, 2, 2>(op, l, a) || try_launch<Op, 2, 4>(op, l, a) || try_launch<Op, 2, 8>(op, l, a) ||
        try_launch<Op, 4, 2>(op, l, a) || try_launch<Op, 4, 4>(op, l, a) || try_launch<Op, 4, 8>(op, l, a);
    if (!done) {                     // requested shape not built for this operator
        l.U = U0;
        l.D = D0;
        try_launch<Op, U0, D0>(op, l, a);
    }
    return hipGetLastError() == hipSuccess ? CX_OK : CX_ERR_HIP;
}

[[maybe_unused]] int check_matrix_args(const void *x_in, const void *x_out, int64_t ld, int64_t rows,
                                       int64_t P, int32_t S, uint32_t flags, int elem_bytes = 4)
{
    if (!x_in || !x_out) return CX_ERR_NULL;
    if (S < 1 || P < 1 || ld < P || rows < 1) return CX_ERR_SHAPE;
    if (rows > (INT64_MAX / 4) / ld) return CX_ERR_SHAPE;
    if (ld % (16 / elem_bytes) != 0 || misaligned(x_in) || misaligned(x_out)) return CX_ERR_ALIGN;
    if (partial_overlap(x_in, x_out, static_cast<uint64_t>(rows) * ld * elem_bytes)) return CX_ERR_ALIAS;
    if (flags != 0) return CX_ERR_UNSUPPORTED;
    return CX_OK;
}

}  // namespace

#endif  // CX_LAUNCH_HPP
