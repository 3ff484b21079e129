// Device half of the gossip-mixing library for gfx950 (MI355X): the mixing kernels behind
// cx_gossip_mix / cx_hier_mix / cx_pushsum_mix / cx_sgd_fused_mix / cx_hier_sgd_fused_mix and
// their 16-bit variants.  Internal header; the pieces: cx_tile.hpp (slices, tiles, fp32 row
// accesses), cx_ops.hpp and cx_ops16.hpp (the row operators), this file (the two kernels and the
// order kernel), cx_launch.hpp (launch shapes, the row-order table's slots, argument checks;
// the header each cx_api_*.hip includes).  Everything has internal linkage.
//
// Mixing is independent per column and every element has to be read once and written once
// (8 B per worker-parameter; 20 B with the fused optimizer), so the whole path is bound by
// HBM bandwidth.  A lane always handles 16-byte column slices (4 fp32 or 8 bfloat16), a
// wavefront 1 KB of contiguous columns per memory instruction.  Two kernels serve the same
// arithmetic:
//
//  gather_kernel (output buffer != input buffer) -- the fast one.
//   * One short-lived workgroup per (gossiping row, column chunk): it loads the row's chunk
//     and its partner's chunk, averages, stores to the other buffer.  Every chunk is
//     fetched twice from L2 but once from HBM: blocks are ordered so that both fetches meet
//     in the L2 of one XCD (block b runs on XCD b mod 8; an XCD walks a cluster of
//     neighbouring chunks row after row; rows follow the cycles of the peer permutation,
//     so a block's partner is the next block's own row).
//   * Long contiguous row visits per XCD keep the DRAM row buffers busy, which a kernel
//     whose waves each wander over all rows cannot do as well.
//   * order_kernel, a few microseconds ahead of it, derives the row order from the
//     device-resident peer table into library-owned device memory (no allocation): one word
//     per (cluster, position) with the row, its partner and a "one segment covers this
//     cluster" bit, so almost every workgroup starts its loads after one scalar load.
//     Workgroups are many and small (one slice per lane for plain gossip): their count of
//     instructions, not only their bytes, decides the rate.
//
//  mix_kernel (in place capable) -- the column-owner cycle walk.
//   * A wavefront owns a tile of 64*U slices (256*U fp32 columns) and visits every row of it.  The peer table
//     of a segment is a permutation, so the rows split into cycles i -> peers[i] -> ...
//     Walking a cycle, the lane keeps the current and the next row's slice in registers,
//     writes (cur + next) * 0.5f to the current row and moves on; the cycle's first slice
//     is kept for its last row.  A row is overwritten only after its two readers have it
//     in registers, so x_out may be x_in.  Loads run D rows ahead of the stores.
//   * The cycle order of a segment is built per wavefront (or once per workgroup in the
//     lock-step variant) in LDS from the peer table; a table that is not a permutation is
//     replaced by the identity, so no row index can leave [0, n).
//
//  Both: tiles wholly inside one segment take the 16-byte vector path; the at most S+1
//  tiles that straddle a segment boundary or the ragged row end run once per overlapped
//  segment with per-element predication.  Row operators (MeanOp / FusedOp / HierFusedOp /
//  PushOp / Row16Op ...) say what loading and storing a "gossiping row" means: the mean of a
//  group of G rows summed in fp64, the momentum-SGD update applied on the way in (to the row or
//  to a group leader fed with the group's mean gradient), the push-sum de-biasing, or the
//  unpacking and rounding of 16-bit rows (bfloat16, binary16).  Each operator also names its
//  measured launch shapes (kGather, kWalk).
#ifndef CX_KERNELS_HPP
#define CX_KERNELS_HPP
#include "cx_ops.hpp"
#include "cx_ops16.hpp"

#pragma clang fp contract(off)

namespace {

// The two groups that build schedules: one wavefront in its private LDS region, or a workgroup.
struct WaveSync {
    __device__ __forceinline__ void sync() const { wave_sync(); }
    __device__ __forceinline__ void add(int *p, int v) const { atomicAdd(p, v); }
};
struct BlockSync {
    __device__ __forceinline__ void sync() const { __syncthreads(); }
    __device__ __forceinline__ void add(int *p, int v) const { atomicAdd(p, v); }
};

// One lane's walk over all cycles of the schedule, software-pipelined: the global loads of
// the rows of steps k+2 .. k+1+D are in flight while step k is averaged and stored.  Rows
// are fetched in schedule order, each exactly once, into a ring of D register slots
// (statically indexed: the step loop is unrolled by D).  Loads are always issued ahead of
// the store of the current row, so a load never waits behind a store's acknowledgement.
template <class Op, int U, int D, bool FULL, bool NT, bool SYNC = false>
__device__ __forceinline__ void walk(const Op &op, const int *sched, int n, bool skip_mix,
                                     int64_t off, const unsigned (&mask)[U])
{
    using WorkT = typename Op::template Work<U>;
    typename Op::template Raw<U> slot[D];
#pragma unroll
    for (int j = 0; j < D; ++j)
        if (j < n) op.template issue<U, FULL, NT>(uniform(sched[j]) & kRowMask, off, mask, slot[j]);

    int e = uniform(sched[0]);
    WorkT cur;
    op.template finish<U, FULL, NT>(e & kRowMask, off, mask, slot[0], cur);
    if (D < n) op.template issue<U, FULL, NT>(uniform(sched[D]) & kRowMask, off, mask, slot[0]);
    if (skip_mix) {                       // a single gossiping row: nothing to average with
        op.template store<U, FULL, NT>(e & kRowMask, off, mask, cur);
        return;
    }
    WorkT first = cur;
    for (int base = 0; base < n; base += D) {
        static_for<0, D>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            constexpr int kNextSlot = (j + 1) % D;
            const int k = base + j;
            if (k < n) {
                if constexpr (SYNC) __syncthreads();   // the workgroup visits each row together
                WorkT nx;
                int e1 = 0;
                if (k + 1 < n) {          // row of step k+1 arrives; its slot is refilled at once
                    e1 = uniform(sched[k + 1]);
                    op.template finish<U, FULL, NT>(e1 & kRowMask, off, mask, slot[kNextSlot], nx);
                    if (k + 1 + D < n)
                        op.template issue<U, FULL, NT>(uniform(sched[k + 1 + D]) & kRowMask, off, mask,
                                                       slot[kNextSlot]);
                }
                const bool last = (e & kLastBit) != 0;      // row k closes its cycle
                WorkT out;
#pragma unroll
                for (int u = 0; u < WorkT::kN; ++u) out.v[u] = average(cur.v[u], last ? first.v[u] : nx.v[u]);
                op.template store<U, FULL, NT>(e & kRowMask, off, mask, out);
                if (last) first = nx;                       // step k+1 opens the next cycle
                cur = nx;
                e = e1;
            }
        });
    }
}

template <class Op, int U, int D, bool NT>
__global__ __launch_bounds__(kWave *kMaxWavesPerBlock) void mix_kernel(
    Op op, int n, int64_t P, int S, const int64_t *__restrict__ seg_off,
    const int32_t *__restrict__ peers, int shift, int skip_mix, int64_t ntiles, int lockstep)
{
    extern __shared__ int lds[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * nwaves + wave;
    constexpr int kSliceCols = Op::kElems;            // columns in one 16-byte slice
    constexpr int kTileCols = kWave * kSliceCols * U;

    if (lockstep) {
        // Workgroup-uniform fast path: the whole super-tile of the workgroup lies inside one
        // segment, so its waves share one schedule and walk the rows in lock-step.
        const int64_t g0 = static_cast<int64_t>(blockIdx.x) * nwaves * kTileCols;
        const int64_t g1 = g0 + static_cast<int64_t>(nwaves) * kTileCols;
        int lo = 1, hi = S;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (seg_off[mid] <= g0) lo = mid + 1; else hi = mid;
        }
        const int s = lo - 1;
        const int64_t b = (s == 0) ? 0 : seg_off[s];
        const int64_t e = (s == S - 1) ? P : seg_off[s + 1];
        if (g1 <= P && b <= g0 && e >= g1) {
            const int *sched = lds + n;
            if (wave == 0) build_schedule(lds, n, lane, kWave, peers, s, shift, WaveSync{});
            __syncthreads();
            unsigned mask[U];
#pragma unroll
            for (int u = 0; u < U; ++u) mask[u] = (1u << kSliceCols) - 1u;
            walk<Op, U, D, true, NT, true>(op, sched, n, skip_mix != 0, column_of<Op>(tile * kTileCols, lane, 0, 0), mask);
            return;
        }
    }
    if (tile >= ntiles) return;                 // from here on waves are independent: no block barrier
    int *work = lds + wave * kScheduleWords(n);
    const int *sched = work + n;

    const int64_t c0 = tile * kTileCols;
    const int64_t c1 = (c0 + kTileCols < P) ? c0 + kTileCols : P;
    const int64_t off = column_of<Op>(c0, lane, 0, 0);     // this lane's first column

    // segment that holds column c0: number of interior boundaries <= c0
    int lo = 1, hi = S;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (seg_off[mid] <= c0) lo = mid + 1; else hi = mid;
    }
    for (int s = lo - 1; s < S; ++s) {
        int64_t b = (s == 0) ? 0 : seg_off[s];
        int64_t e = (s == S - 1) ? P : seg_off[s + 1];
        b = b < 0 ? 0 : (b > P ? P : b);
        e = e < 0 ? 0 : (e > P ? P : e);
        if (b >= c1) break;
        if (b < c0) b = c0;
        if (e > c1) e = c1;
        if (b >= e) continue;
        build_schedule(work, n, lane, kWave, peers, s, shift, WaveSync{});
        unsigned mask[U];
        if (b == c0 && e == c0 + kTileCols) {
#pragma unroll
            for (int u = 0; u < U; ++u) mask[u] = (1u << kSliceCols) - 1u;
            walk<Op, U, D, true, NT>(op, sched, n, skip_mix != 0, off, mask);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                mask[u] = 0;
#pragma unroll
                for (int q = 0; q < kSliceCols; ++q) {
                    const int64_t c = column_of<Op>(c0, lane, u, q);
                    if (c >= b && c < e) mask[u] |= 1u << q;
                }
            }
            walk<Op, U, D, false, NT>(op, sched, n, skip_mix != 0, off, mask);
        }
    }
}

// ---------------------------------------------------------------------------------
// Row order of the out-of-place path: a table of 32-bit words in device memory that the
// library owns (no allocation at run time), written by order_kernel and read by gather_kernel
// through a pointer both receive as an argument.
//
// Entry (cluster, k): the k-th row the cluster's workgroups visit, that row's partner in the
// segment of the cluster's first column, and a flag saying that this segment covers every
// column of the cluster (so a whole tile of the cluster needs no segment lookup at all).
//
// The ordinary entry points keep kOrderSlots tables of kOrderEntries words per GPU and entry
// point (g_order).  A slot serves ONE stream at a time: calls on a stream run in stream order,
// so a table is never rewritten while an earlier call still reads it.  A stream keeps its slot
// while it has work in flight; a slot whose stream has drained (or has been destroyed) can be
// taken over by another stream.  Streams that find no free slot run without a table (natural
// row order: same results, slower).
// ---------------------------------------------------------------------------------
constexpr int kOrderSlots = 4;
constexpr int kOrderEntries = 1 << 18;
constexpr int kOrderRowBits = kRowBits;
constexpr unsigned kOrderRowField = (1u << kOrderRowBits) - 1u;
constexpr unsigned kOrderOneSegment = 1u << (2 * kOrderRowBits);
__device__ __align__(256) unsigned g_order[kOrderSlots][kOrderEntries];

// The row that gossiping row `row` averages with in segment s (Algorithm 1: receive_from):
// the fixed shift of the push-sum schedule, or the peer table's entry; an entry outside
// [0, n) means the row itself.
__device__ __forceinline__ int partner_of(const int32_t *__restrict__ peers, int shift, int n, int s, int row)
{
    int peer = row;
    if (shift > 0) peer = row >= shift ? row - shift : row - shift + n;
    else if (peers) peer = peers[static_cast<int64_t>(s) * n + row];
    if (static_cast<unsigned>(peer) >= static_cast<unsigned>(n)) peer = row;
    return peer;
}

// One workgroup per segment: builds the segment's cycle schedule and writes it as the row
// order of every cluster whose first column lies in that segment.
__global__ __launch_bounds__(256) void order_kernel(int n, int64_t P, int S,
                                                    const int64_t *__restrict__ seg_off,
                                                    const int32_t *__restrict__ peers, int shift,
                                                    int64_t cluster_cols, int nclusters,
                                                    unsigned *__restrict__ order)
{
    extern __shared__ int lds[];
    const int *sched = lds + n;
    const int s = blockIdx.x;
    build_schedule(lds, n, static_cast<int>(threadIdx.x), static_cast<int>(blockDim.x), peers, s, shift, BlockSync{});
    int64_t sb = (s == 0) ? 0 : seg_off[s];
    int64_t se = (s == S - 1) ? P : seg_off[s + 1];
    sb = sb < 0 ? 0 : (sb > P ? P : sb);
    se = se < 0 ? 0 : (se > P ? P : se);
    const int64_t c_lo = (sb + cluster_cols - 1) / cluster_cols;
    int64_t c_hi = (se + cluster_cols - 1) / cluster_cols;
    if (c_hi > nclusters) c_hi = nclusters;
    // the table as the schedule was built from it: a table that is not a permutation has become
    // the identity there, but the gather serves it as written, so partners come from the source
    const unsigned un = static_cast<unsigned>(n);
    const unsigned total = static_cast<unsigned>(c_hi > c_lo ? c_hi - c_lo : 0) * un;   // fits: the table does
    for (unsigned idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const unsigned k = idx % un;
        const int64_t c = c_lo + idx / un;
        const int row = sched[k] & kRowMask;
        const int64_t last_col = (c + 1) * cluster_cols < P ? (c + 1) * cluster_cols : P;
        unsigned e = static_cast<unsigned>(row) |
                     (static_cast<unsigned>(partner_of(peers, shift, n, s, row)) << kOrderRowBits);
        if (last_col <= se) e |= kOrderOneSegment;
        order[c * n + k] = e;
    }
}

// ---------------------------------------------------------------------------------
// Out-of-place path: one short-lived workgroup per (gossiping row, column chunk).  It loads
// the row's chunk and its partner's chunk, averages, and stores to the other buffer.  Each
// chunk is fetched twice (once as "own", once as somebody's partner); the block order makes
// the two fetches meet in one XCD's L2, so HBM still sees every element once:
//   * workgroups go to the XCDs round-robin by block id, so block b belongs to XCD b % nxcd;
//   * an XCD works through clusters of CL neighbouring chunks, row after row (CL chunks of one
//     row, then CL chunks of the next).  Rows are taken in the order of the segment's
//     permutation cycles (order_kernel), so the partner chunk a block fetches is the own
//     chunk of the block that follows it: only two row visits have to stay in L2;
//   * the XCDs hold neighbouring clusters at the same time, which keeps the stream of every
//     row dense in DRAM.
// Needs x_out != x_in (and v_out != v_in): a partner's input may be read after its owner
// has stored.  Any table with entries in [0, n) is served, permutation or not.
// ---------------------------------------------------------------------------------
template <class Op, int U, bool NT>
__global__ __launch_bounds__(kWave *kMaxWavesPerBlock) void gather_kernel(
    Op op, int n, int64_t P, int S, const int64_t *__restrict__ seg_off,
    const int32_t *__restrict__ peers, int shift, int skip_mix, unsigned nchunks, unsigned CL,
    unsigned nwaves, int xcd_shift, const unsigned *__restrict__ order)
{
    // grid: x = (chunk within cluster, xcd) with the xcd in the low bits, y = gossiping row,
    // z = cluster.  Blocks are dispatched x-fastest, so an XCD sees, for one cluster, row 0's
    // CL chunks, then row 1's, ... and no integer division is needed to decode the block.
    // Chunk and tile numbers fit 32 bits (checked by the host), so the block is decoded with
    // a handful of scalar instructions, and the two ways out of the grid's padding share one
    // branch: the kernel's arguments are fetched once, ahead of it.
    const int lane = threadIdx.x & (kWave - 1);
    const unsigned wave = uniform(threadIdx.x >> 6);
    const unsigned xcd = blockIdx.x & ((1u << xcd_shift) - 1u);
    const unsigned t = blockIdx.x >> xcd_shift;
    const unsigned cluster = (blockIdx.z << xcd_shift) + xcd;
    const unsigned chunk = cluster * CL + t;
    constexpr int kSliceCols = Op::kElems;
    constexpr int kTileCols = kWave * kSliceCols * U;
    const int64_t c0 = static_cast<int64_t>(chunk * nwaves + wave) * kTileCols;
    if (chunk >= nchunks || c0 >= P) return;
    const int64_t c1 = (c0 + kTileCols < P) ? c0 + kTileCols : P;
    const int64_t off = column_of<Op>(c0, lane, 0, 0);     // this lane's first column
    unsigned full_mask[U];
#pragma unroll
    for (int u = 0; u < U; ++u) full_mask[u] = (1u << kSliceCols) - 1u;

    // `mine` holds (or will hold) this row's data; average it with the partner's and store.
    // Operators with many rows behind a gossiping row (hierarchical groups) reduce their
    // own rows before the partner's are requested, which halves the registers in flight.
    int row = blockIdx.y;
    typename Op::template Raw<U> mine;
    auto mix_and_store = [&](auto full_c, const unsigned (&m)[U], int peer) {
        constexpr bool FULL = decltype(full_c)::value;
        using WorkT = typename Op::template Work<U>;
        constexpr bool kOneAtATime = Op::kRawPerSlice * WorkT::kN >= 16 ||            // 16-byte registers per phase
                                     (WorkT::kRegs == 8 && Op::kRawPerSlice * U >= 6);  // fp64 chains take more
        typename Op::template Work<U> a, out;
        if (skip_mix) {
            op.template finish<U, FULL, NT, true>(row, off, m, mine, a);
            out = a;
        } else {
            typename Op::template Work<U> c;
            if constexpr (kOneAtATime) {
                op.template finish<U, FULL, NT, true>(row, off, m, mine, a);
                op.template issue<U, FULL, false>(peer, off, m, mine);
                op.template finish<U, FULL, NT, false>(peer, off, m, mine, c);
            } else {
                typename Op::template Raw<U> theirs;
                op.template issue<U, FULL, false>(peer, off, m, theirs);
                op.template finish<U, FULL, NT, true>(row, off, m, mine, a);
                op.template finish<U, FULL, NT, false>(peer, off, m, theirs, c);
            }
#pragma unroll
            for (int u = 0; u < Op::template Work<U>::kN; ++u) out.v[u] = average(a.v[u], c.v[u]);
        }
        op.template store<U, FULL, NT>(row, off, m, out);
    };

    // y is the position in the cluster's row order: with the order kernel's table, rows follow
    // the permutation cycles, so this block's partner is the next block's own row (fresh in L2).
    // Fast path, almost every tile: the table entry also names the partner and says that one
    // segment covers the cluster, so a tile that does not hang over the row end starts all its
    // loads after a single scalar load.  Whatever the table holds, no access leaves the
    // matrix: rows are checked against n and the tile against P.
    if (order) {
        const unsigned e = order[cluster * static_cast<unsigned>(n) + blockIdx.y];
        const int r = static_cast<int>(e & kOrderRowField);
        const int q = static_cast<int>((e >> kOrderRowBits) & kOrderRowField);
        if (r < n) row = r;
        if constexpr (LdsStaged<Op>::value) {
            // the whole chunk of this workgroup inside one segment and inside the row: every wavefront
            // of the workgroup takes this branch together (the table entry and the chunk are shared)
            const int64_t chunk_c0 = static_cast<int64_t>(chunk) * nwaves * kTileCols;
            if ((e & kOrderOneSegment) != 0 && r < n && q < n && !skip_mix && U == 1 &&
                nwaves * kWave == blockDim.x && static_cast<size_t>(nwaves) * nwaves * kWave * sizeof(f4) == LdsStaged<Op>::bytes &&
                chunk_c0 + static_cast<int64_t>(nwaves) * kTileCols <= P) {
                extern __shared__ f4 staging[];
                op.template lds_mix<NT>(row, q, chunk_c0, lane, static_cast<int>(wave), staging);
                return;
            }
        }
        if ((e & kOrderOneSegment) != 0 && r < n && q < n && c0 + kTileCols <= P) {
            op.template issue<U, true, false>(row, off, full_mask, mine);
            mix_and_store(std::true_type{}, full_mask, q);
            return;
        }
    }

    // General path: tiles of clusters that a segment boundary or the row end crosses, and every
    // tile when there is no order table.  With up to 63 segments one vector load brings the
    // whole offset table and this row's partner in every segment into lanes 0..S at once (a
    // single memory latency); the segment of c0 is then a ballot + popcount and the table
    // entries are read across lanes.  Longer tables fall back to a scalar binary search.
    // The row's own data does not depend on the segment: a tile that does not hang over the
    // row end puts its loads in flight before the lookup.
    const bool whole = c0 + kTileCols <= P;
    if (whole) op.template issue<U, true, false>(row, off, full_mask, mine);
    const bool in_lanes = S <= 63;
    int64_t lane_off = 0;
    int lane_peer = row;
    int first_seg;
    if (in_lanes) {
        if (lane <= S && S > 1) lane_off = seg_off[lane];
        if (lane < S) lane_peer = partner_of(peers, shift, n, lane, row);
        const bool below = lane >= 1 && lane < S && lane_off <= c0;
        first_seg = __builtin_popcountll(__builtin_amdgcn_ballot_w64(below));
    } else {
        int lo = 1, hi = S;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (seg_off[mid] <= c0) lo = mid + 1; else hi = mid;
        }
        first_seg = lo - 1;
    }
    auto offset_at = [&](int k) -> int64_t {
        if (!in_lanes) return seg_off[k];
        const unsigned lo32 = __builtin_amdgcn_readlane(static_cast<int>(lane_off), k);
        const unsigned hi32 = __builtin_amdgcn_readlane(static_cast<int>(lane_off >> 32), k);
        return static_cast<int64_t>((static_cast<uint64_t>(hi32) << 32) | lo32);
    };
    for (int s = first_seg; s < S; ++s) {
        int64_t sb = (s == 0) ? 0 : offset_at(s);
        int64_t se = (s == S - 1) ? P : offset_at(s + 1);
        sb = sb < 0 ? 0 : (sb > P ? P : sb);
        se = se < 0 ? 0 : (se > P ? P : se);
        if (sb >= c1) break;
        if (sb < c0) sb = c0;
        if (se > c1) se = c1;
        if (sb >= se) continue;
        const int peer = in_lanes ? __builtin_amdgcn_readlane(lane_peer, s) : partner_of(peers, shift, n, s, row);
        if (whole && sb == c0 && se == c0 + kTileCols) {  // one segment covers the whole tile
            mix_and_store(std::true_type{}, full_mask, peer);
            return;
        }
        // boundary tile: per-element predication, once per overlapped segment
        unsigned mask[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            mask[u] = 0;
#pragma unroll
            for (int q = 0; q < kSliceCols; ++q) {
                const int64_t c = column_of<Op>(c0, lane, u, q);
                if (c >= sb && c < se) mask[u] |= 1u << q;
            }
        }
        op.template issue<U, false, false>(row, off, mask, mine);
        mix_and_store(std::false_type{}, mask, peer);
    }
}

}  // namespace

#endif  // CX_KERNELS_HPP
