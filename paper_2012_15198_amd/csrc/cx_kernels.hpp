// Device half of the gossip-mixing library for gfx950 (MI355X): the mixing kernels behind
// cx_gossip_mix / cx_hier_mix / cx_pushsum_mix / cx_sgd_fused_mix / cx_hier_sgd_fused_mix and
// their launch logic.  Internal header: each cx_api_*.hip includes it and defines one entry
// point, so the operators compile in parallel; everything here has internal linkage (each
// translation unit carries its own row-order table).
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
//     whose waves each wander over all rows cannot do (measured: 75 % vs 71 % of peak).
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
//  PushOp / Row16Op) say what loading and storing a "gossiping row" means: the pairwise-tree
//  mean of a group of G rows, the momentum-SGD update applied on the way in (to the row or
//  to a group leader fed with the group's mean gradient), the push-sum de-biasing, or the
//  unpacking and rounding of 16-bit rows (bfloat16, binary16).  Each operator also names its
//  measured launch shapes (kGather, kWalk).
#ifndef CX_KERNELS_HPP
#define CX_KERNELS_HPP
#include "cx_mix.h"

#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <type_traits>

#define CX_SCHED_FN __device__ __forceinline__
#include "cx_schedule.hpp"          // build_schedule: the cycle order of a peer table
static_assert(CX_MAX_ROWS <= (1 << kRowBits), "row ids must fit the schedule's packed fields");

#pragma clang fp contract(off)

extern "C" int cx_get_tuning(int32_t key);

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kMaxWavesPerBlock = 8;

typedef double d4 __attribute__((ext_vector_type(4)));

template <int U>
struct Tile {
    static constexpr int kN = U;
    static constexpr int kRegs = 4;        // 32-bit registers per vector
    f4 v[U];
};

// The same columns held as doubles: the optimizer operators carry their whole chain,
// pairwise average included, in fp64 registers and round once on the way out.
template <int U>
struct WideTile {
    static constexpr int kN = U;
    static constexpr int kRegs = 8;
    d4 v[U];
};

// Algorithm 1's averaging line on one vector of columns, in the precision of the tile.
__device__ __forceinline__ f4 average(const f4 &a, const f4 &b) { return (a + b) * 0.5f; }
__device__ __forceinline__ d4 average(const d4 &a, const d4 &b) { return (a + b) * 0.5; }
__device__ __forceinline__ d4 widen(const f4 &a) { return __builtin_convertvector(a, d4); }   // exact
__device__ __forceinline__ f4 narrow(const d4 &a) { return __builtin_convertvector(a, f4); }  // one rounding, nearest even

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Compile-time loop: f(integral_constant<int, I>) for I in [I0, N).
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Column of element q of slice u in this lane: a lane owns kElems consecutive columns per slice.
template <class Op>
__device__ __forceinline__ int64_t column_of(int64_t c0, int lane, int u, int q)
{
    constexpr int kSliceCols = Op::kElems;
    return c0 + kSliceCols * lane + u * (kWave * kSliceCols) + q;
}

// Orders LDS traffic between the lanes of ONE wavefront (wave-private LDS regions).
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------------------------
// Tile I/O.  `p` points at this lane's first slice of the row (row base + tile start
// + 4*lane); slice u sits 256 floats further.  FULL: whole 16-byte slices.  Otherwise
// bit e of mask[u] says whether element e of slice u belongs to this lane right now.
// ---------------------------------------------------------------------------------
template <int U, bool FULL, bool NT>
__device__ __forceinline__ void tile_load(const float *p, const unsigned (&mask)[U], Tile<U> &t)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (FULL) {
            const f4 *q = reinterpret_cast<const f4 *>(p + u * 256);
            t.v[u] = NT ? __builtin_nontemporal_load(q) : *q;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) t.v[u][e] = ((mask[u] >> e) & 1u) ? p[u * 256 + e] : 0.0f;
        }
    }
}

template <int U, bool FULL, bool NT>
__device__ __forceinline__ void tile_store(float *p, const unsigned (&mask)[U], const Tile<U> &t)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (FULL) {
            f4 *q = reinterpret_cast<f4 *>(p + u * 256);
            if (NT) __builtin_nontemporal_store(t.v[u], q); else *q = t.v[u];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((mask[u] >> e) & 1u) p[u * 256 + e] = t.v[u][e];
        }
    }
}

// ---------------------------------------------------------------------------------
// Row operators: what "load gossiping row r" and "store gossiping row r" mean.
// ---------------------------------------------------------------------------------
// Each operator splits "load gossiping row r" into issue() -- put the row's global loads in
// flight into a Raw slot -- and finish() -- turn the arrived data into the tile that takes
// part in the pairwise average.  kRawPerSlice = 16-byte registers per slice and slot.
// kGather = the operator's default launch shape in the out-of-place kernel, kWalk = in the
// in-place kernel (measured optima on MI355X).
struct GatherShape {
    int U, waves, visit_kb, wgs_per_cu;   // slices per lane, waves per workgroup, KB of one row visit
};                                        // per XCD, resident workgroups per CU (0 = as many as fit)
struct WalkShape {
    int U, D, waves, wgs_per_cu;       // slices per lane, rows in flight, waves per workgroup,
};                                     // resident workgroups per CU (0 = as many as fit)

// Plain gossip (G == 1) and hierarchical mode (a gossiping row = a group of G rows).
// G == 1 is Algorithm 1's averaging line in fp32, as written.  For G > 1 the group sum (rows in
// order, from zero), the division by G and the average between leaders run in fp64 registers and
// the result is rounded ONCE to fp32: the correctly rounded value of the plain definition, whatever
// cancels inside the group -- an fp32 sum of values that cancel cannot promise an error relative to
// the result.  The kernel is bound by HBM bandwidth; the fp64 rate is not what limits it.
template <int G>
struct MeanOp {
    static constexpr int kElems = 4;                       // fp32 columns per 16-byte slice
    template <int U> using Work = std::conditional_t<G == 1, Tile<U>, WideTile<U>>;
    static constexpr int kRawPerSlice = G;
    // out-of-place launch: slices per lane, waves per workgroup, KB of one visit to a gossiping row
    // (all G rows behind it) per XCD -- measured optima on MI355X, on matrices spread over the
    // physical memory (cx_hbm_alloc)
    static constexpr GatherShape kGather =
        G == 1 ? GatherShape{1, 4, 256, 0} : G <= 4 ? GatherShape{1, 8, 512, 0} : GatherShape{1, 8, 768, 0};
    static constexpr int kVisitKbFewRows = G >= 8 ? 256 : kGather.visit_kb;      // see VisitKb
    static constexpr WalkShape kWalk =
        G == 1 ? WalkShape{1, 2, 2, 8} : G == 2 ? WalkShape{2, 4, 2, 2} : G <= 8 ? WalkShape{1, 4, 2, 2} : WalkShape{1, 2, 2, 2};
    template <int U> struct Raw { Tile<U> r[G]; };
    const float *xin;
    float *xout;
    int64_t ld;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void issue(int row, int64_t off, const unsigned (&mask)[U], Raw<U> &raw) const
    {
        const float *p = xin + static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_load<U, FULL, NT>(p + j * ld, mask, raw.r[j]);
    }
    template <int U, bool FULL, bool NT, bool COMMIT = true>
    __device__ __forceinline__ void finish(int row, int64_t off, const unsigned (&mask)[U], const Raw<U> &raw, Work<U> &t) const
    {
        if constexpr (G == 1) {
            t = raw.r[0];
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                d4 sum = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int j = 0; j < G; ++j) sum = sum + widen(raw.r[j].v[u]);
                t.v[u] = sum / static_cast<double>(G);
            }
        }
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Work<U> &t) const
    {
        Tile<U> out;
        if constexpr (G == 1) {
            out = t;
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) out.v[u] = narrow(t.v[u]);
        }
        float *p = xout + static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_store<U, FULL, NT>(p + j * ld, mask, out);
    }
};

// The hierarchical mean staged through LDS, kept for measurement next to the sum in registers (launch
// parameter 10).  A workgroup is G wavefronts and owns G tiles of 256 columns; wavefront j fetches
// row j of its group and of the partner group (G contiguous 1-KB loads each), the rows meet in
// LDS (G x G KB), wavefront w reduces tile w over the G rows in the same order and precision, and
// the result travels back through LDS so that wavefront j stores row j.  Same arithmetic in the
// same order as MeanOp<G>, hence the same bits; five barriers per workgroup.  Chunks that a
// segment boundary or the row end crosses take MeanOp<G>'s register path.
template <int G>
struct MeanLdsOp : MeanOp<G> {
    static constexpr bool kLdsStaged = true;
    static constexpr size_t kLdsBytes = static_cast<size_t>(G) * G * kWave * sizeof(f4);

    template <bool NT>
    __device__ __forceinline__ void lds_mix(int row, int peer, int64_t chunk_c0, int lane, int wave, f4 *lds) const
    {
        const int64_t col = chunk_c0 + 4 * lane;
        const float *own = this->xin + (static_cast<int64_t>(row) * G + wave) * this->ld + col;
        const float *oth = this->xin + (static_cast<int64_t>(peer) * G + wave) * this->ld + col;
        f4 mine[G], theirs[G];
#pragma unroll
        for (int t = 0; t < G; ++t) mine[t] = *reinterpret_cast<const f4 *>(own + t * 256);
#pragma unroll
        for (int t = 0; t < G; ++t) theirs[t] = *reinterpret_cast<const f4 *>(oth + t * 256);
#pragma unroll
        for (int t = 0; t < G; ++t) lds[(wave * G + t) * kWave + lane] = mine[t];        // [row][tile][lane]
        __syncthreads();
        d4 a = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int j = 0; j < G; ++j) a = a + widen(lds[(j * G + wave) * kWave + lane]);
        a = a / static_cast<double>(G);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < G; ++t) lds[(wave * G + t) * kWave + lane] = theirs[t];
        __syncthreads();
        d4 c = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int j = 0; j < G; ++j) c = c + widen(lds[(j * G + wave) * kWave + lane]);
        c = c / static_cast<double>(G);
        __syncthreads();
        lds[wave * kWave + lane] = narrow(average(a, c));                                        // result tile `wave`
        __syncthreads();
        float *dst = this->xout + (static_cast<int64_t>(row) * G + wave) * this->ld + col;
#pragma unroll
        for (int t = 0; t < G; ++t) {
            f4 *q = reinterpret_cast<f4 *>(dst + t * 256);
            const f4 v = lds[t * kWave + lane];
            if (NT) __builtin_nontemporal_store(v, q); else *q = v;
        }
    }
};

// Operators that change between memory order and lane order through LDS say how much each wavefront
// needs and are told where their areas start.
template <class Op, class = void>
struct StageBytes {
    static constexpr int value = 0;
};
template <class Op>
struct StageBytes<Op, std::void_t<decltype(Op::kStageBytes)>> {
    static constexpr int value = Op::kStageBytes;
};
template <class Op>
Op with_stage_base(const Op &op, size_t base)
{
    Op copy = op;
    if constexpr (StageBytes<Op>::value > 0) copy.stage_base = static_cast<int>(base);
    return copy;
}

// Visit length of the out-of-place kernel: the operator's kGather.visit_kb, except that an operator with
// groups behind its rows may name a shorter visit for tables of few gossiping rows.  A pair that closes
// a cycle finds its partner in L2 only if all visits in between are still there: with at most
// kFewRows rows the longest cycle's visits fit one XCD's 4 MB L2 at the short length (measured, 8 leaders:
// L2-miss traffic 1.060 -> 1.019 x algorithmic, +0.8 points); with more rows they cannot fit anyway and
// the long visit's DRAM locality wins (32 leaders: 77.1 % at 768 KB against 76.3 % at 384 KB).
constexpr int kFewRows = 8;
template <class Op, class = void>
struct VisitKb {
    static constexpr int of(int) { return Op::kGather.visit_kb; }
};
template <class Op>
struct VisitKb<Op, std::void_t<decltype(Op::kVisitKbFewRows)>> {
    static constexpr int of(int n) { return n <= kFewRows ? Op::kVisitKbFewRows : Op::kGather.visit_kb; }
};

template <class Op, class = void>
struct LdsStaged {
    static constexpr bool value = false;
    static constexpr size_t bytes = 0;
};
template <class Op>
struct LdsStaged<Op, std::void_t<decltype(Op::kLdsStaged)>> {
    static constexpr bool value = Op::kLdsStaged;
    static constexpr size_t bytes = Op::kLdsBytes;
};

// Momentum-SGD applied as the row arrives; the mix then averages the updated rows.
// The whole chain runs in fp64 registers, in the order the formula is written:
//     t = g + wd*x ;  v' = mu*v + t ;  h = x - lr*v' ;  x' = (h_i + h_peer) * 0.5
// (every input widened exactly, the hyper-parameters as the doubles of their fp32 values, no
// fused multiply-add), and v' and x' are each rounded ONCE to fp32 when they are stored.  An
// fp32 chain would round six times against intermediates larger than the result and misses a
// 1e-6 relative bound once the momentum has grown; the kernel is bound by HBM bandwidth, so
// the fp64 rate is not what limits it.

struct SgdStep {
    double lr, mu, wd;
    // one optimizer step on a vector of columns: returns h, leaves v' in `v`
    __device__ __forceinline__ d4 apply(const d4 &x, d4 &v, const d4 &g) const
    {
        const d4 decayed = g + x * wd;
        v = v * mu + decayed;
        return x - v * lr;
    }
};

struct FusedOp {
    static constexpr int kElems = 4;                       // fp32 columns per 16-byte slice
    template <int U> using Work = WideTile<U>;             // the updated row, in fp64
    static constexpr int kRawPerSlice = 3;
    static constexpr GatherShape kGather{1, 8, 128, 3};
    static constexpr WalkShape kWalk{2, 2, 4, 2};
    static constexpr int kMaxU = 2;                        // fp64 rows: two slices per lane fill the registers
    template <int U> struct Raw { Tile<U> x, v, g; };
    const float *xin;
    float *xout;
    const float *vin;
    float *vout;
    const float *g;
    int64_t ld;
    SgdStep sgd;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void issue(int row, int64_t off, const unsigned (&mask)[U], Raw<U> &raw) const
    {
        const int64_t o = static_cast<int64_t>(row) * ld + off;
        tile_load<U, FULL, NT>(xin + o, mask, raw.x);
        tile_load<U, FULL, NT>(vin + o, mask, raw.v);
        tile_load<U, FULL, NT>(g + o, mask, raw.g);
    }
    // COMMIT: also write v' of this row (false when the row is only recomputed as a partner)
    template <int U, bool FULL, bool NT, bool COMMIT = true>
    __device__ __forceinline__ void finish(int row, int64_t off, const unsigned (&mask)[U], const Raw<U> &raw, Work<U> &t) const
    {
        Tile<U> v32;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            d4 v = widen(raw.v.v[u]);
            t.v[u] = sgd.apply(widen(raw.x.v[u]), v, widen(raw.g.v[u]));
            v32.v[u] = narrow(v);
        }
        if constexpr (COMMIT) tile_store<U, FULL, NT>(vout + static_cast<int64_t>(row) * ld + off, mask, v32);
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Work<U> &t) const
    {
        Tile<U> out;
#pragma unroll
        for (int u = 0; u < U; ++u) out.v[u] = narrow(t.v[u]);
        tile_store<U, FULL, NT>(xout + static_cast<int64_t>(row) * ld + off, mask, out);
    }
};

// Hierarchical step with gradients: a gossiping row is a group; loading it reduces the G
// gradient rows, applies the momentum-SGD step to the LEADER's parameters and momentum, and
// hands the updated leader parameters to the mix; storing broadcasts.  fp64 registers as in
// FusedOp: the gradients are summed in row order starting from zero and divided by G.
template <int G>
struct HierFusedOp {
    static constexpr int kElems = 4;                       // fp32 columns per 16-byte slice
    template <int U> using Work = WideTile<U>;             // the updated leader row, in fp64
    static constexpr int kRawPerSlice = G + 2;
    // out-of-place launch: slices, waves, group visit KB per XCD
    static constexpr GatherShape kGather =
        G == 1 ? GatherShape{1, 8, 256, 0} : G <= 4 ? GatherShape{1, 8, 512, 0} : GatherShape{1, 8, 768, 0};
    static constexpr int kVisitKbFewRows = G >= 8 ? 256 : kGather.visit_kb;      // see VisitKb
    static constexpr WalkShape kWalk = G <= 4 ? WalkShape{1, 4, 2, 2} : WalkShape{1, 2, 2, 2};
    static constexpr int kMaxU = G <= 2 ? 2 : 1;
    template <int U> struct Raw { Tile<U> g[G], x, v; };
    const float *xin;
    float *xout;
    const float *vin;     // [L][ld]
    float *vout;          // [L][ld]
    const float *g;       // [W][ld]
    int64_t ld;
    SgdStep sgd;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void issue(int row, int64_t off, const unsigned (&mask)[U], Raw<U> &raw) const
    {
        const int64_t lead = static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_load<U, FULL, NT>(g + lead + j * ld, mask, raw.g[j]);
        tile_load<U, FULL, NT>(xin + lead, mask, raw.x);
        tile_load<U, FULL, NT>(vin + static_cast<int64_t>(row) * ld + off, mask, raw.v);
    }
    template <int U, bool FULL, bool NT, bool COMMIT = true>
    __device__ __forceinline__ void finish(int row, int64_t off, const unsigned (&mask)[U], const Raw<U> &raw, Work<U> &t) const
    {
        Tile<U> v32;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            d4 gsum = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int j = 0; j < G; ++j) gsum = gsum + widen(raw.g[j].v[u]);
            const d4 gbar = gsum / static_cast<double>(G);
            d4 v = widen(raw.v.v[u]);
            t.v[u] = sgd.apply(widen(raw.x.v[u]), v, gbar);
            v32.v[u] = narrow(v);
        }
        if constexpr (COMMIT) tile_store<U, FULL, NT>(vout + static_cast<int64_t>(row) * ld + off, mask, v32);
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Work<U> &t) const
    {
        Tile<U> out;
#pragma unroll
        for (int u = 0; u < U; ++u) out.v[u] = narrow(t.v[u]);
        float *p = xout + static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_store<U, FULL, NT>(p + j * ld, mask, out);
    }
};

// ---------------------------------------------------------------------------------
// 16-bit rows (8 columns per 16-byte slice), bfloat16 or IEEE binary16, averaged in fp32:
//     out = round_to_nearest_even_16((float(a) + float(b)) * 0.5f)
// ---------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(unsigned h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ float f16_bits_to_float(unsigned h)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));   // exact, subnormals kept
}

template <int U, bool FULL, bool NT>
__device__ __forceinline__ void tile_load16(const uint16_t *p, const unsigned (&mask)[U], Tile<U> &raw)
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (FULL) {
            const f4 *q = reinterpret_cast<const f4 *>(p + u * (kWave * 8));
            raw.v[u] = NT ? __builtin_nontemporal_load(q) : *q;
        } else {
            u4 w = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if ((mask[u] >> e) & 1u) w[e >> 1] |= static_cast<unsigned>(p[u * (kWave * 8) + e]) << (16 * (e & 1));
            raw.v[u] = __builtin_bit_cast(f4, w);
        }
    }
}

template <int U, bool FULL, bool NT>
__device__ __forceinline__ void tile_store16(uint16_t *p, const unsigned (&mask)[U], const Tile<U> &raw)
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (FULL) {
            f4 *q = reinterpret_cast<f4 *>(p + u * (kWave * 8));
            if (NT) __builtin_nontemporal_store(raw.v[u], q); else *q = raw.v[u];
        } else {
            const u4 w = __builtin_bit_cast(u4, raw.v[u]);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if ((mask[u] >> e) & 1u)
                    p[u * (kWave * 8) + e] = static_cast<uint16_t>(w[e >> 1] >> (16 * (e & 1)));
        }
    }
}

// double -> fp32 with rounding to odd: the discarded bits survive as a sticky last bit, so that the
// hardware's round-to-nearest-even conversion to 16 bits that follows is ONE rounding of the double.
__device__ __forceinline__ float to_f32_round_to_odd(double d)
{
    const float f = static_cast<float>(d);                 // nearest even
    const double back = static_cast<double>(f);
    unsigned bits = __float_as_uint(f);
    if (back != d && d == d) {                             // inexact (and not a NaN)
        if (__builtin_fabs(back) > __builtin_fabs(d)) bits -= 1;   // step back to the truncated value
        bits |= 1u;                                        // and remember that something was cut off
    }
    return __uint_as_float(bits);
}

// half hh (words 2*hh, 2*hh+1) of a packed 16-bit slice, widened exactly to doubles
template <bool IEEE_HALF>
__device__ __forceinline__ d4 widen16_half(const f4 &packed, int hh)
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    const u4 w = __builtin_bit_cast(u4, packed);
    d4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const unsigned pair = hh == 0 ? w[e >> 1] : w[2 + (e >> 1)];
        const unsigned h = (pair >> (16 * (e & 1))) & 0xffffu;
        out[e] = static_cast<double>(IEEE_HALF ? f16_bits_to_float(h) : bf16_bits_to_float(h));
    }
    return out;
}

// eight doubles -> one packed 16-bit slice, each rounded once (nearest even)
template <bool IEEE_HALF>
__device__ __forceinline__ f4 narrow16_once(const d4 &lo, const d4 &hi)
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    u4 w;
#pragma unroll
    for (int pair = 0; pair < 4; ++pair) {
        const d4 &src = pair < 2 ? lo : hi;
        const f2 two = {to_f32_round_to_odd(src[2 * (pair & 1)]), to_f32_round_to_odd(src[2 * (pair & 1) + 1])};
        if constexpr (IEEE_HALF) w[pair] = __builtin_bit_cast(unsigned, __builtin_convertvector(two, h2));
        else w[pair] = __builtin_bit_cast(unsigned, __builtin_convertvector(two, b2));
    }
    return __builtin_bit_cast(f4, w);
}

// G == 1: plain gossip on 16-bit rows: widen, add and halve in fp32, round once.  G > 1: hierarchical
// mode, a gossiping row = a group of G rows whose widened values are summed (rows in order), divided
// by G and averaged between leaders in fp64 registers, as in MeanOp<G>, and rounded ONCE to the 16-bit
// format on the way out.
template <bool IEEE_HALF, int G = 1>
struct Row16Op {
    static constexpr int kElems = 8;                       // 16-bit columns per 16-byte slice
    template <int U> using Work = std::conditional_t<G == 1, Tile<2 * U>, WideTile<2 * U>>;   // 8 values per slice
    static constexpr int kRawPerSlice = G;
    static constexpr GatherShape kGather =
        G == 1 ? GatherShape{1, 8, 96, 0} : G <= 4 ? GatherShape{1, 8, 256, 0} : GatherShape{1, 8, 384, 0};
    static constexpr WalkShape kWalk = G == 1 ? WalkShape{1, 2, 8, 0} : WalkShape{1, 2, 2, 2};
    static constexpr int kMaxU = G == 1 ? 4 : 1;           // grouped: one slice per lane fills the registers
    template <int U> struct Raw { Tile<U> r[G]; };         // packed 16-bit pairs, as loaded
    const uint16_t *xin;
    uint16_t *xout;
    int64_t ld;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void issue(int row, int64_t off, const unsigned (&mask)[U], Raw<U> &raw) const
    {
        const uint16_t *p = xin + static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_load16<U, FULL, NT>(p + j * ld, mask, raw.r[j]);
    }
    template <int U>
    static __device__ __forceinline__ void widen(const Tile<U> &packed, Tile<2 * U> &t)
    {
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u4 w = __builtin_bit_cast(u4, packed.v[u]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned h = (w[e >> 1] >> (16 * (e & 1))) & 0xffffu;
                t.v[2 * u + (e >> 2)][e & 3] = IEEE_HALF ? f16_bits_to_float(h) : bf16_bits_to_float(h);
            }
        }
    }
    template <int U, bool FULL, bool NT, bool COMMIT = true>
    __device__ __forceinline__ void finish(int row, int64_t off, const unsigned (&mask)[U], const Raw<U> &raw, Work<U> &t) const
    {
        if constexpr (G == 1) {
            widen<U>(raw.r[0], t);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    d4 sum = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                    for (int j = 0; j < G; ++j) sum = sum + widen16_half<IEEE_HALF>(raw.r[j].v[u], hh);
                    t.v[2 * u + hh] = sum / static_cast<double>(G);
                }
        }
    }
    // fp32 values of a tile -> packed 16-bit pairs, round-to-nearest-even in hardware
    template <int U>
    static __device__ __forceinline__ void pack(const Tile<2 * U> &t, Tile<U> &packed)
    {
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        typedef float f2 __attribute__((ext_vector_type(2)));
        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            u4 w;
#pragma unroll
            for (int pair = 0; pair < 4; ++pair) {
                const f2 two = {t.v[2 * u + (pair >> 1)][2 * (pair & 1)], t.v[2 * u + (pair >> 1)][2 * (pair & 1) + 1]};
                if constexpr (IEEE_HALF) w[pair] = __builtin_bit_cast(unsigned, __builtin_convertvector(two, h2));
                else w[pair] = __builtin_bit_cast(unsigned, __builtin_convertvector(two, b2));
            }
            packed.v[u] = __builtin_bit_cast(f4, w);
        }
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Work<U> &t) const
    {
        Tile<U> packed;
        if constexpr (G == 1) {
            pack<U>(t, packed);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) packed.v[u] = narrow16_once<IEEE_HALF>(t.v[2 * u], t.v[2 * u + 1]);
        }
        uint16_t *p = xout + static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_store16<U, FULL, NT>(p + j * ld, mask, packed);
    }
};

using Bf16Op = Row16Op<false>;
using Fp16Op = Row16Op<true>;

// The SGP-style push-sum comparison on 16-bit rows (PushOp below is the fp32-row one): the rows are widened
// exactly, averaged in fp32 like Row16Op's, and the de-biased copy z = average / w' is the quotient of the
// UNROUNDED fp32 average, narrowed once like x'.  The weights stay fp32.
template <bool IEEE_HALF>
struct Push16Op : Row16Op<IEEE_HALF, 1> {
    using Base = Row16Op<IEEE_HALF, 1>;
    static constexpr GatherShape kGather{2, 4, 192, 0};    // measured on C4: one slice per lane 52 %, two 76 %
    static constexpr WalkShape kWalk{1, 2, 8, 0};
    uint16_t *zout;       // may be null
    const float *win;
    int n, hop;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Tile<2 * U> &t) const
    {
        Base::template store<U, FULL, NT>(row, off, mask, t);
        if (zout) {
            const int from = row >= hop ? row - hop : row - hop + n;
            const float wn = (win[row] + win[from]) * 0.5f;
            Tile<2 * U> z;
#pragma unroll
            for (int u = 0; u < 2 * U; ++u) z.v[u] = t.v[u] / wn;
            Tile<U> packed;
            Base::template pack<U>(z, packed);
            tile_store16<U, FULL, NT>(zout + static_cast<int64_t>(row) * this->ld + off, mask, packed);
        }
    }
};

// ---------------------------------------------------------------------------------
// The optimizer operators on 16-bit rows: parameters and gradients are 16-bit (8 columns per
// 16-byte slice), the momentum stays fp32 (the same 8 columns are two 16-byte registers).
// Everything is widened exactly, the chain runs in fp64 as in FusedOp, v' is rounded once to
// fp32 and x' ONCE to the 16-bit format: the double is first narrowed to fp32 with rounding to
// odd (the discarded bits survive as a sticky last bit), which makes the hardware's
// round-to-nearest-even conversion to 16 bits equal to one rounding of the double itself.
// ---------------------------------------------------------------------------------
// fp32 companion rows of 16-bit rows.  A lane owns 8 consecutive columns of a 512-column slice:
// one 16-byte register of a 16-bit row, but TWO of an fp32 row, 32 bytes apart from the
// neighbouring lane's -- read like that, every 16-byte access of a wavefront leaves half of each
// cache line to the other access, and the fused step runs 7 % slower.  So whole slices of the
// fp32 rows move between memory and registers in MEMORY order (register hh of lane l = columns
// 256*hh + 4*l .. +3: each access of the wavefront one contiguous KB) and change to the lane's own
// columns through 2 KB of LDS per wavefront (stage_to_own / stage_from_own).  Boundary tiles,
// handled element by element, address the lane's own columns directly.
template <int U, bool FULL, bool NT>
__device__ __forceinline__ void tile_load8(const float *p, const unsigned (&mask)[U], Tile<2 * U> &t)
{
    // p = row base + this lane's first column (tile start + 8 * lane)
    const int lane = static_cast<int>(threadIdx.x & (kWave - 1));
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            if constexpr (FULL) {
                const f4 *q4 = reinterpret_cast<const f4 *>(p - 4 * lane + u * (kWave * 8) + 256 * hh);   // memory order
                t.v[2 * u + hh] = NT ? __builtin_nontemporal_load(q4) : *q4;
            } else {
                const float *q = p + u * (kWave * 8) + 4 * hh;                                           // own columns
#pragma unroll
                for (int e = 0; e < 4; ++e) t.v[2 * u + hh][e] = ((mask[u] >> (4 * hh + e)) & 1u) ? q[e] : 0.0f;
            }
        }
}

template <int U, bool FULL, bool NT>
__device__ __forceinline__ void tile_store8(float *p, const unsigned (&mask)[U], const Tile<2 * U> &t)
{
    const int lane = static_cast<int>(threadIdx.x & (kWave - 1));
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            if constexpr (FULL) {
                f4 *q4 = reinterpret_cast<f4 *>(p - 4 * lane + u * (kWave * 8) + 256 * hh);
                if (NT) __builtin_nontemporal_store(t.v[2 * u + hh], q4); else *q4 = t.v[2 * u + hh];
            } else {
                float *q = p + u * (kWave * 8) + 4 * hh;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((mask[u] >> (4 * hh + e)) & 1u) q[e] = t.v[2 * u + hh][e];
            }
        }
}

// This wavefront's 2 KB of the workgroup's dynamic LDS, `stage_base` bytes in (the schedules of
// the in-place kernel come first).
constexpr int kStageBytesPerWave = 2048;
__device__ __forceinline__ f4 *stage_of_this_wave(int stage_base)
{
    extern __shared__ f4 cx_dynamic_lds[];
    return cx_dynamic_lds + (stage_base >> 4) + (threadIdx.x >> 6) * (kStageBytesPerWave / 16);
}

// registers in memory order -> the lane's own columns (register 0 = columns 8l..8l+3, 1 = 8l+4..8l+7)
template <int U>
__device__ __forceinline__ void stage_to_own(f4 *stage, Tile<2 * U> &t)
{
    const int lane = static_cast<int>(threadIdx.x & (kWave - 1));
#pragma unroll
    for (int u = 0; u < U; ++u) {
        stage[lane] = t.v[2 * u];
        stage[kWave + lane] = t.v[2 * u + 1];
        wave_sync();
        t.v[2 * u] = stage[2 * lane];
        t.v[2 * u + 1] = stage[2 * lane + 1];
        wave_sync();
    }
}

// and back, for the store
template <int U>
__device__ __forceinline__ void stage_from_own(f4 *stage, Tile<2 * U> &t)
{
    const int lane = static_cast<int>(threadIdx.x & (kWave - 1));
#pragma unroll
    for (int u = 0; u < U; ++u) {
        stage[2 * lane] = t.v[2 * u];
        stage[2 * lane + 1] = t.v[2 * u + 1];
        wave_sync();
        t.v[2 * u] = stage[lane];
        t.v[2 * u + 1] = stage[kWave + lane];
        wave_sync();
    }
}

// cx_sgd_fused_mix_bf16 / _f16: FusedOp with 16-bit x and g rows and fp32 momentum rows.
template <bool IEEE_HALF>
struct Fused16Op {
    static constexpr int kElems = 8;                       // 16-bit columns per 16-byte slice
    template <int U> using Work = WideTile<2 * U>;         // the updated row, 8 doubles per slice
    static constexpr int kRawPerSlice = 4;                 // x, g: one register each; v: two
    static constexpr GatherShape kGather{1, 4, 96, 0};
    static constexpr WalkShape kWalk{1, 2, 4, 2};
    static constexpr int kMaxU = 1;
    static constexpr int kStageBytes = kStageBytesPerWave; // LDS per wavefront (see tile_load8)
    template <int U> struct Raw { Tile<U> x, g; Tile<2 * U> v; };
    const uint16_t *xin;
    uint16_t *xout;
    const float *vin;
    float *vout;
    const uint16_t *g;
    int64_t ld;
    SgdStep sgd;
    int stage_base = 0;   // bytes into the dynamic LDS where the wavefronts' staging areas start (set at launch)

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void issue(int row, int64_t off, const unsigned (&mask)[U], Raw<U> &raw) const
    {
        const int64_t o = static_cast<int64_t>(row) * ld + off;
        tile_load16<U, FULL, NT>(xin + o, mask, raw.x);
        tile_load8<U, FULL, NT>(vin + o, mask, raw.v);
        tile_load16<U, FULL, NT>(g + o, mask, raw.g);
    }
    template <int U, bool FULL, bool NT, bool COMMIT = true>
    __device__ __forceinline__ void finish(int row, int64_t off, const unsigned (&mask)[U], const Raw<U> &raw, Work<U> &t) const
    {
        Tile<2 * U> v32 = raw.v;
        if constexpr (FULL) stage_to_own<U>(stage_of_this_wave(stage_base), v32);     // memory order -> own columns
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                d4 v = widen(v32.v[2 * u + hh]);
                t.v[2 * u + hh] = sgd.apply(widen16_half<IEEE_HALF>(raw.x.v[u], hh), v, widen16_half<IEEE_HALF>(raw.g.v[u], hh));
                v32.v[2 * u + hh] = narrow(v);
            }
        if constexpr (COMMIT) {
            if constexpr (FULL) stage_from_own<U>(stage_of_this_wave(stage_base), v32);
            tile_store8<U, FULL, NT>(vout + static_cast<int64_t>(row) * ld + off, mask, v32);
        }
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Work<U> &t) const
    {
        Tile<U> packed;
#pragma unroll
        for (int u = 0; u < U; ++u) packed.v[u] = narrow16_once<IEEE_HALF>(t.v[2 * u], t.v[2 * u + 1]);
        tile_store16<U, FULL, NT>(xout + static_cast<int64_t>(row) * ld + off, mask, packed);
    }
};

// cx_hier_sgd_fused_mix_bf16 / _f16: HierFusedOp with 16-bit x and g rows, fp32 leader momentum.
template <bool IEEE_HALF, int G>
struct HierFused16Op {
    static constexpr int kElems = 8;
    template <int U> using Work = WideTile<2 * U>;
    static constexpr int kRawPerSlice = G + 3;             // G gradient rows, x, and two registers of v
    static constexpr GatherShape kGather =
        G == 1 ? GatherShape{1, 8, 192, 0} : G <= 4 ? GatherShape{1, 8, 256, 0} : GatherShape{1, 8, 384, 0};
    static constexpr WalkShape kWalk{1, 2, 2, 2};
    static constexpr int kMaxU = 1;
    static constexpr int kStageBytes = kStageBytesPerWave;
    template <int U> struct Raw { Tile<U> g[G], x; Tile<2 * U> v; };
    const uint16_t *xin;
    uint16_t *xout;
    const float *vin;     // [L][ld]
    float *vout;          // [L][ld]
    const uint16_t *g;    // [W][ld]
    int64_t ld;
    SgdStep sgd;
    int stage_base = 0;   // as in Fused16Op

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void issue(int row, int64_t off, const unsigned (&mask)[U], Raw<U> &raw) const
    {
        const int64_t lead = static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_load16<U, FULL, NT>(g + lead + j * ld, mask, raw.g[j]);
        tile_load16<U, FULL, NT>(xin + lead, mask, raw.x);
        tile_load8<U, FULL, NT>(vin + static_cast<int64_t>(row) * ld + off, mask, raw.v);
    }
    template <int U, bool FULL, bool NT, bool COMMIT = true>
    __device__ __forceinline__ void finish(int row, int64_t off, const unsigned (&mask)[U], const Raw<U> &raw, Work<U> &t) const
    {
        Tile<2 * U> v32 = raw.v;
        if constexpr (FULL) stage_to_own<U>(stage_of_this_wave(stage_base), v32);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                d4 gsum = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int j = 0; j < G; ++j) gsum = gsum + widen16_half<IEEE_HALF>(raw.g[j].v[u], hh);
                const d4 gbar = gsum / static_cast<double>(G);
                d4 v = widen(v32.v[2 * u + hh]);
                t.v[2 * u + hh] = sgd.apply(widen16_half<IEEE_HALF>(raw.x.v[u], hh), v, gbar);
                v32.v[2 * u + hh] = narrow(v);
            }
        if constexpr (COMMIT) {
            if constexpr (FULL) stage_from_own<U>(stage_of_this_wave(stage_base), v32);
            tile_store8<U, FULL, NT>(vout + static_cast<int64_t>(row) * ld + off, mask, v32);
        }
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Work<U> &t) const
    {
        Tile<U> packed;
#pragma unroll
        for (int u = 0; u < U; ++u) packed.v[u] = narrow16_once<IEEE_HALF>(t.v[2 * u], t.v[2 * u + 1]);
        uint16_t *p = xout + static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_store16<U, FULL, NT>(p + j * ld, mask, packed);
    }
};

// Push-sum: plain rows, optional de-biased copy z = x' / w'.
struct PushOp {
    static constexpr int kElems = 4;                       // fp32 columns per 16-byte slice
    template <int U> using Work = Tile<U>;                 // fp32 values a lane works on
    static constexpr int kRawPerSlice = 1;
    static constexpr GatherShape kGather{2, 4, 512, 0};
    static constexpr WalkShape kWalk{2, 2, 8, 2};
    template <int U> struct Raw { Tile<U> x; };
    const float *xin;
    float *xout;
    float *zout;          // may be null
    const float *win;
    int64_t ld;
    int n, hop;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void issue(int row, int64_t off, const unsigned (&mask)[U], Raw<U> &raw) const
    {
        tile_load<U, FULL, NT>(xin + static_cast<int64_t>(row) * ld + off, mask, raw.x);
    }
    template <int U, bool FULL, bool NT, bool COMMIT = true>
    __device__ __forceinline__ void finish(int row, int64_t off, const unsigned (&mask)[U], const Raw<U> &raw, Tile<U> &t) const
    {
        t = raw.x;
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Tile<U> &t) const
    {
        const int64_t o = static_cast<int64_t>(row) * ld + off;
        tile_store<U, FULL, NT>(xout + o, mask, t);
        if (zout) {
            const int from = row >= hop ? row - hop : row - hop + n;
            const float wn = (win[row] + win[from]) * 0.5f;
            Tile<U> z;
#pragma unroll
            for (int u = 0; u < U; ++u) z.v[u] = t.v[u] / wn;
            tile_store<U, FULL, NT>(zout + o, mask, z);
        }
    }
};

// w_out[i] = (w_in[i] + w_in[(i - hop) mod n]) * 0.5f  (push-sum weights, n <= CX_MAX_ROWS): the de-biasing in
// PushOp / Push16Op reads w_in, so the new weights are written by their own tiny launch
[[maybe_unused]] __global__ void pushsum_weight_kernel(const float *__restrict__ w_in, float *__restrict__ w_out,
                                                       int n, int hop)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const int from = i >= hop ? i - hop : i - hop + n;
        w_out[i] = (w_in[i] + w_in[from]) * 0.5f;
    }
}

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

#endif  // CX_KERNELS_HPP
