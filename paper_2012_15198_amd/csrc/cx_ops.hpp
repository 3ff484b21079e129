// Row operators on fp32 rows (internal header): the plain and the hierarchical mean (Section 3.3), the
// momentum-SGD step fused in front of the mix (Section 3.1), its gradient-reducing hierarchical form, and the
// push-sum comparison (Sections 2.1, 3); with the traits through which the kernels ask an operator for its
// launch shapes and LDS needs.
#ifndef CX_OPS_HPP
#define CX_OPS_HPP
#include "cx_tile.hpp"

#pragma clang fp contract(off)

namespace {

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
    static constexpr WalkShape kWalk{2, 2, 8, 2};
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

}  // namespace

#endif  // CX_OPS_HPP
