// Device half of the gossip-mixing library for gfx950 (MI355X): the column-owner
// mixing kernels behind cx_gossip_mix / cx_hier_mix / cx_pushsum_mix /
// cx_sgd_fused_mix, and their C-ABI launchers.
//
// Design (one kernel, one HBM pass per round):
//  * Mixing is independent per column, so one lane OWNS a 16-byte column slice
//    (4 consecutive fp32 columns) -- U slices per lane, 1 KB contiguous per wave per
//    row access -- and visits every row of that slice.  A wavefront owns a tile of
//    256*U columns; wavefronts never talk to each other (no barriers, no atomics on
//    global memory).
//  * The per-segment peer table is a permutation, so the rows of a column split into
//    cycles i -> peers[i] -> peers[peers[i]] ...  Walking a cycle, the lane holds the
//    current and the next row's slice in registers, writes (cur + next) * 0.5f to the
//    current row and moves on; the cycle's first slice is kept for its last row.
//    Every element is therefore read once and written once (8 B per worker-parameter),
//    and the update may run in place: a row is overwritten only after its two readers
//    (itself and the one row that receives from it) have it in registers.
//  * The cycle order of a segment is built per wavefront in LDS (wave-private, a few
//    hundred bytes) from the device-resident peer table; a table that is not a
//    permutation is replaced by the identity, so no row index can leave [0, n).
//  * Tiles that lie wholly inside one segment take the 16-byte vector path; the at most
//    S+1 tiles that straddle a segment boundary or the ragged end of the row take the
//    same walk once per overlapped segment with per-element predication.
//  * Hierarchical mode loads the G rows of a group and reduces them in registers with a
//    fixed pairwise tree before the walk over group leaders; the result is stored to all
//    G rows.  The fused mode applies the momentum-SGD update as each row is loaded.
//    Push-sum is the walk over the shift permutation, plus the scalar weights.
#include "cx_mix.h"

#include <hip/hip_runtime.h>

#include <cstdint>

#pragma clang fp contract(off)

extern "C" int cx_get_tuning(int32_t key);

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kLastBit = 1 << 30;          // schedule entry flag: last row of its cycle
constexpr int kRowMask = kLastBit - 1;
constexpr int kMaxWavesPerBlock = 8;

template <int U>
struct Tile {
    f4 v[U];
};

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

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

// Pairwise tree over N tiles: split at the largest power of two below N.
template <int N, int U>
__device__ __forceinline__ Tile<U> tree_sum(const Tile<U> *r)
{
    if constexpr (N == 1) {
        return r[0];
    } else {
        constexpr int H = (N > 16) ? 16 : (N > 8) ? 8 : (N > 4) ? 4 : (N > 2) ? 2 : 1;
        static_assert(N <= 32, "group size");
        const Tile<U> a = tree_sum<H, U>(r);
        const Tile<U> b = tree_sum<N - H, U>(r + H);
        Tile<U> s;
#pragma unroll
        for (int u = 0; u < U; ++u) s.v[u] = a.v[u] + b.v[u];
        return s;
    }
}

// ---------------------------------------------------------------------------------
// Row operators: what "load gossiping row r" and "store gossiping row r" mean.
// ---------------------------------------------------------------------------------
// Plain gossip (G == 1) and hierarchical mode (a gossiping row = a group of G rows).
template <int G>
struct MeanOp {
    const float *xin;
    float *xout;
    int64_t ld;
    float inv_g;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void load(int row, int64_t off, const unsigned (&mask)[U], Tile<U> &t) const
    {
        const float *p = xin + static_cast<int64_t>(row) * G * ld + off;
        if constexpr (G == 1) {
            tile_load<U, FULL, NT>(p, mask, t);
        } else {
            Tile<U> r[G];
#pragma unroll
            for (int j = 0; j < G; ++j) tile_load<U, FULL, NT>(p + j * ld, mask, r[j]);
            t = tree_sum<G, U>(r);
#pragma unroll
            for (int u = 0; u < U; ++u) t.v[u] = t.v[u] * inv_g;
        }
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Tile<U> &t) const
    {
        float *p = xout + static_cast<int64_t>(row) * G * ld + off;
#pragma unroll
        for (int j = 0; j < G; ++j) tile_store<U, FULL, NT>(p + j * ld, mask, t);
    }
};

// Momentum-SGD applied while the row is loaded; the walk then mixes the updated rows.
struct FusedOp {
    const float *xin;
    float *xout;
    const float *vin;
    float *vout;
    const float *g;
    int64_t ld;
    float lr, mu, wd;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void load(int row, int64_t off, const unsigned (&mask)[U], Tile<U> &t) const
    {
        const int64_t o = static_cast<int64_t>(row) * ld + off;
        Tile<U> x, v, gr;
        tile_load<U, FULL, NT>(xin + o, mask, x);
        tile_load<U, FULL, NT>(vin + o, mask, v);
        tile_load<U, FULL, NT>(g + o, mask, gr);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const f4 decayed = gr.v[u] + x.v[u] * wd;     // g' = g + wd*x
            v.v[u] = v.v[u] * mu + decayed;               // v' = mu*v + g'
            t.v[u] = x.v[u] - v.v[u] * lr;                // x_half = x - lr*v'
        }
        tile_store<U, FULL, NT>(vout + o, mask, v);
    }
    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void store(int row, int64_t off, const unsigned (&mask)[U], const Tile<U> &t) const
    {
        tile_store<U, FULL, NT>(xout + static_cast<int64_t>(row) * ld + off, mask, t);
    }
};

// Push-sum: plain rows, optional de-biased copy z = x' / w'.
struct PushOp {
    const float *xin;
    float *xout;
    float *zout;          // may be null
    const float *win;
    int64_t ld;
    int n, hop;

    template <int U, bool FULL, bool NT>
    __device__ __forceinline__ void load(int row, int64_t off, const unsigned (&mask)[U], Tile<U> &t) const
    {
        tile_load<U, FULL, NT>(xin + static_cast<int64_t>(row) * ld + off, mask, t);
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

// ---------------------------------------------------------------------------------
// Cycle schedule of one segment, built by one wavefront in its private LDS region.
//   tab[0..n)  : the table, then scratch for the walk
//   sched[0..n): rows in cycle order; kLastBit marks the last row of a cycle
// Source of the table: shift > 0 -> row i receives from (i - shift) mod n;
// peers == null -> identity; else peers[seg*n + i].
// ---------------------------------------------------------------------------------
__device__ __forceinline__ void build_schedule(int *tab, int *sched, int n, int lane,
                                               const int32_t *peers, int seg, int shift)
{
    bool ok = true;
    for (int i = lane; i < n; i += kWave) {
        int v = i;
        if (shift > 0) v = i >= shift ? i - shift : i - shift + n;
        else if (peers) v = peers[static_cast<int64_t>(seg) * n + i];
        if (static_cast<unsigned>(v) >= static_cast<unsigned>(n)) { ok = false; v = i; }
        tab[i] = v;
        sched[i] = 0;
    }
    wave_sync();
    for (int i = lane; i < n; i += kWave) atomicAdd(&sched[tab[i]], 1);   // in-degree
    wave_sync();
    for (int i = lane; i < n; i += kWave) ok = ok && (sched[i] == 1);
    const bool valid = __builtin_amdgcn_ballot_w64(!ok) == 0;
    wave_sync();
    if (!valid)
        for (int i = lane; i < n; i += kWave) tab[i] = i;
    wave_sync();
    if (lane == 0) {
        int k = 0;
        for (int start = 0; start < n && k < n; ++start) {
            if (tab[start] < 0) continue;             // already on an earlier cycle
            int cur = start;
            do {
                const int nxt = tab[cur];
                tab[cur] = ~nxt;                      // mark visited
                sched[k++] = cur;
                cur = nxt;
            } while (cur != start && k < n);
            sched[k - 1] |= kLastBit;
        }
    }
    wave_sync();
}

// One lane's walk over all cycles of the schedule.
template <class Op, int U, bool FULL, bool NT>
__device__ __forceinline__ void walk(const Op &op, const int *sched, int n, bool skip_mix,
                                     int64_t off, const unsigned (&mask)[U])
{
    int k = 0;
    while (k < n) {
        int e = uniform(sched[k]);
        Tile<U> cur;
        op.template load<U, FULL, NT>(e & kRowMask, off, mask, cur);
        const Tile<U> first = cur;
        for (;;) {
            const bool last = (e & kLastBit) != 0;
            Tile<U> nxt;
            int e2 = 0;
            if (!last) {
                e2 = uniform(sched[k + 1]);
                op.template load<U, FULL, NT>(e2 & kRowMask, off, mask, nxt);
            } else {
                nxt = first;
            }
            Tile<U> out;
#pragma unroll
            for (int u = 0; u < U; ++u) out.v[u] = skip_mix ? cur.v[u] : (cur.v[u] + nxt.v[u]) * 0.5f;
            op.template store<U, FULL, NT>(e & kRowMask, off, mask, out);
            ++k;
            if (last) break;
            cur = nxt;
            e = e2;
        }
    }
}

template <class Op, int U, bool NT>
__global__ __launch_bounds__(kWave *kMaxWavesPerBlock) void mix_kernel(
    Op op, int n, int64_t P, int S, const int64_t *__restrict__ seg_off,
    const int32_t *__restrict__ peers, int shift, int skip_mix, int64_t ntiles)
{
    extern __shared__ int lds[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * (blockDim.x >> 6) + wave;
    if (tile >= ntiles) return;                 // waves are independent: no block barrier anywhere
    int *tab = lds + wave * 2 * n;
    int *sched = tab + n;

    constexpr int kTileCols = 256 * U;
    const int64_t c0 = tile * kTileCols;
    const int64_t c1 = (c0 + kTileCols < P) ? c0 + kTileCols : P;
    const int64_t off = c0 + 4 * lane;

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
        build_schedule(tab, sched, n, lane, peers, s, shift);
        unsigned mask[U];
        if (b == c0 && e == c0 + kTileCols) {
#pragma unroll
            for (int u = 0; u < U; ++u) mask[u] = 0xFu;
            walk<Op, U, true, NT>(op, sched, n, skip_mix != 0, off, mask);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                mask[u] = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t c = off + u * 256 + q;
                    if (c >= b && c < e) mask[u] |= 1u << q;
                }
            }
            walk<Op, U, false, NT>(op, sched, n, skip_mix != 0, off, mask);
        }
    }
}

// w_out[i] = (w_in[i] + w_in[(i - hop) mod n]) * 0.5f  (push-sum weights, n <= CX_MAX_ROWS)
__global__ void pushsum_weight_kernel(const float *__restrict__ w_in, float *__restrict__ w_out,
                                      int n, int hop)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const int from = i >= hop ? i - hop : i - hop + n;
        w_out[i] = (w_in[i] + w_in[from]) * 0.5f;
    }
}

template <int U, bool NT>
__global__ __launch_bounds__(256) void copy_kernel(const float *src, float *dst, int64_t ntiles,
                                                   int64_t nslices)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * (blockDim.x >> 6) + wave;
    if (tile >= ntiles) return;
    const int64_t first = tile * (64 * U) + lane;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t q = first + u * 64;
        if (q < nslices) {
            const f4 *s = reinterpret_cast<const f4 *>(src) + q;
            f4 *d = reinterpret_cast<f4 *>(dst) + q;
            if (NT) __builtin_nontemporal_store(__builtin_nontemporal_load(s), d); else *d = *s;
        }
    }
}

// ---------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------
struct Launch {
    int U, waves, nt;
};

Launch pick_launch(int default_u)
{
    Launch l;
    l.U = cx_get_tuning(0);
    if (l.U != 1 && l.U != 2 && l.U != 4) l.U = default_u;
    l.waves = cx_get_tuning(1);
    if (l.waves < 1 || l.waves > kMaxWavesPerBlock) l.waves = 4;
    l.nt = cx_get_tuning(2);
    if (l.nt != 0 && l.nt != 1) l.nt = 1;
    return l;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// true if the byte ranges [a, a+bytes) and [b, b+bytes) overlap without being identical
bool partial_overlap(const void *a, const void *b, uint64_t bytes)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    if (x == y) return false;
    return x < y ? (y - x) < bytes : (x - y) < bytes;
}
bool any_overlap(const void *a, const void *b, uint64_t bytes)
{
    return a == b || partial_overlap(a, b, bytes);
}

template <class Op>
int launch_mix(const Op &op, int default_u, int n, int64_t P, int S, const int64_t *seg_off,
               const int32_t *peers, int shift, int skip_mix, hipStream_t stream)
{
    const Launch l = pick_launch(default_u);
    const int64_t tile_cols = 256 * l.U;
    const int64_t ntiles = (P + tile_cols - 1) / tile_cols;
    const int64_t nblocks = (ntiles + l.waves - 1) / l.waves;
    if (nblocks > 0x7fffffffLL) return CX_ERR_SHAPE;
    const dim3 grid(static_cast<unsigned>(nblocks)), block(kWave * l.waves);
    const size_t lds = sizeof(int) * 2 * static_cast<size_t>(n) * l.waves;
#define CX_LAUNCH(UU, NTT) \
    hipLaunchKernelGGL((mix_kernel<Op, UU, NTT>), grid, block, lds, stream, op, n, P, S, seg_off, \
                       peers, shift, skip_mix, ntiles)
    if (l.nt) {
        if (l.U == 1) CX_LAUNCH(1, true); else if (l.U == 2) CX_LAUNCH(2, true); else CX_LAUNCH(4, true);
    } else {
        if (l.U == 1) CX_LAUNCH(1, false); else if (l.U == 2) CX_LAUNCH(2, false); else CX_LAUNCH(4, false);
    }
#undef CX_LAUNCH
    return hipGetLastError() == hipSuccess ? CX_OK : CX_ERR_HIP;
}

int check_matrix_args(const void *x_in, const void *x_out, int64_t ld, int64_t rows, int64_t P,
                      int32_t S, uint32_t flags)
{
    if (!x_in || !x_out) return CX_ERR_NULL;
    if (S < 1 || P < 1 || ld < P || rows < 1) return CX_ERR_SHAPE;
    if (rows > (INT64_MAX / 4) / ld) return CX_ERR_SHAPE;
    if ((ld & 3) != 0 || misaligned(x_in) || misaligned(x_out)) return CX_ERR_ALIGN;
    if (partial_overlap(x_in, x_out, static_cast<uint64_t>(rows) * ld * 4u)) return CX_ERR_ALIAS;
    if (flags != 0) return CX_ERR_UNSUPPORTED;
    return CX_OK;
}

}  // namespace

extern "C" {

int cx_gossip_mix(const float *x_in, float *x_out, int64_t ld, int32_t W, int64_t P, int32_t S,
                  const int64_t *seg_off_dev, const int32_t *peers_dev, uint32_t flags,
                  void *stream)
{
    if (!seg_off_dev || !peers_dev) return CX_ERR_NULL;
    if (W < 2 || W > CX_MAX_ROWS) return (!x_in || !x_out) ? CX_ERR_NULL : CX_ERR_SHAPE;
    const int rc = check_matrix_args(x_in, x_out, ld, W, P, S, flags);
    if (rc != CX_OK) return rc;
    const MeanOp<1> op{x_in, x_out, ld, 1.0f};
    return launch_mix(op, 4, W, P, S, seg_off_dev, peers_dev, 0, 0, static_cast<hipStream_t>(stream));
}

int cx_hier_mix(const float *x_in, float *x_out, int64_t ld, int32_t W, int64_t P, int32_t G,
                int32_t S, const int64_t *seg_off_dev, const int32_t *leader_peers_dev,
                uint32_t flags, void *stream)
{
    if (!seg_off_dev || !x_in || !x_out) return CX_ERR_NULL;
    if (W < 1 || G < 1 || W % G != 0) return CX_ERR_SHAPE;
    const int32_t L = W / G;
    if (L > CX_MAX_ROWS) return CX_ERR_SHAPE;
    if (L > 1 && !leader_peers_dev) return CX_ERR_NULL;
    const int rc = check_matrix_args(x_in, x_out, ld, W, P, S, flags);
    if (rc != CX_OK) return rc;
    const hipStream_t st = static_cast<hipStream_t>(stream);
    const float inv_g = 1.0f / static_cast<float>(G);
    const int skip = (L == 1) ? 1 : 0;
    const int32_t *peers = (L == 1) ? nullptr : leader_peers_dev;
    switch (G) {
    case 1: return launch_mix(MeanOp<1>{x_in, x_out, ld, inv_g}, 4, L, P, S, seg_off_dev, peers, 0, skip, st);
    case 2: return launch_mix(MeanOp<2>{x_in, x_out, ld, inv_g}, 4, L, P, S, seg_off_dev, peers, 0, skip, st);
    case 4: return launch_mix(MeanOp<4>{x_in, x_out, ld, inv_g}, 2, L, P, S, seg_off_dev, peers, 0, skip, st);
    case 8: return launch_mix(MeanOp<8>{x_in, x_out, ld, inv_g}, 2, L, P, S, seg_off_dev, peers, 0, skip, st);
    case 16: return launch_mix(MeanOp<16>{x_in, x_out, ld, inv_g}, 1, L, P, S, seg_off_dev, peers, 0, skip, st);
    default: return CX_ERR_UNSUPPORTED;
    }
}

int cx_pushsum_mix(const float *x_in, float *x_out, const float *w_in, float *w_out, float *z_out,
                   int64_t ld, int32_t W, int64_t P, int32_t hop, uint32_t flags, void *stream)
{
    if (!w_in || !w_out || !x_in || !x_out) return CX_ERR_NULL;
    if (W < 2 || W > CX_MAX_ROWS || hop < 1 || hop >= W) return CX_ERR_SHAPE;
    const int rc = check_matrix_args(x_in, x_out, ld, W, P, 1, flags);
    if (rc != CX_OK) return rc;
    const uint64_t bytes = static_cast<uint64_t>(W) * ld * 4u;
    if (any_overlap(w_in, w_out, static_cast<uint64_t>(W) * 4u)) return CX_ERR_ALIAS;
    if (z_out) {
        if (misaligned(z_out)) return CX_ERR_ALIGN;
        if (any_overlap(z_out, x_in, bytes) || any_overlap(z_out, x_out, bytes)) return CX_ERR_ALIAS;
    }
    const hipStream_t st = static_cast<hipStream_t>(stream);
    // the de-biasing reads w_in, so the weights are written by their own tiny launch
    hipLaunchKernelGGL(pushsum_weight_kernel, dim3(1), dim3(256), 0, st, w_in, w_out, W, hop);
    if (hipGetLastError() != hipSuccess) return CX_ERR_HIP;
    const PushOp op{x_in, x_out, z_out, w_in, ld, W, hop};
    return launch_mix(op, 4, W, P, 1, /*seg_off: unused for S == 1*/ nullptr, nullptr, hop, 0, st);
}

int cx_sgd_fused_mix(const float *x_in, float *x_out, const float *v_in, float *v_out,
                     const float *g, float lr, float mu, float wd, int64_t ld, int32_t W,
                     int64_t P, int32_t S, const int64_t *seg_off_dev, const int32_t *peers_dev,
                     uint32_t flags, void *stream)
{
    if (!seg_off_dev || !peers_dev || !v_in || !v_out || !g) return CX_ERR_NULL;
    if (W < 2 || W > CX_MAX_ROWS) return (!x_in || !x_out) ? CX_ERR_NULL : CX_ERR_SHAPE;
    int rc = check_matrix_args(x_in, x_out, ld, W, P, S, flags);
    if (rc != CX_OK) return rc;
    rc = check_matrix_args(v_in, v_out, ld, W, P, S, flags);
    if (rc != CX_OK) return rc;
    if (misaligned(g)) return CX_ERR_ALIGN;
    const uint64_t bytes = static_cast<uint64_t>(W) * ld * 4u;
    if (any_overlap(x_in, v_in, bytes) || any_overlap(x_in, v_out, bytes) ||
        any_overlap(x_out, v_in, bytes) || any_overlap(x_out, v_out, bytes) ||
        any_overlap(g, x_out, bytes) || any_overlap(g, v_out, bytes))
        return CX_ERR_ALIAS;
    const FusedOp op{x_in, x_out, v_in, v_out, g, ld, lr, mu, wd};
    return launch_mix(op, 2, W, P, S, seg_off_dev, peers_dev, 0, 0, static_cast<hipStream_t>(stream));
}

int cx_copy_baseline(const float *src, float *dst, int64_t n, void *stream)
{
    if (!src || !dst) return CX_ERR_NULL;
    if (n < 4 || (n & 3) != 0) return CX_ERR_SHAPE;
    if (misaligned(src) || misaligned(dst)) return CX_ERR_ALIGN;
    if (any_overlap(src, dst, static_cast<uint64_t>(n) * 4u)) return CX_ERR_ALIAS;
    const Launch l = pick_launch(4);
    const int64_t nslices = n / 4;
    const int64_t ntiles = (nslices + 64 * l.U - 1) / (64 * l.U);
    const int64_t nblocks = (ntiles + 3) / 4;
    if (nblocks > 0x7fffffffLL) return CX_ERR_SHAPE;
    const dim3 grid(static_cast<unsigned>(nblocks)), block(256);
    const hipStream_t st = static_cast<hipStream_t>(stream);
#define CX_COPY(UU, NTT) hipLaunchKernelGGL((copy_kernel<UU, NTT>), grid, block, 0, st, src, dst, ntiles, nslices)
    if (l.nt) {
        if (l.U == 1) CX_COPY(1, true); else if (l.U == 2) CX_COPY(2, true); else CX_COPY(4, true);
    } else {
        if (l.U == 1) CX_COPY(1, false); else if (l.U == 2) CX_COPY(2, false); else CX_COPY(4, false);
    }
#undef CX_COPY
    return hipGetLastError() == hipSuccess ? CX_OK : CX_ERR_HIP;
}

}  // extern "C"
