// Row operators on 16-bit rows, bfloat16 and IEEE binary16 (internal header; Section 4.1's mixed precision):
// exact widening, the single rounding on the way out, the flat and hierarchical mean, the push-sum comparison,
// and the two optimizer steps with fp32 momentum staged through LDS.
#ifndef CX_OPS16_HPP
#define CX_OPS16_HPP
#include "cx_ops.hpp"

#pragma clang fp contract(off)

namespace {

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

// The SGP-style push-sum comparison on 16-bit rows (PushOp in cx_ops.hpp is the fp32-row one): the rows are widened
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

}  // namespace

#endif  // CX_OPS16_HPP
