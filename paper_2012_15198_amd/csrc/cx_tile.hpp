// Building blocks of the device half (internal header): the 16-byte column slice a lane handles, the tiles
// of slices a lane keeps in registers (fp32, and fp64 for the operators that compute there), the pairwise
// average, and the fp32 row accesses -- full tiles as one 16-byte access per slice, boundary tiles element by
// element under a mask.  The overview of the kernels is at the top of cx_kernels.hpp.
#ifndef CX_TILE_HPP
#define CX_TILE_HPP
#include "cx_mix.h"

#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <type_traits>

#define CX_SCHED_FN __device__ __forceinline__
#include "cx_schedule.hpp"          // build_schedule: the cycle order of a peer table
static_assert(CX_MAX_ROWS <= (1 << kRowBits), "row ids must fit the schedule's packed fields");

extern "C" int cx_get_tuning(int32_t key);

#pragma clang fp contract(off)

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

}  // namespace

#endif  // CX_TILE_HPP
