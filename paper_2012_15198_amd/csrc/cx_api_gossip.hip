// C-ABI entry point(s) cx_gossip_mix, cx_copy_baseline: argument checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

namespace {

// Plain streaming copy with the mixing kernels' load/store instructions (cx_copy_baseline).
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
    const MeanOp<1> op{x_in, x_out, ld};
    const MixArgs a{W, P, S, seg_off_dev, peers_dev, 0, 0, static_cast<hipStream_t>(stream), x_in != x_out, 1};
    return launch_mix<MeanOp<1>>(op, a);
}

int cx_copy_baseline(const float *src, float *dst, int64_t n, void *stream)
{
    if (!src || !dst) return CX_ERR_NULL;
    if (n < 4 || (n & 3) != 0) return CX_ERR_SHAPE;
    if (misaligned(src) || misaligned(dst)) return CX_ERR_ALIGN;
    if (any_overlap(src, dst, static_cast<uint64_t>(n) * 4u)) return CX_ERR_ALIAS;
    const Launch l = pick_launch(WalkShape{1, 2, 4, 0});
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
