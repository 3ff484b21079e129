// C-ABI entry point(s) cx_pushsum_mix: argument checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

extern "C" {

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
    hipLaunchKernelGGL(pushsum_weight_kernel, dim3(1), dim3(256), 0, st, w_in, w_out, W, hop);
    if (hipGetLastError() != hipSuccess) return CX_ERR_HIP;
    const PushOp op{x_in, x_out, z_out, w_in, ld, W, hop};
    const MixArgs a{W, P, 1, /*seg_off: unused for S == 1*/ nullptr, nullptr, hop, 0, st, x_in != x_out, 1};
    return launch_mix<PushOp>(op, a);
}

}  // extern "C"
