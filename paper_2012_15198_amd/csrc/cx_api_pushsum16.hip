// C-ABI entry points cx_pushsum_mix_bf16, cx_pushsum_mix_f16: argument checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

namespace {

template <bool IEEE_HALF>
int pushsum16(const uint16_t *x_in, uint16_t *x_out, const float *w_in, float *w_out, uint16_t *z_out,
              int64_t ld, int32_t W, int64_t P, int32_t hop, uint32_t flags, void *stream)
{
    if (!w_in || !w_out || !x_in || !x_out) return CX_ERR_NULL;
    if (W < 2 || W > CX_MAX_ROWS || hop < 1 || hop >= W) return CX_ERR_SHAPE;
    const int rc = check_matrix_args(x_in, x_out, ld, W, P, 1, flags, 2);
    if (rc != CX_OK) return rc;
    const uint64_t bytes = static_cast<uint64_t>(W) * ld * 2u;
    if (any_overlap(w_in, w_out, static_cast<uint64_t>(W) * 4u)) return CX_ERR_ALIAS;
    if (z_out) {
        if (misaligned(z_out)) return CX_ERR_ALIGN;
        if (any_overlap(z_out, x_in, bytes) || any_overlap(z_out, x_out, bytes)) return CX_ERR_ALIAS;
    }
    const hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(pushsum_weight_kernel, dim3(1), dim3(256), 0, st, w_in, w_out, W, hop);
    if (hipGetLastError() != hipSuccess) return CX_ERR_HIP;
    using Op = Push16Op<IEEE_HALF>;
    const Op op{{x_in, x_out, ld}, z_out, w_in, W, hop};
    const MixArgs a{W, P, 1, /*seg_off: unused for S == 1*/ nullptr, nullptr, hop, 0, st, x_in != x_out, 1};
    return launch_mix<Op>(op, a);
}

}  // namespace

extern "C" {

int cx_pushsum_mix_bf16(const uint16_t *x_in, uint16_t *x_out, const float *w_in, float *w_out, uint16_t *z_out,
                        int64_t ld, int32_t W, int64_t P, int32_t hop, uint32_t flags, void *stream)
{
    return pushsum16<false>(x_in, x_out, w_in, w_out, z_out, ld, W, P, hop, flags, stream);
}

int cx_pushsum_mix_f16(const uint16_t *x_in, uint16_t *x_out, const float *w_in, float *w_out, uint16_t *z_out,
                       int64_t ld, int32_t W, int64_t P, int32_t hop, uint32_t flags, void *stream)
{
    return pushsum16<true>(x_in, x_out, w_in, w_out, z_out, ld, W, P, hop, flags, stream);
}

}  // extern "C"
