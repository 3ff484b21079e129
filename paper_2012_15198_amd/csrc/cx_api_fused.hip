// C-ABI entry point(s) cx_sgd_fused_mix: argument checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

extern "C" {

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
    const FusedOp op{x_in, x_out, v_in, v_out, g, ld, SgdStep{lr, mu, wd}};
    const MixArgs a{W, P, S, seg_off_dev, peers_dev, 0, 0, static_cast<hipStream_t>(stream),
                    x_in != x_out && v_in != v_out, 1};
    return launch_mix<FusedOp>(op, a);
}

}  // extern "C"
