// C-ABI entry point cx_gossip_mix_bf16: argument checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

extern "C" {

int cx_gossip_mix_bf16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P,
                       int32_t S, const int64_t *seg_off_dev, const int32_t *peers_dev,
                       uint32_t flags, void *stream)
{
    if (!seg_off_dev || !peers_dev) return CX_ERR_NULL;
    if (W < 2 || W > CX_MAX_ROWS) return (!x_in || !x_out) ? CX_ERR_NULL : CX_ERR_SHAPE;
    const int rc = check_matrix_args(x_in, x_out, ld, W, P, S, flags, 2);
    if (rc != CX_OK) return rc;
    const Bf16Op op{x_in, x_out, ld};
    const MixArgs a{W, P, S, seg_off_dev, peers_dev, 0, 0, static_cast<hipStream_t>(stream), x_in != x_out, 1};
    return launch_mix<Bf16Op>(op, a);
}

}  // extern "C"
