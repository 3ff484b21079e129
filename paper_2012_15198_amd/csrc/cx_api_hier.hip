// C-ABI entry point(s) cx_hier_mix: argument checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

extern "C" {

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
    const int skip = (L == 1) ? 1 : 0;
    const int32_t *peers = (L == 1) ? nullptr : leader_peers_dev;
    const MixArgs a{L, P, S, seg_off_dev, peers, 0, skip, st, x_in != x_out, G};
    switch (G) {
    case 1: return launch_mix<MeanOp<1>>(MeanOp<1>{x_in, x_out, ld}, a);
    case 2: return launch_mix<MeanOp<2>>(MeanOp<2>{x_in, x_out, ld}, a);
    case 3: return launch_mix<MeanOp<3>>(MeanOp<3>{x_in, x_out, ld}, a);
    case 4: return launch_mix<MeanOp<4>>(MeanOp<4>{x_in, x_out, ld}, a);
    case 5: return launch_mix<MeanOp<5>>(MeanOp<5>{x_in, x_out, ld}, a);
    case 6: return launch_mix<MeanOp<6>>(MeanOp<6>{x_in, x_out, ld}, a);
    case 7: return launch_mix<MeanOp<7>>(MeanOp<7>{x_in, x_out, ld}, a);
    case 8:
        // launch parameter 10: the group mean staged through LDS (one row per wavefront) instead of the
        // sum in registers -- same results, kept so that the two can be measured side by side
        if (cx_get_tuning(10) == 1) return launch_mix<MeanLdsOp<8>>(MeanLdsOp<8>{{x_in, x_out, ld}}, a);
        return launch_mix<MeanOp<8>>(MeanOp<8>{x_in, x_out, ld}, a);
    case 16: return launch_mix<MeanOp<16>>(MeanOp<16>{x_in, x_out, ld}, a);
    default: return CX_ERR_UNSUPPORTED;
    }
}

}  // extern "C"
