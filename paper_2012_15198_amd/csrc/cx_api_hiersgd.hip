// C-ABI entry point(s) cx_hier_sgd_fused_mix: argument checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

extern "C" {

int cx_hier_sgd_fused_mix(const float *x_in, float *x_out, const float *v_in, float *v_out,
                          const float *g, float lr, float mu, float wd, int64_t ld, int32_t W,
                          int64_t P, int32_t G, int32_t S, const int64_t *seg_off_dev,
                          const int32_t *leader_peers_dev, uint32_t flags, void *stream)
{
    if (!seg_off_dev || !x_in || !x_out || !v_in || !v_out || !g) return CX_ERR_NULL;
    if (W < 1 || G < 1 || W % G != 0) return CX_ERR_SHAPE;
    const int32_t L = W / G;
    if (L > CX_MAX_ROWS) return CX_ERR_SHAPE;
    if (L > 1 && !leader_peers_dev) return CX_ERR_NULL;
    int rc = check_matrix_args(x_in, x_out, ld, W, P, S, flags);
    if (rc != CX_OK) return rc;
    rc = check_matrix_args(v_in, v_out, ld, L, P, S, flags);
    if (rc != CX_OK) return rc;
    if (misaligned(g)) return CX_ERR_ALIGN;
    if ((x_in == x_out) != (v_in == v_out)) return CX_ERR_ALIAS;
    const uint64_t xbytes = static_cast<uint64_t>(W) * ld * 4u, vbytes = static_cast<uint64_t>(L) * ld * 4u;
    // v against x and g (ranges of different length: test with the longer one from the x/g side)
    const auto overlap2 = [](const void *a, uint64_t na, const void *b, uint64_t nb) {
        const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
        return x < y ? (y - x) < na : (x - y) < nb;
    };
    if (overlap2(x_in, xbytes, v_in, vbytes) || overlap2(x_in, xbytes, v_out, vbytes) ||
        overlap2(x_out, xbytes, v_in, vbytes) || overlap2(x_out, xbytes, v_out, vbytes) ||
        overlap2(g, xbytes, v_out, vbytes) || any_overlap(g, x_out, xbytes))
        return CX_ERR_ALIAS;
    const hipStream_t st = static_cast<hipStream_t>(stream);
    const SgdStep sgd{lr, mu, wd};
    const int skip = (L == 1) ? 1 : 0;
    const int32_t *peers = (L == 1) ? nullptr : leader_peers_dev;
    const MixArgs a{L, P, S, seg_off_dev, peers, 0, skip, st, x_in != x_out, G};
    switch (G) {
    case 1: return launch_mix<HierFusedOp<1>>(HierFusedOp<1>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 2: return launch_mix<HierFusedOp<2>>(HierFusedOp<2>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 3: return launch_mix<HierFusedOp<3>>(HierFusedOp<3>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 4: return launch_mix<HierFusedOp<4>>(HierFusedOp<4>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 5: return launch_mix<HierFusedOp<5>>(HierFusedOp<5>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 6: return launch_mix<HierFusedOp<6>>(HierFusedOp<6>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 7: return launch_mix<HierFusedOp<7>>(HierFusedOp<7>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 8: return launch_mix<HierFusedOp<8>>(HierFusedOp<8>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 16: return launch_mix<HierFusedOp<16>>(HierFusedOp<16>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    default: return CX_ERR_UNSUPPORTED;
    }
}

}  // extern "C"
