// C-ABI entry points cx_hier_mix_bf16 / cx_hier_mix_f16: argument checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

namespace {

template <bool IEEE_HALF>
int hier_mix16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P, int32_t G,
               int32_t S, const int64_t *seg_off_dev, const int32_t *leader_peers_dev, uint32_t flags,
               void *stream)
{
    if (!seg_off_dev || !x_in || !x_out) return CX_ERR_NULL;
    if (W < 1 || G < 1 || W % G != 0) return CX_ERR_SHAPE;
    if (G == 1 && W >= 2)             // groups of one: the flat 16-bit mix, bit for bit
        return IEEE_HALF ? cx_gossip_mix_f16(x_in, x_out, ld, W, P, S, seg_off_dev, leader_peers_dev, flags, stream)
                         : cx_gossip_mix_bf16(x_in, x_out, ld, W, P, S, seg_off_dev, leader_peers_dev, flags, stream);
    if (G == 1) return CX_ERR_SHAPE;  // a single row has nothing to mix with
    const int32_t L = W / G;
    if (L > CX_MAX_ROWS) return CX_ERR_SHAPE;
    if (L > 1 && !leader_peers_dev) return CX_ERR_NULL;
    const int rc = check_matrix_args(x_in, x_out, ld, W, P, S, flags, 2);
    if (rc != CX_OK) return rc;
    const hipStream_t st = static_cast<hipStream_t>(stream);
    const int skip = (L == 1) ? 1 : 0;
    const int32_t *peers = (L == 1) ? nullptr : leader_peers_dev;
    const MixArgs a{L, P, S, seg_off_dev, peers, 0, skip, st, x_in != x_out, G};
    switch (G) {
    case 2: return launch_mix<Row16Op<IEEE_HALF, 2>>(Row16Op<IEEE_HALF, 2>{x_in, x_out, ld}, a);
    case 3: return launch_mix<Row16Op<IEEE_HALF, 3>>(Row16Op<IEEE_HALF, 3>{x_in, x_out, ld}, a);
    case 4: return launch_mix<Row16Op<IEEE_HALF, 4>>(Row16Op<IEEE_HALF, 4>{x_in, x_out, ld}, a);
    case 5: return launch_mix<Row16Op<IEEE_HALF, 5>>(Row16Op<IEEE_HALF, 5>{x_in, x_out, ld}, a);
    case 6: return launch_mix<Row16Op<IEEE_HALF, 6>>(Row16Op<IEEE_HALF, 6>{x_in, x_out, ld}, a);
    case 7: return launch_mix<Row16Op<IEEE_HALF, 7>>(Row16Op<IEEE_HALF, 7>{x_in, x_out, ld}, a);
    case 8: return launch_mix<Row16Op<IEEE_HALF, 8>>(Row16Op<IEEE_HALF, 8>{x_in, x_out, ld}, a);
    default: return CX_ERR_UNSUPPORTED;
    }
}

}  // namespace

extern "C" {

int cx_hier_mix_bf16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P, int32_t G,
                     int32_t S, const int64_t *seg_off_dev, const int32_t *leader_peers_dev,
                     uint32_t flags, void *stream)
{
    return hier_mix16<false>(x_in, x_out, ld, W, P, G, S, seg_off_dev, leader_peers_dev, flags, stream);
}

int cx_hier_mix_f16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P, int32_t G,
                    int32_t S, const int64_t *seg_off_dev, const int32_t *leader_peers_dev,
                    uint32_t flags, void *stream)
{
    return hier_mix16<true>(x_in, x_out, ld, W, P, G, S, seg_off_dev, leader_peers_dev, flags, stream);
}

}  // extern "C"
