// C-ABI entry points cx_sgd_fused_mix_bf16 / _f16 and cx_hier_sgd_fused_mix_bf16 / _f16: argument
// checks and launch (see include/cx_mix.h).
#include "cx_launch.hpp"

namespace {

// true if [a, a+na) and [b, b+nb) share a byte
bool ranges_overlap(const void *a, uint64_t na, const void *b, uint64_t nb)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y ? (y - x) < na : (x - y) < nb;
}

// x, g: uint16 [W][ld]; v: float [vrows][ld].  Every buffer 16-byte aligned, ld % 8 == 0; outputs
// either are their inputs or overlap nothing.
int check_mixed_args(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out, const uint16_t *g,
                     int64_t ld, int64_t W, int64_t vrows, int64_t P, int32_t S, uint32_t flags)
{
    int rc = check_matrix_args(x_in, x_out, ld, W, P, S, flags, 2);
    if (rc != CX_OK) return rc;
    rc = check_matrix_args(v_in, v_out, ld, vrows, P, S, flags, 4);
    if (rc != CX_OK) return rc;
    if (ld % 8 != 0 || misaligned(g)) return CX_ERR_ALIGN;
    if ((x_in == x_out) != (v_in == v_out)) return CX_ERR_ALIAS;
    const uint64_t xb = static_cast<uint64_t>(W) * ld * 2u, vb = static_cast<uint64_t>(vrows) * ld * 4u;
    if (ranges_overlap(x_in, xb, v_in, vb) || ranges_overlap(x_in, xb, v_out, vb) ||
        ranges_overlap(x_out, xb, v_in, vb) || ranges_overlap(x_out, xb, v_out, vb) ||
        ranges_overlap(g, xb, v_out, vb) || ranges_overlap(g, xb, x_out, xb))
        return CX_ERR_ALIAS;
    return CX_OK;
}

template <bool IEEE_HALF>
int fused16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out, const uint16_t *g, float lr,
            float mu, float wd, int64_t ld, int32_t W, int64_t P, int32_t S, const int64_t *seg_off_dev,
            const int32_t *peers_dev, uint32_t flags, void *stream)
{
    if (!seg_off_dev || !peers_dev || !x_in || !x_out || !v_in || !v_out || !g) return CX_ERR_NULL;
    if (W < 2 || W > CX_MAX_ROWS) return CX_ERR_SHAPE;
    const int rc = check_mixed_args(x_in, x_out, v_in, v_out, g, ld, W, W, P, S, flags);
    if (rc != CX_OK) return rc;
    const Fused16Op<IEEE_HALF> op{x_in, x_out, v_in, v_out, g, ld, SgdStep{lr, mu, wd}};
    const MixArgs a{W, P, S, seg_off_dev, peers_dev, 0, 0, static_cast<hipStream_t>(stream), x_in != x_out, 1};
    return launch_mix<Fused16Op<IEEE_HALF>>(op, a);
}

template <bool IEEE_HALF>
int hier_fused16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out, const uint16_t *g, float lr,
                 float mu, float wd, int64_t ld, int32_t W, int64_t P, int32_t G, int32_t S,
                 const int64_t *seg_off_dev, const int32_t *leader_peers_dev, uint32_t flags, void *stream)
{
    if (!seg_off_dev || !x_in || !x_out || !v_in || !v_out || !g) return CX_ERR_NULL;
    if (W < 1 || G < 1 || W % G != 0) return CX_ERR_SHAPE;
    const int32_t L = W / G;
    if (L > CX_MAX_ROWS) return CX_ERR_SHAPE;
    if (L > 1 && !leader_peers_dev) return CX_ERR_NULL;
    const int rc = check_mixed_args(x_in, x_out, v_in, v_out, g, ld, W, L, P, S, flags);
    if (rc != CX_OK) return rc;
    const SgdStep sgd{lr, mu, wd};
    const int skip = (L == 1) ? 1 : 0;
    const int32_t *peers = (L == 1) ? nullptr : leader_peers_dev;
    const MixArgs a{L, P, S, seg_off_dev, peers, 0, skip, static_cast<hipStream_t>(stream), x_in != x_out, G};
    switch (G) {
    case 1: return launch_mix<HierFused16Op<IEEE_HALF, 1>>(HierFused16Op<IEEE_HALF, 1>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 2: return launch_mix<HierFused16Op<IEEE_HALF, 2>>(HierFused16Op<IEEE_HALF, 2>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 3: return launch_mix<HierFused16Op<IEEE_HALF, 3>>(HierFused16Op<IEEE_HALF, 3>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 4: return launch_mix<HierFused16Op<IEEE_HALF, 4>>(HierFused16Op<IEEE_HALF, 4>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 5: return launch_mix<HierFused16Op<IEEE_HALF, 5>>(HierFused16Op<IEEE_HALF, 5>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 6: return launch_mix<HierFused16Op<IEEE_HALF, 6>>(HierFused16Op<IEEE_HALF, 6>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 7: return launch_mix<HierFused16Op<IEEE_HALF, 7>>(HierFused16Op<IEEE_HALF, 7>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    case 8: return launch_mix<HierFused16Op<IEEE_HALF, 8>>(HierFused16Op<IEEE_HALF, 8>{x_in, x_out, v_in, v_out, g, ld, sgd}, a);
    default: return CX_ERR_UNSUPPORTED;
    }
}

}  // namespace

extern "C" {

int cx_sgd_fused_mix_bf16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out, const uint16_t *g,
                          float lr, float mu, float wd, int64_t ld, int32_t W, int64_t P, int32_t S,
                          const int64_t *seg_off_dev, const int32_t *peers_dev, uint32_t flags, void *stream)
{
    return fused16<false>(x_in, x_out, v_in, v_out, g, lr, mu, wd, ld, W, P, S, seg_off_dev, peers_dev, flags, stream);
}

int cx_sgd_fused_mix_f16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out, const uint16_t *g,
                         float lr, float mu, float wd, int64_t ld, int32_t W, int64_t P, int32_t S,
                         const int64_t *seg_off_dev, const int32_t *peers_dev, uint32_t flags, void *stream)
{
    return fused16<true>(x_in, x_out, v_in, v_out, g, lr, mu, wd, ld, W, P, S, seg_off_dev, peers_dev, flags, stream);
}

int cx_hier_sgd_fused_mix_bf16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out,
                               const uint16_t *g, float lr, float mu, float wd, int64_t ld, int32_t W, int64_t P,
                               int32_t G, int32_t S, const int64_t *seg_off_dev, const int32_t *leader_peers_dev,
                               uint32_t flags, void *stream)
{
    return hier_fused16<false>(x_in, x_out, v_in, v_out, g, lr, mu, wd, ld, W, P, G, S, seg_off_dev, leader_peers_dev,
                               flags, stream);
}

int cx_hier_sgd_fused_mix_f16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out,
                              const uint16_t *g, float lr, float mu, float wd, int64_t ld, int32_t W, int64_t P,
                              int32_t G, int32_t S, const int64_t *seg_off_dev, const int32_t *leader_peers_dev,
                              uint32_t flags, void *stream)
{
    return hier_fused16<true>(x_in, x_out, v_in, v_out, g, lr, mu, wd, ld, W, P, G, S, seg_off_dev, leader_peers_dev,
                              flags, stream);
}

}  // extern "C"
