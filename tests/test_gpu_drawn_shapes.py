"""Every entry point on shapes drawn from a seeded generator instead of a hand-picked list: row
counts, group sizes, row lengths that end anywhere inside a tile, row strides with and without
padding, ragged segment tables with empty segments, in place and out of place.  Each result must
be the oracle's, bit for bit (fp64 references rounded once, as the parity bars say)."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2012_15198_amd import cxmix as cx
from paper_2012_15198_amd import workloads as WL
from gpu_util import Tuning, dev, host, once, same_bits

pytestmark = pytest.mark.gpu

CASES = 60
LR, MU, WD = 0.1, 0.9, 1e-4


def d16(a):
    return dev(np.ascontiguousarray(a).view(np.int16))


def h16(t):
    return host(t).view(np.uint16)


def draw_shape(rng, align, grouped):
    """(W, G, P, ld, seg_off): P from one column to a few dozen tiles, ld = P rounded up to the
    alignment plus sometimes a few slices of padding, S - 1 boundaries anywhere (repeats = empty segments)."""
    G = int(rng.integers(1, 9)) if grouped else 1
    L = int(rng.integers(2, 13)) if G > 1 else int(rng.integers(2, 41))
    if G > 1 and rng.random() < 0.15:
        L = 1                                    # one group: no leader gossip, every row the mean
    P = int(rng.choice([rng.integers(1, 64), rng.integers(64, 5000), rng.integers(5000, 60000)]))
    ld = (P + align - 1) // align * align + align * int(rng.integers(0, 3))
    S = int(rng.integers(1, 10))
    inner = np.sort(rng.integers(0, P + 1, size=S - 1))
    seg_off = np.concatenate([[0], inner, [P]]).astype(np.int64)
    return L * G, G, P, ld, seg_off


def tables(seed, L, S):
    return O.topology(seed, L, S, 0, 1)[0] if L > 1 else None


def tdev(t):
    return dev(t) if t is not None else None


@pytest.mark.parametrize("case", range(CASES))
def test_gossip_and_hierarchical_mix(case):
    rng = np.random.default_rng(1000 + case)
    W, G, P, ld, so = draw_shape(rng, 4, grouped=case % 2 == 1)
    x = WL.gen_matrix(W, P, 0.05, seed=1000 + case, ld=ld)
    pe = tables(case, W // G, len(so) - 1)
    print(f"W={W} G={G} P={P} ld={ld} seg_off={so.tolist()}", flush=True)
    if G == 1:
        want = O.gossip_mix(x, P, so, pe)
        call = lambda a, b: cx.cx_gossip_mix(a, b, P, dev(so), dev(pe))
    else:
        want = once(O.hier_mix_f64(x, P, G, so, pe))
        call = lambda a, b: cx.cx_hier_mix(a, b, P, G, dev(so), tdev(pe))
    a, b = dev(x), torch.full((W, ld), float("nan"), device="cuda:0")
    b[:, P:] = a[:, P:]
    call(a, b)
    c = dev(x)
    call(c, c)
    torch.cuda.synchronize()
    assert same_bits(host(b), want) and same_bits(host(c), want)
    assert same_bits(host(a), x)


@pytest.mark.parametrize("case", range(CASES))
def test_optimizer_steps(case):
    rng = np.random.default_rng(2000 + case)
    W, G, P, ld, so = draw_shape(rng, 4, grouped=case % 2 == 1)
    L = W // G
    x = WL.gen_matrix(W, P, 0.05, seed=2000 + case, ld=ld)
    v = WL.gen_matrix(L, P, 0.02, seed=2000 + case, ld=ld, stream=1)
    g = WL.gen_matrix(W, P, 0.01, seed=2000 + case, ld=ld, stream=2)
    pe = tables(case, L, len(so) - 1)
    print(f"W={W} G={G} P={P} ld={ld} seg_off={so.tolist()}", flush=True)
    if case % 4 == 0:
        wx, wv = (once(t) for t in O.sgd_fused_mix_f64(x, v, g, LR, MU, WD, P, so, pe))
        call = lambda xi, xo, vi, vo: cx.cx_sgd_fused_mix(xi, xo, vi, vo, dev(g), LR, MU, WD, P, dev(so), dev(pe))
    else:
        wx, wv = (once(t) for t in O.hier_sgd_fused_mix_f64(x, v, g, LR, MU, WD, P, G, so, pe))
        call = lambda xi, xo, vi, vo: cx.cx_hier_sgd_fused_mix(xi, xo, vi, vo, dev(g), LR, MU, WD, P, G, dev(so), tdev(pe))
    xi, vi = dev(x), dev(v)
    xo, vo = dev(x), dev(v)
    call(xi, xo, vi, vo)
    xc, vc = dev(x), dev(v)
    call(xc, xc, vc, vc)
    torch.cuda.synchronize()
    assert same_bits(host(xo), wx) and same_bits(host(vo), wv)
    assert same_bits(host(xc), wx) and same_bits(host(vc), wv)


@pytest.mark.parametrize("case", range(CASES))
def test_pushsum(case):
    rng = np.random.default_rng(3000 + case)
    W, _, P, ld, _ = draw_shape(rng, 4, grouped=False)
    hop = int(rng.integers(1, W))
    x = WL.gen_matrix(W, P, 0.05, seed=3000 + case, ld=ld)
    w = (0.5 + rng.random(W)).astype(np.float32)
    print(f"W={W} P={P} ld={ld} hop={hop}", flush=True)
    wx, ww, wz = O.pushsum_mix_f32(x, w, P, hop, True)
    xi, wi = dev(x), dev(w)
    xo, wo, z = dev(x), torch.zeros_like(wi), torch.zeros_like(xi)
    cx.cx_pushsum_mix(xi, xo, wi, wo, z, P, hop)
    xc, wc = dev(x), torch.zeros_like(wi)
    cx.cx_pushsum_mix(xc, xc, wi, wc, None, P, hop)
    torch.cuda.synchronize()
    assert same_bits(host(xo), wx) and same_bits(host(wo), ww) and same_bits(host(z)[:, :P], wz[:, :P])
    assert same_bits(host(xc), wx) and same_bits(host(wc), ww)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
@pytest.mark.parametrize("case", range(CASES))
def test_sixteen_bit_rows(case, fmt):
    """Case by case one of: flat mix, hierarchical mix, fused step, gradient-reducing step, push-sum."""
    rng = np.random.default_rng(4000 + case)
    kind = case % 5
    W, G, P, ld, so = draw_shape(rng, 8, grouped=kind in (1, 3))
    L = W // G
    narrow = O.f32_to_bf16 if fmt == "bf16" else O.f32_to_f16
    pick = lambda name: getattr(cx, f"{name}_{fmt}")
    x = narrow(WL.gen_matrix(W, P, 0.05, seed=4000 + case, ld=ld))
    pe = tables(case, L, len(so) - 1)
    print(f"kind={kind} W={W} G={G} P={P} ld={ld} seg_off={so.tolist()}", flush=True)
    sod = dev(so)
    if kind == 0:
        want = (O.gossip_mix_bf16 if fmt == "bf16" else O.gossip_mix_f16)(x, P, so, pe)
        for inplace in (False, True):
            a = d16(x)
            b = a if inplace else d16(x)
            pick("cx_gossip_mix")(a, b, P, sod, dev(pe))
            torch.cuda.synchronize()
            assert (h16(b) == want).all(), inplace
    elif kind == 1:
        want = O.hier_mix16(fmt, x, P, G, so, pe) if G > 1 else \
            (O.gossip_mix_bf16 if fmt == "bf16" else O.gossip_mix_f16)(x, P, so, pe)
        for inplace in (False, True):
            a = d16(x)
            b = a if inplace else d16(x)
            pick("cx_hier_mix")(a, b, P, G, sod, tdev(pe))
            torch.cuda.synchronize()
            assert (h16(b) == want).all(), inplace
    elif kind in (2, 3):
        v = WL.gen_matrix(L, P, 0.02, seed=4000 + case, ld=ld, stream=1)
        g = narrow(WL.gen_matrix(W, P, 0.01, seed=4000 + case, ld=ld, stream=2))
        if kind == 2:
            wx, wv = O.sgd_fused_mix16(fmt, x, v, g, LR, MU, WD, P, so, pe)
            call = lambda xi, xo, vi, vo: pick("cx_sgd_fused_mix")(xi, xo, vi, vo, d16(g), LR, MU, WD, P, sod, dev(pe))
        else:
            wx, wv = O.hier_sgd_fused_mix16(fmt, x, v, g, LR, MU, WD, P, G, so, pe)
            call = lambda xi, xo, vi, vo: pick("cx_hier_sgd_fused_mix")(xi, xo, vi, vo, d16(g), LR, MU, WD, P, G, sod,
                                                                          tdev(pe))
        for inplace in (False, True):
            xi, vi = d16(x), dev(v)
            xo, vo = (xi, vi) if inplace else (d16(x), dev(v))
            call(xi, xo, vi, vo)
            torch.cuda.synchronize()
            assert (h16(xo) == wx).all() and same_bits(host(vo), wv), inplace
    else:
        hop = int(rng.integers(1, W))
        w = (0.5 + rng.random(W)).astype(np.float32)
        wx, ww, wz = O.pushsum_mix16(fmt, x, w, P, hop, True)
        for inplace in (False, True):
            xi, wi = d16(x), dev(w)
            xo = xi if inplace else d16(x)
            wo, z = torch.zeros_like(wi), d16(x)
            pick("cx_pushsum_mix")(xi, xo, wi, wo, z, P, hop)
            torch.cuda.synchronize()
            assert (h16(xo) == wx).all() and same_bits(host(wo), ww), inplace
            assert (h16(z)[:, :P] == wz[:, :P]).all(), inplace


def draw_tuning(rng):
    """Launch parameters anywhere in their documented ranges (-1 = the operator's default)."""
    pick = lambda values: int(rng.choice(values))
    return Tuning(slices=pick([-1, 1, 2, 4]), waves=pick([-1, 1, 2, 3, 4, 5, 8]), nt=pick([-1, 0, 1]),
                  depth=pick([-1, 2, 4, 8]), lockstep=pick([-1, 0, 1]), force_walk=pick([-1, 0, 0, 1]),
                  cluster=pick([-1, 1, 2, 3, 7, 64, 4096]), xcd_aware=pick([-1, 0, 1]), ordered=pick([-1, 0, 1, 1]),
                  wgs_per_cu=pick([-1, 0, 1, 2, 8, 16]), lds_mean=pick([-1, 0, 1]))


@pytest.mark.parametrize("case", range(CASES))
def test_drawn_shapes_under_drawn_launch_parameters(case):
    """Shape and launch shape both drawn: flat or hierarchical mix (groups of 8 every third case, which
    the LDS-staged mean serves), then the matching optimizer step, fp32 and bf16 rows."""
    rng = np.random.default_rng(5000 + case)
    W, G, P, ld, so = draw_shape(rng, 8, grouped=case % 2 == 1)
    if case % 3 == 0:
        L = int(rng.integers(2, 10))
        W, G = 8 * L, 8
    L = W // G
    tune = draw_tuning(rng)
    print(f"W={W} G={G} P={P} ld={ld} seg_off={so.tolist()} tuning={tune.v}", flush=True)
    x = WL.gen_matrix(W, P, 0.05, seed=5000 + case, ld=ld)
    v = WL.gen_matrix(L, P, 0.02, seed=5000 + case, ld=ld, stream=1)
    g = WL.gen_matrix(W, P, 0.01, seed=5000 + case, ld=ld, stream=2)
    x16, g16 = O.f32_to_bf16(x), O.f32_to_bf16(g)
    pe = tables(case, L, len(so) - 1)
    sod, ped = dev(so), tdev(pe)
    if G == 1:
        want = O.gossip_mix(x, P, so, pe)
        want16 = O.gossip_mix_bf16(x16, P, so, pe)
    else:
        want = once(O.hier_mix_f64(x, P, G, so, pe))
        want16 = O.hier_mix16("bf16", x16, P, G, so, pe)
    wx, wv = (once(t) for t in O.hier_sgd_fused_mix_f64(x, v, g, LR, MU, WD, P, G, so, pe))
    wx16, wv16 = O.hier_sgd_fused_mix16("bf16", x16, v, g16, LR, MU, WD, P, G, so, pe)
    with tune:
        for inplace in (False, True):
            a = dev(x)
            b = a if inplace else dev(x)
            cx.cx_hier_mix(a, b, P, G, sod, ped)
            a16 = d16(x16)
            b16 = a16 if inplace else d16(x16)
            cx.cx_hier_mix_bf16(a16, b16, P, G, sod, ped)
            xi, vi = dev(x), dev(v)
            xo, vo = (xi, vi) if inplace else (dev(x), dev(v))
            cx.cx_hier_sgd_fused_mix(xi, xo, vi, vo, dev(g), LR, MU, WD, P, G, sod, ped)
            yi, ui = d16(x16), dev(v)
            yo, uo = (yi, ui) if inplace else (d16(x16), dev(v))
            cx.cx_hier_sgd_fused_mix_bf16(yi, yo, ui, uo, d16(g16), LR, MU, WD, P, G, sod, ped)
            torch.cuda.synchronize()
            assert same_bits(host(b), want), inplace
            assert (h16(b16) == want16).all(), inplace
            assert same_bits(host(xo), wx) and same_bits(host(vo), wv), inplace
            assert (h16(yo) == wx16).all() and same_bits(host(uo), wv16), inplace


def test_largest_row_count_in_every_entry_point():
    """CX_MAX_ROWS gossiping rows -- the longest peer table and the longest cycles the library takes --
    through the optimizer steps, push-sum and the 16-bit rows, in both buffer modes."""
    W, P, ld, S = cx.CX_MAX_ROWS, 777, 784, 3
    so = WL.equal_seg_off(P, S)
    pe = O.topology(77, W, S, 0, 1)[0]
    sod, ped = dev(so), dev(pe)
    x = WL.gen_matrix(W, P, 0.05, seed=77, ld=ld)
    v = WL.gen_matrix(W, P, 0.02, seed=77, ld=ld, stream=1)
    g = WL.gen_matrix(W, P, 0.01, seed=77, ld=ld, stream=2)
    w = (0.5 + np.random.default_rng(77).random(W)).astype(np.float32)
    x16, g16 = O.f32_to_f16(x), O.f32_to_f16(g)
    fx, fv = (once(t) for t in O.sgd_fused_mix_f64(x, v, g, LR, MU, WD, P, so, pe))
    hx, hv = (once(t) for t in O.hier_sgd_fused_mix_f64(x, v, g, LR, MU, WD, P, 1, so, pe))
    px, pw, pz = O.pushsum_mix_f32(x, w, P, W - 1, True)
    m16 = O.gossip_mix_f16(x16, P, so, pe)
    fx16, fv16 = O.sgd_fused_mix16("f16", x16, v, g16, LR, MU, WD, P, so, pe)
    px16, pw16, pz16 = O.pushsum_mix16("f16", x16, w, P, W - 1, True)
    assert same_bits(fx, hx) and same_bits(fv, hv)        # groups of one: the flat step
    for inplace in (False, True):
        xi, vi = dev(x), dev(v)
        xo, vo = (xi, vi) if inplace else (dev(x), dev(v))
        cx.cx_sgd_fused_mix(xi, xo, vi, vo, dev(g), LR, MU, WD, P, sod, ped)
        yi, ui = dev(x), dev(v)
        yo, uo = (yi, ui) if inplace else (dev(x), dev(v))
        cx.cx_hier_sgd_fused_mix(yi, yo, ui, uo, dev(g), LR, MU, WD, P, 1, sod, ped)
        pi, wi = dev(x), dev(w)
        po = pi if inplace else dev(x)
        wo, z = torch.zeros_like(wi), torch.zeros_like(pi)
        cx.cx_pushsum_mix(pi, po, wi, wo, z, P, W - 1)
        a16 = d16(x16)
        b16 = a16 if inplace else d16(x16)
        cx.cx_gossip_mix_f16(a16, b16, P, sod, ped)
        c16, cv = d16(x16), dev(v)
        e16, ev = (c16, cv) if inplace else (d16(x16), dev(v))
        cx.cx_sgd_fused_mix_f16(c16, e16, cv, ev, d16(g16), LR, MU, WD, P, sod, ped)
        q16 = d16(x16)
        r16 = q16 if inplace else d16(x16)
        wo16, z16 = torch.zeros_like(wi), d16(x16)
        cx.cx_pushsum_mix_f16(q16, r16, wi, wo16, z16, P, W - 1)
        torch.cuda.synchronize()
        assert same_bits(host(xo), fx) and same_bits(host(vo), fv), inplace
        assert same_bits(host(yo), hx) and same_bits(host(uo), hv), inplace
        assert same_bits(host(po), px) and same_bits(host(wo), pw) and same_bits(host(z)[:, :P], pz[:, :P]), inplace
        assert (h16(b16) == m16).all(), inplace
        assert (h16(e16) == fx16).all() and same_bits(host(ev), fv16), inplace
        assert (h16(r16) == px16).all() and same_bits(host(wo16), pw16), inplace
        assert (h16(z16)[:, :P] == pz16[:, :P]).all(), inplace
