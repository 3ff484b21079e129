"""GPU parity of the push-sum comparison on 16-bit rows (cx_pushsum_mix_bf16 / _f16) against the oracle,
through the C ABI: x' and z bit for bit in the 16-bit format (any NaN equals any NaN), w' bit for bit in
fp32; all launch shapes; the exponential graph reaching the mean; every pattern of the format once."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2012_15198_amd import cxmix as cx
from paper_2012_15198_amd import workloads as WL
from gpu_util import ALL_TUNINGS, Tuning, dev, host, same_bits

pytestmark = pytest.mark.gpu

NARROW = {"bf16": O.f32_to_bf16, "f16": O.f32_to_f16}
WIDEN = {"bf16": O.bf16_to_f32, "f16": O.f16_to_f32}
PUSH = {"bf16": cx.cx_pushsum_mix_bf16, "f16": cx.cx_pushsum_mix_f16}
NAN = {"bf16": (0x7F80, 0x007F), "f16": (0x7C00, 0x03FF)}
HALF_ULP = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11}


def same16(fmt, a, b):
    e, m = NAN[fmt]
    isnan = lambda h: ((h & e) == e) & ((h & m) != 0)
    a, b = np.asarray(a, dtype=np.uint16), np.asarray(b, dtype=np.uint16)
    return bool(((a == b) | (isnan(a) & isnan(b))).all())


def d16(a):
    return dev(np.ascontiguousarray(a).view(np.int16))


def h16(t):
    return host(t).view(np.uint16)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
@pytest.mark.parametrize("W,P,ld,hop", [(2, 5, 8, 1), (8, 5003, 5008, 1), (8, 5003, 5008, 4), (6, 3000, 3000, 4),
                                        (128, 1100, 1104, 64), (13, 8195, 8320, 8)])
@pytest.mark.parametrize("inplace", [False, True])
@pytest.mark.parametrize("want_z", [False, True])
def test_pushsum16_bit_exact(fmt, W, P, ld, hop, inplace, want_z):
    x = NARROW[fmt](WL.gen_matrix(W, P, 0.05, seed=61 + W, ld=ld))
    w = (1.0 + 0.5 * np.random.default_rng(61).random(W)).astype(np.float32)
    xd, wd = d16(x), dev(w)
    xo = xd if inplace else xd.clone()
    wo = torch.zeros_like(wd)
    z = torch.full_like(xd, 0x1234) if want_z else None
    PUSH[fmt](xd, xo, wd, wo, z, P, hop)
    torch.cuda.synchronize()
    wx, ww, wz = O.pushsum_mix16(fmt, x, w, P, hop, want_z)
    assert same16(fmt, h16(xo), wx) and same_bits(host(wo), ww)
    if not inplace:
        assert (h16(xd) == x).all()
    if want_z:
        gz = h16(z)
        assert same16(fmt, gz[:, :P], wz[:, :P]) and (gz[:, P:] == 0x1234).all()
    # and within half a unit in the last place (+ the fp32 step) of the double reference
    x64, _, z64 = O.pushsum_mix16_f64(fmt, x, w, P, hop, want_z)
    for got, ref in ((h16(xo), x64), (h16(z), z64) if want_z else (None, None)):
        if got is None:
            continue
        val = WIDEN[fmt](got[:, :P]).astype(np.float64)
        assert (np.abs(val - ref[:, :P]) <= np.abs(ref[:, :P]) * (HALF_ULP[fmt] + 2.0 ** -22) + 2.0 ** -25).all()


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_pushsum16_every_launch_shape(fmt):
    W, P, ld, hop = 16, 12301, 12416, 5
    x = NARROW[fmt](WL.gen_matrix(W, P, 1.0, seed=62, ld=ld))
    w = (0.5 + np.random.default_rng(62).random(W)).astype(np.float32)
    wx, ww, wz = O.pushsum_mix16(fmt, x, w, P, hop)
    for tuning in ALL_TUNINGS:
        with Tuning(*tuning):
            for inplace in (False, True):
                xd, wd = d16(x), dev(w)
                xo = xd if inplace else torch.zeros_like(xd)
                if not inplace:
                    xo[:, P:] = xd[:, P:]
                wo, z = torch.zeros_like(wd), torch.zeros_like(xd)
                PUSH[fmt](xd, xo, wd, wo, z, P, hop)
                torch.cuda.synchronize()
                assert same16(fmt, h16(xo)[:, :P], wx[:, :P]), (tuning, inplace)
                assert same16(fmt, h16(z)[:, :P], wz[:, :P]) and same_bits(host(wo), ww), (tuning, inplace)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_pushsum16_exponential_graph_reaches_the_mean(fmt):
    """W = 64, hops 1 .. 32 in place: multiples of 64 below 2^7 * 64 stay exact in both formats, so after six
    rounds every row is the exact mean and every weight is one."""
    W, P = 64, 4104
    rng = np.random.default_rng(63)
    x = (rng.integers(0, 4, size=(W, P)) * 64).astype(np.float32)
    xd = d16(NARROW[fmt](x))
    w0, w1 = torch.ones(W, device=xd.device), torch.zeros(W, device=xd.device)
    for k in range(6):
        PUSH[fmt](xd, xd, w0, w1, None, P, 2 ** k)
        w0, w1 = w1, w0
    torch.cuda.synchronize()
    assert (host(w0) == 1.0).all()
    assert np.array_equal(WIDEN[fmt](h16(xd)), np.tile(x.mean(axis=0, dtype=np.float64).astype(np.float32), (W, 1)))


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_pushsum16_every_pattern_of_the_format(fmt):
    """Row 0 holds all 65,536 patterns, row 1 a few partners in turn: x' and z for every pattern (zeros, subnormals,
    infinities, NaNs) equal the oracle's."""
    P = 65536
    pats = np.arange(P, dtype=np.uint16)
    w = np.array([1.5, 0.75], dtype=np.float32)
    for partner in (0x0000, 0x3F80 if fmt == "bf16" else 0x3C00, 0x8001, 0x7F7F if fmt == "bf16" else 0x7BFF):
        x = np.stack([pats, np.full(P, partner, dtype=np.uint16)])
        xd, wd = d16(x), dev(w)
        xo, wo, z = torch.zeros_like(xd), torch.zeros_like(wd), torch.zeros_like(xd)
        PUSH[fmt](xd, xo, wd, wo, z, P, 1)
        torch.cuda.synchronize()
        wx, ww, wz = O.pushsum_mix16(fmt, x, w, P, 1)
        assert same16(fmt, h16(xo), wx) and same16(fmt, h16(z), wz) and same_bits(host(wo), ww), hex(partner)


def test_pushsum16_argument_errors_on_a_gpu():
    x = torch.zeros((4, 16), dtype=torch.int16, device="cuda:0")
    w = torch.ones(4, device="cuda:0")
    with pytest.raises(cx.CxError, match="CX_ERR_SHAPE"):
        cx.cx_pushsum_mix_bf16(x, x.clone(), w, w.clone(), None, 16, 4)
    with pytest.raises(cx.CxError, match="CX_ERR_ALIAS"):
        cx.cx_pushsum_mix_bf16(x, x.clone(), w, w, None, 16, 1)
    with pytest.raises(cx.CxError, match="CX_ERR_ALIAS"):
        cx.cx_pushsum_mix_f16(x, x.clone(), w, w.clone(), x, 16, 1)
    with pytest.raises(ValueError):
        cx.cx_pushsum_mix_f16(x, x.clone().float(), w, w.clone(), None, 16, 1)
