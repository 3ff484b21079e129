"""Pins for the oracle's optimizer steps on 16-bit rows (bfloat16 / binary16 parameters and
gradients, fp32 momentum): the double -> 16-bit rounding against an exact-rational nearest search
and numpy, the steps by hand, against the pinned fp32-row steps, and against a library optimizer.
CPU only."""
import bisect
from fractions import Fraction

import numpy as np
import pytest

import oracle as O
from paper_2012_15198_amd import workloads as WL

FMT = {"bf16": dict(keep=7, widen=O.bf16_to_f32, narrow=O.f64_to_bf16, inf=0x7F80),
       "f16": dict(keep=10, widen=O.f16_to_f32, narrow=O.f64_to_f16, inf=0x7C00)}


def finite_values(fmt):
    """Every non-negative finite value of the format as an exact Fraction, in pattern order
    (patterns of non-negative finite values ascend with the value)."""
    pats = np.arange(0, FMT[fmt]["inf"], dtype=np.uint16)
    return [Fraction(float(v)) for v in FMT[fmt]["widen"](pats)]


def nearest_by_search(fmt, vals, d):
    """Round-to-nearest-even by exact comparison with the two neighbouring values of the format."""
    f = FMT[fmt]
    if d != d:
        return None
    sign = 0x8000 if np.signbit(d) else 0
    if np.isinf(d):
        return sign | f["inf"]
    a = abs(Fraction(d))
    over = 2 * vals[-1] - vals[-2]               # the value the next pattern (infinity's) would stand for
    grid = vals + [over]
    hi = bisect.bisect_left(grid, a)
    if hi >= len(grid):
        return sign | f["inf"]
    if grid[hi] == a:
        return sign | hi
    lo = hi - 1
    if a - grid[lo] < grid[hi] - a:
        return sign | lo
    if a - grid[lo] > grid[hi] - a:
        return sign | hi
    return sign | (lo if lo % 2 == 0 else hi)    # tie: the even pattern


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_double_to_16bit_is_one_rounding_to_nearest_even(fmt):
    f = FMT[fmt]
    vals = finite_values(fmt)
    rng = np.random.default_rng(5)
    cases = []
    # random doubles over the whole range of the format and beyond both ends
    lo_exp, hi_exp = (-140, 130) if fmt == "bf16" else (-30, 18)
    cases += list(np.ldexp(rng.standard_normal(3000), rng.integers(lo_exp, hi_exp, 3000)))
    # every 97th value of the format, the exact midpoint to its successor, and doubles just beside it:
    # the midpoints are exact in fp32 too, so rounding through fp32 would tie where one rounding does not
    for k in list(range(0, len(vals) - 1, 97)) + [0, 1, 2, len(vals) - 2]:
        mid = float((vals[k] + vals[k + 1]) / 2)
        cases += [float(vals[k]), mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf)]
    top = float(vals[-1])
    cases += [top, float(2 * vals[-1] - vals[-2]), np.nextafter(float((3 * vals[-1] - vals[-2]) / 2), 0.0),
              float((3 * vals[-1] - vals[-2]) / 2), 1e300, 5e-324, 0.0, np.inf]
    cases = np.array(cases + [-c for c in cases], dtype=np.float64)
    got = f["narrow"](cases)
    want = [nearest_by_search(fmt, vals, float(d)) for d in cases]
    bad = [(float(d), hex(int(g)), hex(w)) for d, g, w in zip(cases, got, want) if int(g) != w]
    assert not bad, bad[:5]
    nan = int(f["narrow"]([np.nan])[0])
    assert (nan & f["inf"]) == f["inf"] and (nan & (0x7FFF ^ f["inf"])) != 0
    # widening and narrowing again is the identity on every finite pattern
    pats = np.arange(0, f["inf"], dtype=np.uint16)
    assert (f["narrow"](f["widen"](pats).astype(np.float64)) == pats).all()


def test_double_to_binary16_agrees_with_the_library_conversion():
    rng = np.random.default_rng(6)
    d = np.concatenate([np.ldexp(rng.standard_normal(20000), rng.integers(-30, 18, 20000)),
                        [65504.0, 65519.99, 65520.0, 2.0 ** -25, np.nextafter(2.0 ** -25, 1.0), 0.0, -0.0]])
    with np.errstate(over="ignore"):
        want = d.astype(np.float16).view(np.uint16)
    assert (O.f64_to_f16(d) == want).all()


def test_one_rounding_differs_from_rounding_through_fp32_where_it_must():
    # 1 + 2^-8 is exactly half way between two bfloat16 values; a little more must round up, but
    # fp32 cannot hold the little more, ties, and picks the even value below
    d = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert O.f64_to_bf16([d])[0] == 0x3F81
    assert O.f32_to_bf16(np.float32(d)) == 0x3F80
    d = 1.0 + 2.0 ** -11 + 2.0 ** -40
    assert O.f64_to_f16([d])[0] == 0x3C01 and O.f32_to_f16(np.float32(d)) == 0x3C00


def rows16(fmt, a):
    return (O.f32_to_bf16 if fmt == "bf16" else O.f32_to_f16)(np.asarray(a, dtype=np.float32))


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_fused16_hand_case(fmt):
    # two workers, one column; every input is exact in both formats
    x = rows16(fmt, [[1.0], [3.0]])
    g = rows16(fmt, [[0.5], [-1.0]])
    v = np.array([[2.0], [4.0]], dtype=np.float32)
    lr, mu, wd = 0.5, 0.5, 0.25
    # worker 0: g' = 0.5 + 0.25 = 0.75, v' = 1 + 0.75 = 1.75, h = 1 - 0.875 = 0.125
    # worker 1: g' = -1 + 0.75 = -0.25, v' = 2 - 0.25 = 1.75, h = 3 - 0.875 = 2.125; average 1.125
    x64, v64 = O.sgd_fused_mix16_f64(fmt, x, v, g, lr, mu, wd, 1, [0, 1], [[1, 0]])
    assert x64.ravel().tolist() == [1.125, 1.125] and v64.ravel().tolist() == [1.75, 1.75]
    xo, vo = O.sgd_fused_mix16(fmt, x, v, g, lr, mu, wd, 1, [0, 1], [[1, 0]])
    assert FMT[fmt]["widen"](xo).ravel().tolist() == [1.125, 1.125] and vo.ravel().tolist() == [1.75, 1.75]
    assert xo.dtype == np.uint16 and vo.dtype == np.float32


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_fused16_rounds_the_double_result_once_not_through_fp32(fmt):
    """A step whose exact result sits 2^-31 above the midpoint of two 16-bit values: one rounding goes
    up; rounding to fp32 first would land on the midpoint and then tie to the even value below."""
    ulp = 2.0 ** -FMT[fmt]["keep"]
    x = rows16(fmt, [[1.0], [1.0 + ulp]])
    g = rows16(fmt, [[-(2.0 ** -10)], [0.0]])
    v = np.zeros((2, 1), dtype=np.float32)
    lr = 2.0 ** -20                                   # h_0 = 1 + 2^-30, h_1 = 1 + ulp, average = 1 + ulp/2 + 2^-31
    x64, _ = O.sgd_fused_mix16_f64(fmt, x, v, g, lr, 0.0, 0.0, 1, [0, 1], [[1, 0]])
    assert x64.ravel().tolist() == [1.0 + ulp / 2 + 2.0 ** -31] * 2
    xo, _ = O.sgd_fused_mix16(fmt, x, v, g, lr, 0.0, 0.0, 1, [0, 1], [[1, 0]])
    one = int(rows16(fmt, [1.0])[0])
    assert xo.ravel().tolist() == [one + 1, one + 1]
    through_fp32 = rows16(fmt, x64.astype(np.float32))
    assert through_fp32.ravel().tolist() == [one, one]
    # the same for the hierarchical step (two groups of one leader and one member)
    x4, g4 = np.repeat(x, 2, 0), np.repeat(g, 2, 0)
    xo, _ = O.hier_sgd_fused_mix16(fmt, x4, v, g4, lr, 0.0, 0.0, 1, 2, [0, 1], [[1, 0]])
    assert xo.ravel().tolist() == [one + 1] * 4


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_fused16_is_the_pinned_fp32_row_step_on_widened_rows_rounded_once(fmt):
    """The 16-bit step == the double step on the exactly widened rows (oracle_sgd_fused_mix_f64, pinned
    by hand, by its library special case and by its invariants), followed by the pinned roundings."""
    W, P, S = 6, 90, 3
    f = FMT[fmt]
    x = rows16(fmt, WL.gen_matrix(W, P, 0.05, 21))
    g = rows16(fmt, WL.gen_matrix(W, P, 0.01, 21, stream=2))
    v = WL.gen_matrix(W, P, 0.02, 21, stream=1)
    so = WL.equal_seg_off(P, S)
    pe = O.topology(21, W, S, 0, 1)[0]
    x64, v64 = O.sgd_fused_mix_f64(f["widen"](x), v, f["widen"](g), 0.1, 0.9, 1e-4, P, so, pe)
    r64x, r64v = O.sgd_fused_mix16_f64(fmt, x, v, g, 0.1, 0.9, 1e-4, P, so, pe)
    assert (r64x == x64).all() and (r64v == v64).all()
    xo, vo = O.sgd_fused_mix16(fmt, x, v, g, 0.1, 0.9, 1e-4, P, so, pe)
    assert (xo == f["narrow"](x64)).all() and (vo == v64.astype(np.float32)).all()
    # within half a unit of the 16-bit format of the exact result
    err = np.abs(f["widen"](xo).astype(np.float64) - x64)
    assert (err <= np.abs(x64) * 2.0 ** -(f["keep"] + 1) + 2.0 ** -150).all()


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_fused16_without_mixing_is_a_library_momentum_sgd_step(fmt):
    """Peers that pair every row with an identical twin switch the averaging off: what is left is one
    step of torch.optim.SGD (momentum, weight decay) in double on the widened values."""
    import torch
    P = 50
    f = FMT[fmt]
    x1 = rows16(fmt, WL.gen_matrix(1, P, 0.05, 22))
    g1 = rows16(fmt, WL.gen_matrix(1, P, 0.01, 22, stream=2))
    v1 = WL.gen_matrix(1, P, 0.02, 22, stream=1)
    x, g, v = np.repeat(x1, 2, 0), np.repeat(g1, 2, 0), np.repeat(v1, 2, 0)
    lr, mu, wd = np.float32(0.1), np.float32(0.9), np.float32(1e-4)
    x64, v64 = O.sgd_fused_mix16_f64(fmt, x, v, g, lr, mu, wd, P, [0, P], [[1, 0]])
    p = torch.tensor(f["widen"](x1)[0].astype(np.float64), requires_grad=True)
    opt = torch.optim.SGD([p], lr=float(lr), momentum=float(mu), weight_decay=float(wd))
    opt.state[p]["momentum_buffer"] = torch.tensor(v1[0].astype(np.float64))
    p.grad = torch.tensor(f["widen"](g1)[0].astype(np.float64))
    opt.step()
    assert np.abs(x64[0] - p.detach().numpy()).max() < 1e-15
    assert np.abs(v64[0] - opt.state[p]["momentum_buffer"].numpy()).max() < 1e-15
    assert (x64[0] == x64[1]).all()


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_fused16_lr0_is_the_16bit_gossip_and_weight_decay_enters_v(fmt):
    W, P, S = 5, 64, 2
    f = FMT[fmt]
    x = rows16(fmt, WL.gen_matrix(W, P, 1.0, 23))
    g = rows16(fmt, WL.gen_matrix(W, P, 0.01, 23, stream=2))
    v = np.zeros((W, P), dtype=np.float32)
    so = WL.equal_seg_off(P, S)
    pe = O.topology(23, W, S, 0, 1)[0]
    xo, vo = O.sgd_fused_mix16(fmt, x, v, g, 0.0, 0.9, 0.5, P, so, pe)
    mix = O.gossip_mix_bf16 if fmt == "bf16" else O.gossip_mix_f16
    # where the fp32 sum of the pair is exact, one rounding of the exact average is what the 16-bit
    # gossip returns (it rounds the fp32 average)
    wx = f["widen"](x).astype(np.float64)
    exact = np.ones_like(wx, dtype=bool)
    for s in range(S):
        a, b = wx[:, so[s]:so[s + 1]], wx[pe[s], so[s]:so[s + 1]]
        exact[:, so[s]:so[s + 1]] = (a + b).astype(np.float32).astype(np.float64) == a + b
    assert exact.mean() > 0.9
    assert (xo[exact] == mix(x, P, so, pe)[exact]).all()
    assert (vo == (f["widen"](g).astype(np.float64) + 0.5 * wx).astype(np.float32)).all()


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_hier_fused16_special_cases(fmt):
    W, G, P, S = 8, 4, 40, 2
    L = W // G
    f = FMT[fmt]
    x = rows16(fmt, WL.gen_matrix(W, P, 0.05, 24))
    g = rows16(fmt, WL.gen_matrix(W, P, 0.01, 24, stream=2))
    v = WL.gen_matrix(L, P, 0.02, 24, stream=1)
    so = WL.equal_seg_off(P, S)
    pe = O.topology(24, L, S, 0, 1)[0]
    args = (0.1, 0.9, 1e-4, P)
    # == the pinned fp32-row step on the widened rows, then the pinned roundings
    x64, v64 = O.hier_sgd_fused_mix_f64(f["widen"](x), v, f["widen"](g), *args, G, so, pe)
    r64x, r64v = O.hier_sgd_fused_mix16_f64(fmt, x, v, g, *args, G, so, pe)
    assert (r64x == x64).all() and (r64v == v64).all()
    xo, vo = O.hier_sgd_fused_mix16(fmt, x, v, g, *args, G, so, pe)
    assert (xo == f["narrow"](x64)).all() and (vo == v64.astype(np.float32)).all()
    assert (xo.reshape(L, G, P) == xo.reshape(L, G, P)[:, :1]).all()          # broadcast to the group
    # groups of one: the flat step
    pw = O.topology(24, W, S, 0, 1)[0]
    vw = WL.gen_matrix(W, P, 0.02, 24, stream=1)
    a = O.hier_sgd_fused_mix16(fmt, x, vw, g, *args, 1, so, pw)
    b = O.sgd_fused_mix16(fmt, x, vw, g, *args, so, pw)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()
    # member rows of x are never read
    x2 = x.copy()
    x2[1::G] = rows16(fmt, np.full((L, P), 7.0))
    c = O.hier_sgd_fused_mix16(fmt, x2, v, g, *args, G, so, pe)
    assert (c[0] == xo).all() and (c[1] == vo).all()
    # one group: SGD on the mean gradient, no gossip
    one = O.hier_sgd_fused_mix16_f64(fmt, x, v[:1], g, *args, W, so, None)
    gbar = f["widen"](g).astype(np.float64).mean(0)
    xl = f["widen"](x)[0].astype(np.float64)
    vn = np.float32(0.9).astype(np.float64) * v[0] + (gbar + np.float32(1e-4).astype(np.float64) * xl)
    assert np.abs(one[1][0] - vn).max() < 1e-12
    assert np.abs(one[0] - (xl - np.float32(0.1).astype(np.float64) * vn)).max() < 1e-12


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_array_narrowing_and_the_once_rounded_hierarchical_step(fmt):
    f = FMT[fmt]
    rng = np.random.default_rng(31)
    d = np.ldexp(rng.standard_normal(5000), rng.integers(-30, 18, 5000))
    assert (O.narrow16(fmt, d) == f["narrow"](d)).all()                       # the array form is the scalar one
    W, G, P, S = 12, 4, 50, 3
    x = rows16(fmt, WL.gen_matrix(W, P, 0.05, 32))
    so = WL.equal_seg_off(P, S)
    pe = O.topology(32, W // G, S, 0, 1)[0]
    y64 = O.hier_mix16_f64(fmt, x, P, G, so, pe)                              # pinned in test_oracle_mix.py
    got = O.hier_mix16(fmt, x, P, G, so, pe)
    assert (got == f["narrow"](y64)).all()
    assert (got.reshape(W // G, G, P) == got.reshape(W // G, G, P)[:, :1]).all()
    # one rounding: a group whose exact mean sits 2^-31 above a tie goes up, where an fp32 sum would tie
    ulp = 2.0 ** -f["keep"]
    tie = rows16(fmt, [[1.0], [1.0 + ulp], [1.0], [1.0 + ulp]])              # mean 1 + ulp/2, exactly the tie
    assert O.hier_mix16(fmt, tie, 1, 4, [0, 1], None).ravel().tolist() == [int(rows16(fmt, [1.0])[0])] * 4
    up = rows16(fmt, [[1.0 + 2 * ulp], [1.0 + ulp], [1.0], [1.0 + ulp]])     # mean 1 + ulp: representable
    assert O.hier_mix16(fmt, up, 1, 4, [0, 1], None).ravel().tolist() == [int(rows16(fmt, [1.0 + ulp])[0])] * 4
