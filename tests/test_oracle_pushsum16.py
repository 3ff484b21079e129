"""Pins for the oracle's push-sum round on 16-bit rows (bfloat16 / binary16 parameters, fp32 weights):
by hand on exactly representable values, the push-sum invariants, convergence of the directed exponential
graph to the global mean, the rounding against the double reference, and against the pinned fp32-row round
combined with the pinned conversions.  CPU only."""
import numpy as np
import pytest

import oracle as O

CONV = {"bf16": (O.f32_to_bf16, O.bf16_to_f32, 2.0 ** -8), "f16": (O.f32_to_f16, O.f16_to_f32, 2.0 ** -11)}


def random_rows(fmt, W, P, seed, scale=1.0):
    rng = np.random.default_rng([seed, 16])
    return CONV[fmt][0]((rng.standard_normal((W, P)) * scale).astype(np.float32))


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_by_hand_on_values_every_step_keeps_exact(fmt):
    """Small integers and weights that are powers of two: no step rounds, so the round is plain arithmetic.
    Row i receives from row (i - hop) mod W -- checked with rows that are all different."""
    to16, to32, _ = CONV[fmt]
    W, P, hop = 5, 7, 2
    x = np.array([[8 * (i + 1) + 16 * c for c in range(P)] for i in range(W)], dtype=np.float32)
    w = np.array([1.0, 2.0, 0.5, 4.0, 1.0], dtype=np.float32)
    xo, wo, zo = O.pushsum_mix16(fmt, to16(x), w, P, hop)
    for i in range(W):
        j = (i - hop) % W
        assert np.array_equal(to32(xo[i]), (x[i] + x[j]) / 2), (i, j)
        assert wo[i] == (w[i] + w[j]) / 2
    # de-biased values: chosen so that the quotient is representable (row 0: wn = (1 + 4) / 2 is not a power of two,
    # so take the rows whose new weight is one)
    for i in range(W):
        j = (i - hop) % W
        wn = (w[i] + w[j]) / 2
        if wn in (0.5, 1.0, 2.0):
            assert np.array_equal(to32(zo[i]), (x[i] + x[j]) / 2 / wn), i
    # without z the first two results are the same and the third is absent
    xo2, wo2, zo2 = O.pushsum_mix16(fmt, to16(x), w, P, hop, want_z=False)
    assert zo2 is None and np.array_equal(xo2, xo) and np.array_equal(wo2, wo)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_push_sum_invariants_in_the_double_reference(fmt):
    """Column sums of x and the sum of the weights are conserved by a round (column-stochastic mixing), and
    z * w' gives x' back."""
    W, P = 12, 257
    x = random_rows(fmt, W, P, 3)
    w = np.random.default_rng(5).uniform(0.25, 2.0, W).astype(np.float32)
    wide = CONV[fmt][1](x).astype(np.float64)
    for hop in (1, 4, 11):
        xo, wo, zo = O.pushsum_mix16_f64(fmt, x, w, P, hop)
        assert np.allclose(xo.sum(axis=0), wide.sum(axis=0), rtol=0, atol=1e-12)
        assert abs(wo.sum() - w.astype(np.float64).sum()) < 1e-12
        assert np.allclose(zo * wo[:, None], xo, rtol=1e-15, atol=0)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_directed_exponential_graph_reaches_the_global_mean(fmt):
    """W = 8 rows, hops 1, 2, 4 (the SGP graph the comparison uses): after log2 W rounds every row holds the mean of
    the start rows.  Values are multiples of 8 below 2^7, so all three rounds stay exact in both formats."""
    to16, to32, _ = CONV[fmt]
    W, P = 8, 33
    rng = np.random.default_rng(11)
    x = (rng.integers(0, 16, size=(W, P)) * 8).astype(np.float32)
    pat, w = to16(x), np.ones(W, dtype=np.float32)
    for hop in (1, 2, 4):
        pat, w, z = O.pushsum_mix16(fmt, pat, w, P, hop)
    assert np.array_equal(to32(pat), np.tile(x.mean(axis=0), (W, 1)))
    assert np.array_equal(w, np.ones(W, dtype=np.float32)) and np.array_equal(z, pat)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_rounding_against_the_double_reference(fmt):
    """x' and z are the double results rounded to the format: equal to the once-rounded double almost everywhere
    (the fp32 average and quotient in between can move a result across a tie: one unit in the last place at most),
    and within half a unit in the last place (+ the fp32 step's 2^-24) of the double result everywhere."""
    to16, to32, half_ulp = CONV[fmt]
    W, P, hop = 16, 4099, 5
    x = random_rows(fmt, W, P, 9)
    w = np.random.default_rng(2).uniform(0.3, 1.7, W).astype(np.float32)
    xo, wo, zo = O.pushsum_mix16(fmt, x, w, P, hop)
    xr, wr, zr = O.pushsum_mix16_f64(fmt, x, w, P, hop)
    assert np.array_equal(wo, wr.astype(np.float32))
    for got, ref in ((xo, xr), (zo, zr)):
        once = O.narrow16(fmt, ref)
        differ = got != once
        assert differ.mean() < 2e-3
        assert np.all(np.abs(got.astype(np.int32) - once.astype(np.int32))[differ] == 1)
        val = to32(got).astype(np.float64)
        ok = np.abs(val - ref) <= np.abs(ref) * (half_ulp + 2.0 ** -22) + 1e-30
        if fmt == "f16":
            ok |= np.abs(val - ref) <= 2.0 ** -25          # binary16 subnormals: absolute spacing 2^-24
        assert ok.all()


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
@pytest.mark.parametrize("hop", [1, 3, 6])
def test_equals_the_fp32_row_round_between_the_pinned_conversions(fmt, hop):
    """Widen with the pinned conversion, run the pinned fp32-row round, narrow with the pinned conversion: the 16-bit
    round must give exactly that, for x', w' and z (edge values included: zeros of both signs, subnormals, infinities)."""
    to16, to32, _ = CONV[fmt]
    W, P = 7, 1031
    x = random_rows(fmt, W, P, 21 + hop, scale=3.0)
    x[0, :6] = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x7BFF if fmt == "f16" else 0x7F7F, 0x7C00 if fmt == "f16" else 0x7F80], dtype=np.uint16)
    w = np.random.default_rng(hop).uniform(0.2, 3.0, W).astype(np.float32)
    x32 = to32(x)
    xf, wf, zf = O.pushsum_mix_f32(x32, w, P, hop)
    xo, wo, zo = O.pushsum_mix16(fmt, x, w, P, hop)
    assert np.array_equal(xo, to16(xf)) and np.array_equal(wo, wf) and np.array_equal(zo, to16(zf))


def test_padding_columns_and_argument_checks():
    x = random_rows("bf16", 4, 10, 1)
    xo, wo, zo = O.pushsum_mix16("bf16", x, np.ones(4, np.float32), 6, 1)
    assert np.array_equal(xo[:, 6:], x[:, 6:]) and np.array_equal(zo[:, 6:], x[:, 6:])
    with pytest.raises(ValueError):
        O.pushsum_mix16("bf16", x, np.ones(4, np.float32), 6, 4)
    with pytest.raises(KeyError):
        O.pushsum_mix16("fp8", x, np.ones(4, np.float32), 6, 1)
