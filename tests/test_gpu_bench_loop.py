"""The loop that bench.py times, checked against the oracle: bench.Runner as the benchmark builds it
(matrices from the placement call, rows padded to 4 KB, per round one host topology draw, one table
upload and one mixing call, buffers swapped) is stepped for several rounds at the full workload size,
and the result is compared on the column sample -- exact, since mixing is independent per column --
with the oracle driven by its own topology.  What is timed is therefore what is correct."""
import numpy as np
import pytest
import torch

import bench
import oracle as O
from paper_2012_15198_amd import workloads as WL
from gpu_util import dev, host, once, same_bits

pytestmark = pytest.mark.gpu

ROUNDS = 6


def grab(t, cold):
    """Sampled columns of a device matrix on the host: float32 as it is, 16-bit rows as bit patterns."""
    if t.dtype == torch.float32:
        return host(t.index_select(1, cold))
    return host(t.view(torch.int16).index_select(1, cold)).view(np.uint16)


@pytest.mark.parametrize("name,kind,rows16", [("C2", "gossip", None), ("C2", "gossip", "bf16"), ("C3", "hier", None),
                                              ("C3", "hiersgd", "bf16"), ("C4", "fused", None),
                                              ("C4", "pushsum", None), ("C4", "pushsum", "f16"), ("C5", "hier", None)])
def test_the_timed_loop_gives_the_oracles_results(name, kind, rows16):
    wl = WL.WORKLOADS[name]
    print(f"{name} {kind} {rows16 or 'fp32'}", flush=True)
    r = bench.Runner(wl, kind, ROUNDS, rows16=rows16)
    print(f"matrices from: {r.allocator}", flush=True)
    so = r.so_host if kind != "pushsum" else np.array([0, wl.P], dtype=np.int64)
    cols = WL.sample_columns(wl.P, so, wl.seed)
    sso, cold, n = WL.sub_seg_off(cols, so), dev(cols), len(cols)
    sx = grab(r.x, cold)
    if kind in ("fused", "hiersgd"):
        sv, sg = grab(r.v, cold), grab(r.g, cold)
        lr, mu, wd = (wl.lr, wl.mu, wl.wd) if kind == "fused" else (r.lr, r.mu, r.wd)
    sw = np.ones(wl.W, dtype=np.float32)
    for k in range(ROUNDS):
        r.step(False)
        tab = O.topology(wl.seed, r.n, r.S, k, 1, r.mode)[0]
        assert (r.tab_np[k] == tab).all(), k             # the table the loop drew and uploaded is the oracle's
        if kind == "gossip":
            mix = {None: O.gossip_mix, "bf16": O.gossip_mix_bf16, "f16": O.gossip_mix_f16}[rows16]
            sx = mix(sx, n, sso, tab)
        elif kind == "hier":
            sx = once(O.hier_mix_f64(sx, n, wl.G, sso, tab))
        elif kind == "fused":
            sx, sv = (once(t) for t in O.sgd_fused_mix_f64(sx, sv, sg, lr, mu, wd, n, sso, tab))
        elif kind == "hiersgd":
            sx, sv = O.hier_sgd_fused_mix16(rows16, sx, sv, sg, lr, mu, wd, n, wl.G, sso, tab)
        elif kind == "pushsum":
            hop = int((0 - int(tab[0, 0])) % wl.W)
            assert hop == 2 ** (k % 7)                   # W = 128: the exponential graph's hops
            if rows16:
                sx, sw, _ = O.pushsum_mix16(rows16, sx, sw, n, hop, False)
            else:
                sx, sw, _ = O.pushsum_mix_f32(sx, sw, n, hop, False)
    torch.cuda.synchronize()
    got = grab(r.x, cold)                                # after the swap r.x is the round's output
    if rows16:
        assert (got == sx).all()
    else:
        assert same_bits(got, sx)
    if kind in ("fused", "hiersgd"):
        assert same_bits(grab(r.v, cold), sv)
    if kind == "pushsum":
        assert same_bits(host(r.w[ROUNDS & 1]), sw)
    del r
    torch.cuda.empty_cache()
