"""The entry point that allocates nothing (cx_gossip_mix_noalloc: scratch in a static device
array) against the ordinary entry point, through the C ABI: bit-identical outputs on two calls in
a row, the second on a smaller input, so the table still holds the first call's words."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2012_15198_amd import cxmix as cx
from paper_2012_15198_amd import workloads as WL
from gpu_util import dev, host, same_bits



def one_call(W, P, S, seed, rnd):
    ld = (P + 1023) // 1024 * 1024
    so = WL.equal_seg_off(P, S)
    x = WL.gen_matrix_device(W, P, 0.05, seed, ld=ld)
    tab = cx.cx_topology_gen(seed, W, S, rnd, 1)[0]
    cx.cx_check_peers(tab)
    want = torch.full_like(x, float("nan"))
    got = torch.full_like(x, float("nan"))
    sod, td = dev(so), dev(tab)
    cx.cx_gossip_mix(x, want, P, sod, td)
    mem_before = torch.cuda.memory_allocated()
    cx.cx_gossip_mix_noalloc(x, got, P, sod, td)
    assert torch.cuda.memory_allocated() == mem_before
    torch.cuda.synchronize()
    assert torch.equal(got[:, :P].view(torch.int32), want[:, :P].view(torch.int32))
    assert torch.isnan(got[:, P:]).all()                      # padding never written
    return x, got, so, tab


@pytest.mark.gpu
def test_noalloc_entry_point_matches_the_ordinary_one_twice_in_a_row():
    # first call: 49 clusters of 64 rows each; second call: a smaller matrix with fewer rows, so
    # most of the table still holds the first call's entries
    x, got, so, tab = one_call(64, 3_000_017, 8, seed=11, rnd=0)
    del x, got
    x, got, so, tab = one_call(6, 200_003, 3, seed=12, rnd=1)
    # and the small result against the oracle itself
    assert same_bits(host(got)[:, :200_003], O.gossip_mix(host(x), 200_003, so, tab)[:, :200_003])


@pytest.mark.gpu
def test_noalloc_entry_point_rejects_what_its_table_cannot_hold_and_in_place():
    L = cx.lib()
    a = torch.zeros((4, 64), device="cuda:0")
    so, tab = dev(np.array([0, 64], dtype=np.int64)), dev(np.array([[1, 0, 3, 2]], dtype=np.int32))
    with pytest.raises(cx.CxError) as e:
        cx.cx_gossip_mix_noalloc(a, a, 64, so, tab)
    assert e.value.status == -6
    # W = 1024 rows of 20 M columns need more than CX_NOALLOC_ORDER_WORDS: refused on the host,
    # before anything is enqueued (the pointers are never dereferenced)
    rc = L.cx_gossip_mix_noalloc(a.data_ptr(), a.data_ptr() + (1 << 40), 20_000_000, 1024, 20_000_000, 1,
                                 so.data_ptr(), tab.data_ptr(), 0, None)
    assert rc == -2


def test_noalloc_limits_are_checked_on_the_host():
    """No GPU needed: the size limit and the in-place refusal are host arithmetic on the arguments.
    Only refused calls are made here, so the made-up addresses are never handed to a kernel."""
    L = cx.lib()
    words = 1 << 18                                           # CX_NOALLOC_ORDER_WORDS
    A, B = 1 << 20, 1 << 44
    call = lambda W, P, out=B: L.cx_gossip_mix_noalloc(A, out, (P + 3) // 4 * 4, W, P, 1, A, A, 0, None)
    assert call(4, 64, out=A) == -6                           # in place
    for W in (128, 1024):
        limit_chunks = 64 * (words // W - 8)                  # the rule the header states
        assert call(W, (limit_chunks + 1) * 1024) == -2       # one chunk of 1024 columns too many
        assert call(W, 64 * (words // W) * 1024) == -2        # and well beyond it
