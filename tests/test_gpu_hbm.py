"""cx_hbm_alloc / cx_hbm_free on the GPU: the blocks are ordinary device memory for torch and for the
mixing calls, a mix on them gives the oracle's bits, and freeing gives the memory back.  (That such
blocks are FASTER to write is a measurement, reported by bench.py; here only correctness.)"""
import gc

import numpy as np
import pytest
import torch

import oracle as O
from paper_2012_15198_amd import cxmix as cx
from paper_2012_15198_amd import workloads as WL

pytestmark = pytest.mark.gpu
MiB = 1 << 20


def test_blocks_are_usable_device_memory_and_are_given_back():
    cx.cx_copy_baseline(torch.zeros(1024, device="cuda:0"), torch.zeros(1024, device="cuda:0"))   # runtime and library set up
    gc.collect()                                       # graphs and streams of earlier tests give their memory back now,
    torch.cuda.empty_cache()                           # not between the two readings below
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    sizes = [300 * MiB + 12345, 70 * MiB, 1]           # several pieces + a ragged tail; under one piece; one byte
    ptrs = cx.cx_hbm_alloc(sizes)
    try:
        assert len(set(ptrs)) == 3 and all(p and p % (2 * MiB) == 0 for p in ptrs)
        held = free0 - torch.cuda.mem_get_info()[0]
        rounded = sum((s + 2 * MiB - 1) // (2 * MiB) * (2 * MiB) for s in sizes)
        # the fillers are gone again; slack for page tables above, for what the runtime frees lazily below
        assert rounded - 64 * MiB <= held <= rounded + 256 * MiB
        with pytest.raises(cx.CxError, match="CX_ERR_UNSUPPORTED"):
            cx.cx_hbm_free(ptrs[0] + 2 * MiB)              # inside a block, not its start
    finally:
        for p in ptrs:
            cx.cx_hbm_free(p)
    with pytest.raises(cx.CxError, match="CX_ERR_UNSUPPORTED"):
        cx.cx_hbm_free(ptrs[0])                            # already released
    assert abs(torch.cuda.mem_get_info()[0] - free0) <= 256 * MiB
    with pytest.raises(cx.CxError, match="CX_ERR_MEMORY"):
        cx.cx_hbm_alloc([torch.cuda.mem_get_info()[1] + MiB])


def test_mix_on_placed_tensors_matches_the_oracle_and_plain_tensors():
    """Every entry point family once on tensors from hbm_empty: rows that cross the 256 MiB pieces
    (ld chosen so that piece boundaries fall inside rows), float32 and 16-bit, out of place and in place."""
    W, P, S = 8, 20 * MiB + 8 * 1031, 5                  # 80 MiB rows: a piece boundary inside rows 3 and 6
    ld = P + 8
    x_host = WL.gen_matrix(W, P, 1.0, 11)
    so = np.array([0, 5, 5, 7 * MiB + 3, 13 * MiB + 2, P], dtype=np.int64)
    peers = cx.cx_topology_gen(3, W, S, 0, 1)[0]
    want = O.gossip_mix(x_host, P, so, peers)
    x, y, x16, y16 = cx.hbm_empty([(W, ld)] * 4, [torch.float32, torch.float32, torch.bfloat16, torch.bfloat16])
    assert x.dtype == torch.float32 and x16.dtype == torch.bfloat16 and x.shape == (W, ld)
    x[:, :P].copy_(torch.from_numpy(x_host)); x[:, P:] = 7.0
    y.fill_(-1.0)
    so_d, peers_d = torch.from_numpy(so).cuda(), torch.from_numpy(peers).cuda()
    cx.cx_gossip_mix(x, y, P, so_d, peers_d)
    got = y[:, :P].cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert bool((y[:, P:] == -1.0).all())                # padding columns untouched
    plain_x, plain_y = x.clone(), torch.empty_like(x)    # torch's own allocation
    cx.cx_gossip_mix(plain_x, plain_y, P, so_d, peers_d)
    assert torch.equal(plain_y[:, :P], y[:, :P])
    cx.cx_gossip_mix(x, x, P, so_d, peers_d)             # in place on a placed block
    assert torch.equal(x[:, :P], y[:, :P])
    # 16-bit rows
    x16[:, :P].copy_(torch.from_numpy(x_host)); x16[:, P:] = 0
    cx.cx_gossip_mix_bf16(x16, y16, P, so_d, peers_d)
    want16 = O.gossip_mix_bf16(np.ascontiguousarray(x16[:, :P].view(torch.int16).cpu().numpy().view(np.uint16)), P, so, peers)
    assert np.array_equal(y16[:, :P].view(torch.int16).cpu().numpy().view(np.uint16), want16)
    # views keep the block alive; dropping the last one releases it
    free_before = torch.cuda.mem_get_info()[0]
    row = x[3]
    del x, y, x16, y16, plain_x, plain_y
    gc.collect()
    assert float(row[:5].sum()) == float(row[:5].sum())  # still mapped
    del row
    gc.collect()
    assert torch.cuda.mem_get_info()[0] >= free_before + 4 * W * ld * 2 - 64 * MiB


def test_placement_on_a_nearly_full_device():
    """Most of the memory held by somebody else (torch): the call still serves what fits -- with little or
    nothing left to skip -- says CX_ERR_MEMORY for what does not, and gives everything back."""
    gc.collect()
    torch.cuda.empty_cache()
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    keep = 24 << 30
    if free0 < keep + (8 << 30):
        pytest.skip("not enough free memory to stage the case")
    hog = torch.empty(free0 - keep, dtype=torch.uint8, device="cuda:0")
    try:
        free1 = torch.cuda.mem_get_info()[0]
        assert free1 <= keep + (1 << 30)
        with pytest.raises(cx.CxError, match="CX_ERR_MEMORY"):
            cx.cx_hbm_alloc([free1 + (64 << 20)])
        assert abs(torch.cuda.mem_get_info()[0] - free1) <= 64 * MiB          # nothing kept after the refusal
        a, b = cx.hbm_empty([(4, 1 << 28), (4, 1 << 28)])                       # 2 x 4 GiB of float32
        a.fill_(1.0)
        b.fill_(3.0)
        assert float(a.min()) == 1.0 and float(a.max()) == 1.0 and float(b.min()) == 3.0 and float(b.max()) == 3.0
        del a, b
        gc.collect()
        torch.cuda.empty_cache()
        assert abs(torch.cuda.mem_get_info()[0] - free1) <= 256 * MiB
    finally:
        del hog
        torch.cuda.empty_cache()
