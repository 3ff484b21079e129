"""CPU-only tests of the Python binding's argument checks.  The C ABI sees one leading dimension and
raw addresses, so a tensor of the wrong shape, stride, element type or device must be refused before
anything is launched: every case below raises ValueError on host tensors (the device check comes
last, so the other mismatches are reachable without a GPU), and the all-correct host case raises the
device error -- no call reaches the library."""
import pytest
import torch

from paper_2012_15198_amd import cxmix as cx

W, P, LD, S, G = 8, 60, 64, 3, 2


def mat(rows=W, ld=LD, dtype=torch.float32):
    return torch.zeros((rows, ld), dtype=dtype)


def tables(n=W, S=S):
    return torch.tensor([0, 20, 40, P], dtype=torch.int64)[:S + 1], torch.zeros((S, n), dtype=torch.int32)


def refuses(fn, *args, match):
    with pytest.raises(ValueError, match=match):
        fn(*args)


def test_correct_host_tensors_reach_only_the_device_check():
    so, pe = tables()
    refuses(cx.cx_gossip_mix, mat(), mat(), P, so, pe, match="device tensors")
    refuses(cx.cx_sgd_fused_mix, mat(), mat(), mat(), mat(), mat(), 0.1, 0.9, 1e-4, P, so, pe, match="device tensors")
    so2, pe2 = tables(W // G)
    refuses(cx.cx_hier_mix, mat(), mat(), P, G, so2, pe2, match="device tensors")
    refuses(cx.cx_hier_sgd_fused_mix, mat(), mat(), mat(W // G), mat(W // G), mat(), 0.1, 0.9, 1e-4, P, G, so2, pe2,
            match="device tensors")
    refuses(cx.cx_pushsum_mix, mat(), mat(), torch.ones(W), torch.ones(W), None, P, 1, match="device tensors")
    refuses(cx.cx_gossip_mix_bf16, mat(dtype=torch.bfloat16), mat(dtype=torch.bfloat16), P, so, pe, match="device tensors")
    refuses(cx.cx_copy_baseline, torch.zeros(64), torch.zeros(64), match="device tensors")


@pytest.mark.parametrize("bad,match", [
    (lambda: mat(ld=P), "row stride"),                           # unpadded next to a padded x_in
    (lambda: mat(rows=W - 1), "rows"),
    (lambda: mat(dtype=torch.float64), "float32"),
    (lambda: mat(dtype=torch.bfloat16), "float32"),
    (lambda: mat(dtype=torch.int32), "float32"),
    (lambda: mat(ld=2 * LD)[:, ::2], "row-major"),               # strided columns
    (lambda: torch.zeros(W * LD), "row-major"),                  # not a matrix
])
def test_every_matrix_argument_is_checked_against_x_in(bad, match):
    so, pe = tables()
    refuses(cx.cx_gossip_mix, mat(), bad(), P, so, pe, match=match)
    refuses(cx.cx_gossip_mix, bad(), mat(), P, so, pe, match=".")          # x_in itself or the mismatch of x_out
    for slot in range(1, 5):                                               # x_out, v_in, v_out, g
        args = [mat(), mat(), mat(), mat(), mat()]
        args[slot] = bad()
        refuses(cx.cx_sgd_fused_mix, *args, 0.1, 0.9, 1e-4, P, so, pe, match=match)
    so2, pe2 = tables(W // G)
    refuses(cx.cx_hier_mix, mat(), bad(), P, G, so2, pe2, match=match)
    refuses(cx.cx_pushsum_mix, mat(), bad(), torch.ones(W), torch.ones(W), None, P, 1, match=match)
    refuses(cx.cx_pushsum_mix, mat(), mat(), torch.ones(W), torch.ones(W), bad(), P, 1, match=match)


def test_hierarchical_gradient_step_checks_the_leader_momentum_shape():
    so, pe = tables(W // G)
    L = W // G
    ok = lambda: [mat(), mat(), mat(L), mat(L), mat()]
    for slot, bad, match in [(2, mat(W), "rows"), (3, mat(L, ld=P), "row stride"), (4, mat(L), "rows"),
                             (1, mat(dtype=torch.float16), "float32")]:
        args = ok()
        args[slot] = bad
        refuses(cx.cx_hier_sgd_fused_mix, *args, 0.1, 0.9, 1e-4, P, G, so, pe, match=match)
    refuses(cx.cx_hier_sgd_fused_mix, *ok(), 0.1, 0.9, 1e-4, P, 3, so, pe, match="divide")


def test_16bit_entry_points_refuse_other_element_sizes():
    so, pe = tables()
    b = lambda: mat(dtype=torch.bfloat16)
    refuses(cx.cx_gossip_mix_bf16, mat(), b(), P, so, pe, match="16-bit")
    refuses(cx.cx_gossip_mix_f16, b(), mat(), P, so, pe, match="16-bit")
    refuses(cx.cx_gossip_mix_bf16, b(), mat(ld=P, dtype=torch.bfloat16), P, so, pe, match="row stride")
    so2, pe2 = tables(W // G)
    refuses(cx.cx_hier_mix_bf16, b(), mat(), P, G, so2, pe2, match="16-bit")
    refuses(cx.cx_gossip_mix, b(), b(), P, so, pe, match="float32")
    refuses(cx.cx_pushsum_mix_bf16, b(), mat(), torch.ones(W), torch.ones(W), None, P, 1, match="16-bit")
    refuses(cx.cx_pushsum_mix_f16, b(), b(), torch.ones(W), torch.ones(W), mat(), P, 1, match="16-bit")
    refuses(cx.cx_pushsum_mix_bf16, b(), b(), torch.ones(W - 1), torch.ones(W), None, P, 1, match="w_in")
    refuses(cx.cx_pushsum_mix, b(), b(), torch.ones(W), torch.ones(W), None, P, 1, match="float32")


def test_tables_and_vectors_are_checked():
    so, pe = tables()
    refuses(cx.cx_gossip_mix, mat(), mat(), P, so.to(torch.int32), pe, match="seg_off_dev")
    refuses(cx.cx_gossip_mix, mat(), mat(), P, so, pe.to(torch.int64), match="peers_dev")
    refuses(cx.cx_gossip_mix, mat(), mat(), P, so, pe[:, :W - 1], match="peers_dev")
    refuses(cx.cx_gossip_mix, mat(), mat(), P, so, torch.zeros((S, W + 1), dtype=torch.int32), match="peers_dev")
    refuses(cx.cx_gossip_mix, mat(), mat(), P, so[:1], pe, match="seg_off_dev")
    refuses(cx.cx_gossip_mix, mat(), mat(), LD + 1, so, pe, match="P must")
    refuses(cx.cx_hier_mix, mat(), mat(), P, G, so, pe, match="peers_dev")          # table for W rows, not W/G
    refuses(cx.cx_pushsum_mix, mat(), mat(), torch.ones(W - 1), torch.ones(W), None, P, 1, match="w_in")
    refuses(cx.cx_pushsum_mix, mat(), mat(), torch.ones(W), torch.ones(W, dtype=torch.float64), None, P, 1, match="w_out")
    refuses(cx.cx_copy_baseline, torch.zeros(64), torch.zeros(32), match="dst")
