"""The allocation-free accept entry point (metasd_accept_logits_noalloc: scratch in an array built into the library)
against metasd_accept_logits on the same inputs: same kernel, so every output is equal bit for bit.  Two calls in a
row on the shared array, the second with a smaller input; then the first shape again; sizes beyond the array are refused."""
import pytest
import torch

import paper_2604_05417_amd as M
import workloads as W

pytestmark = pytest.mark.gpu


def outputs(rows, gamma):
    return dict(n_acc=torch.full((rows,), -7, dtype=torch.int32, device="cuda"), token=torch.full((rows,), -7, dtype=torch.int32, device="cuda"),
                mask=torch.full((rows,), -7, dtype=torch.int32, device="cuda"), bd=torch.full((rows, gamma), -7.0, dtype=torch.float64, device="cuda"))


def case(rows, gamma, vocab, T, variant):
    c = W.config2(1.0, rows=rows, gamma=gamma, vocab=vocab, device="cuda", variant=variant)
    d = torch.stack([M.sample_logits(c["Q"][:, j].contiguous(), max(T, 1.0), c["seed"], variant, j, 0) for j in range(gamma)], 1).contiguous()
    return c["P"], c["Q"], d


@pytest.mark.parametrize("T", [1.0, 0.7, 0.0])
def test_noalloc_accept_equals_accept_logits_two_calls_in_a_row(T):
    shapes = [(64, 5, 32000, 0), (7, 3, 1040, 1), (64, 5, 32000, 2)]       # large, smaller, large again: the array keeps old contents
    for rows, gamma, vocab, variant in shapes:
        P, Q, d = case(rows, gamma, vocab, T, variant)
        ref = M.accept_logits(P, Q, d, T, 1, rnd=variant, seq0=3)
        got = M.accept_logits_noalloc(P, Q, d, T, 1, variant, 3, outputs(rows, gamma))
        torch.cuda.synchronize()
        assert (ref["token"] >= 0).all()
        for key in ("n_acc", "token", "mask"):
            assert torch.equal(got[key], ref[key]), (key, rows)
        assert torch.equal(got["bd"], ref["bd"])
    # back to back on one stream without a synchronisation in between: the second call's clearing kernel runs after the first call's kernels
    P1, Q1, d1 = case(64, 5, 32000, T, 0)
    P2, Q2, d2 = case(7, 3, 1040, T, 1)
    o1, o2 = outputs(64, 5), outputs(7, 3)
    M.accept_logits_noalloc(P1, Q1, d1, T, 1, 0, 3, o1)
    M.accept_logits_noalloc(P2, Q2, d2, T, 1, 1, 3, o2)
    torch.cuda.synchronize()
    r1, r2 = M.accept_logits(P1, Q1, d1, T, 1, rnd=0, seq0=3), M.accept_logits(P2, Q2, d2, T, 1, rnd=1, seq0=3)
    torch.cuda.synchronize()
    for key in ("n_acc", "token", "mask", "bd"):
        assert torch.equal(o1[key], r1[key]) and torch.equal(o2[key], r2[key]), key


def test_noalloc_accept_refuses_sizes_beyond_its_array():
    rows, gamma = M.ACCEPT_NOALLOC_MAX_ITEMS // 4 + 1, 3                # rows * (gamma + 1) = maximum + 4
    P = torch.zeros((rows, gamma + 1, 16), device="cuda")
    Q = torch.zeros((rows, gamma, 16), device="cuda")
    d = torch.zeros((rows, gamma), dtype=torch.int32, device="cuda")
    with pytest.raises(M.MetaSDError) as e:
        M.accept_logits_noalloc(P, Q, d, 1.0, 1, 0, 0, outputs(rows, gamma))
    assert e.value.code == -1 and "exceeds" in str(e.value)
    rows = M.ACCEPT_NOALLOC_MAX_ITEMS // 4                              # exactly the maximum: accepted
    out = M.accept_logits_noalloc(P[:rows].contiguous(), Q[:rows].contiguous(), d[:rows].contiguous(), 1.0, 1, 0, 0, outputs(rows, gamma))
    torch.cuda.synchronize()
    assert ((out["token"] >= 0) & (out["token"] < 16)).all()
