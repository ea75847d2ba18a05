"""GPU parity of the accept / sampling kernels against the oracle on seeded logits (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_05417_amd as M
import workloads as W

pytestmark = pytest.mark.gpu
RATIO_TIE, CDF_TIE = 1e-3, 1e-6


def oracle_uniforms(seed, rows, gamma, rnd, seq0=0):
    ua = np.stack([oracle.uniform_batch(seed, seq0, rows, rnd, j, 0) for j in range(gamma)], 1)
    ur = oracle.uniform_batch(seed, seq0, rows, rnd, 0, 1)
    return ua, ur


def check_accept(P, Q, T, seed, rnd, seq0=0):
    rows, gamma, V = Q.shape
    Ph, Qh = P.cpu().numpy(), Q.cpu().numpy()
    # draft tokens: drawn from q by the GPU sampler and checked against the oracle's draw
    d_gpu = torch.stack([M.sample_logits(Q[:, j].contiguous(), T, seed, rnd, j, seq0) for j in range(gamma)], 1).contiguous()
    ties = 0
    d_or = np.empty((rows, gamma), np.int32)
    for j in range(gamma):
        tok, mg = oracle.sample_batch(Qh[:, j], T, oracle.uniform_batch(seed, seq0, rows, rnd, j, 2), with_margin=True)
        d_or[:, j] = tok
        bad = tok != d_gpu[:, j].cpu().numpy()
        assert (mg[bad] < CDF_TIE).all(), f"draft draw mismatch beyond near-tie at position {j}"
        ties += int(bad.sum())
    d = torch.from_numpy(d_or).cuda()
    out = M.accept_logits(P, Q, d, T, seed, rnd, seq0)
    torch.cuda.synchronize()
    ua, ur = oracle_uniforms(seed, rows, gamma, rnd, seq0)
    ref = oracle.accept_batch(Ph, Qh, d_or, T, ua, ur)
    mask = out["mask"].cpu().numpy()
    n_acc, token, bd = out["n_acc"].cpu().numpy(), out["token"].cpu().numpy(), out["bd"].cpu().numpy()
    ref_mask = (ref["mask"] << np.arange(gamma)[None, :]).sum(1)
    for b in range(rows):
        if mask[b] != ref_mask[b]:
            diff = [j for j in range(gamma) if (mask[b] >> j) & 1 != (ref_mask[b] >> j) & 1]
            assert all(abs(ua[b, j] - min(1.0, ref["ratio"][b, j])) < RATIO_TIE for j in diff), (b, diff)
            ties += 1
            continue
        assert n_acc[b] == ref["n_acc"][b], b
        if token[b] != ref["token"][b]:
            assert ref["margin"][b] < CDF_TIE, (b, token[b], ref["token"][b], ref["margin"][b])
            ties += 1
    if T > 0:
        assert np.abs(bd - ref["bd"]).max() < 1e-6
    # N_acc is the index of the first cleared mask bit
    first0 = np.array([next((j for j in range(gamma) if not (m >> j) & 1), gamma) for m in mask])
    assert (first0 == n_acc).all()
    return dict(ties=ties, n_acc=n_acc, alpha=float(ref["bd"].mean()) if T > 0 else None)


@pytest.mark.parametrize("sigma", [0.5, 1.0, 2.0])
def test_config2_accept_matches_oracle(sigma):
    """Accept microbench configuration: 64 rows x gamma 5 x vocab 32000, T = 1, seed 1."""
    cfg = W.config2(sigma, device="cuda")
    r = check_accept(cfg["P"], cfg["Q"], 1.0, cfg["seed"], rnd=3)
    assert r["ties"] <= 2, r
    # the accepted length tracks the closed form for the measured mean acceptance rate
    a = r["alpha"]
    assert abs(r["n_acc"].mean() - (a - a ** 6) / (1 - a)) < 0.6


@pytest.mark.parametrize("V,rows,gamma,T", [(8, 300, 1, 1.0), (512, 33, 4, 1.0), (2048 + 4, 5, 3, 0.7), (32768, 3, 2, 1.0),
                                            (32000, 7, 7, 0.7), (12, 40, 15, 1.3)])
def test_accept_shapes_and_temperatures(V, rows, gamma, T):
    g = torch.Generator(device="cuda").manual_seed(V * 131 + rows)
    P = torch.randn((rows, gamma + 1, V), generator=g, device="cuda") * 2
    Q = (P[:, :gamma] + torch.randn((rows, gamma, V), generator=g, device="cuda")).contiguous()
    r = check_accept(P, Q, T, seed=9, rnd=1, seq0=1000)
    assert r["ties"] <= 2


def test_accept_greedy_and_degenerate_rows():
    V, gamma, rows = 1000, 4, 16
    g = torch.Generator(device="cuda").manual_seed(5)
    P = torch.randn((rows, gamma + 1, V), generator=g, device="cuda")
    Q = (P[:, :gamma] + 0.3 * torch.randn((rows, gamma, V), generator=g, device="cuda")).contiguous()
    P[0, 0, 17] = P[0, 0, 903] = 50.0                      # exact tie: lowest index wins
    r = check_accept(P, Q, 0.0, seed=2, rnd=0)
    assert r["ties"] == 0
    # p == q everywhere: every test passes (u < 1), the bonus token is drawn from p
    P2 = torch.randn((rows, gamma + 1, V), generator=g, device="cuda")
    r = check_accept(P2, P2[:, :gamma].contiguous(), 1.0, seed=2, rnd=1)
    assert (r["n_acc"] == gamma).all()
    # disjoint supports: never accept; the emitted token follows p
    P3 = torch.full((rows, gamma + 1, V), -float("inf"), device="cuda")
    Q3 = torch.full((rows, gamma, V), -float("inf"), device="cuda")
    P3[:, :, : V // 2] = torch.randn((rows, gamma + 1, V // 2), generator=g, device="cuda")
    Q3[:, :, V // 2:] = torch.randn((rows, gamma, V // 2), generator=g, device="cuda")
    r = check_accept(P3, Q3, 1.0, seed=2, rnd=2)
    assert (r["n_acc"] == 0).all()


def test_sampler_distribution_and_argmax():
    V, rows = 8, 200_000
    logits = torch.tensor(np.log([0.05, 0.3, 0.1, 0.05, 0.2, 0.1, 0.15, 0.05]), dtype=torch.float32, device="cuda")
    L = logits.repeat(rows, 1).contiguous()
    tok = M.sample_logits(L, 1.0, seed=4, rnd=2, pos=1).cpu().numpy()
    ref = oracle.sample_batch(L.cpu().numpy(), 1.0, oracle.uniform_batch(4, 0, rows, 2, 1, 2))
    assert (tok == ref).mean() > 0.9999
    assert (M.sample_logits(L[:64], 0.0, seed=4).cpu().numpy() == 1).all()


def test_stream_read_digest():
    """The streaming-read measurement aid reads every 1-KiB chunk exactly once: the xor of its per-wavefront digests equals
    the xor of all 32-bit words of the buffer (ragged: 1000 chunks + a tail below one chunk that is left out)."""
    torch.manual_seed(5)
    n_words = 1000 * 256 + 77
    src = torch.randint(-2**31, 2**31 - 1, (n_words,), dtype=torch.int32, device="cuda")
    sink = torch.zeros(M.STREAM_READ_SINK_WORDS, dtype=torch.int32, device="cuda")
    M.stream_read(src, sink)
    torch.cuda.synchronize()
    want = np.bitwise_xor.reduce(src[:1000 * 256].cpu().numpy().view(np.uint32))
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert int(got) == int(want)


def test_philox_words_match_oracle():
    n = 1_000_000
    w = M.philox_words(12345678901234567, 4_294_000_000, n, 7, 3, 2).cpu().numpy().view(np.uint32)
    idx = np.concatenate([np.arange(0, 2000), np.random.default_rng(0).integers(0, n, 3000), [n - 1]])
    for i in idx:
        c0 = (4_294_000_000 + int(i)) & 0xFFFFFFFF          # the counter word wraps around
        assert (w[i] == oracle.philox(12345678901234567, c0, 7, 3, 2)).all(), i
    assert len(np.unique(w[:, 0].astype(np.uint64) << np.uint64(32) | w[:, 1])) == n


def test_bad_arguments():
    P = torch.zeros((2, 3, 10), device="cuda")
    with pytest.raises(M.MetaSDError):                     # vocab not a multiple of 4
        M.accept_logits(P, P[:, :2].contiguous(), torch.zeros((2, 2), dtype=torch.int32, device="cuda"), 1.0, 1)
    P = torch.zeros((1, 2, 32772), device="cuda")
    with pytest.raises(M.MetaSDError):                     # vocab above the kernel's maximum
        M.sample_logits(P[0], 1.0, 1)
    # an out-of-range draft token is clamped by the kernel, never dereferenced out of bounds
    P = torch.randn((1, 2, 16), device="cuda")
    out = M.accept_logits(P, P[:, :1].contiguous(), torch.full((1, 1), 999, dtype=torch.int32, device="cuda"), 1.0, 1)
    torch.cuda.synchronize()
    assert 0 <= int(out["token"][0]) < 16


def test_accept_bounded_wait_reports_failure_and_recovers(monkeypatch):
    """The four workgroups of a position meet through memory with bounded polls.  With the bound forced to
    zero from the host every poll gives up at once: all waves exit, every row reports token -2, nothing
    hangs; the next call with the normal bound and the same scratch buffer is correct again."""
    c = W.config2(1.0, rows=8, device="cuda")
    P, Q = c["P"], c["Q"]
    d = torch.stack([M.sample_logits(Q[:, j].contiguous(), 1.0, 1, 0, j, 0) for j in range(c["gamma"])], 1).contiguous()
    good = M.accept_logits(P, Q, d, 1.0, 1, 0, 0)
    torch.cuda.synchronize()
    ref_tok, ref_n = good["token"].clone(), good["n_acc"].clone()
    monkeypatch.setenv("METASD_ACCEPT_SPIN_LIMIT", "0")
    bad = M.accept_logits(P, Q, d, 1.0, 1, 0, 0, out=good)
    torch.cuda.synchronize()
    assert (bad["token"] == -2).all()
    monkeypatch.delenv("METASD_ACCEPT_SPIN_LIMIT")
    again = M.accept_logits(P, Q, d, 1.0, 1, 0, 0, out=good)
    torch.cuda.synchronize()
    assert torch.equal(again["token"], ref_tok) and torch.equal(again["n_acc"], ref_n)
