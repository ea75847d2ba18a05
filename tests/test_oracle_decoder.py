"""Pins for the oracle's decoder forward.  The paper fixes only "Llama architecture, SiLU"
(Sec. 4, App. "Drafter training"), so the forward is pinned by reduction to library routines:
a model assembled from torch's embedding / rms_norm / linear / scaled_dot_product_attention /
silu / gelu (float64), with rotary embedding done as a complex multiplication; plus closed-form
special cases of the rotary embedding and the consistency of block and single-row passes."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads as W


def torch_forward(desc, weights, tokens, bf16=False):
    """Prefill from an empty cache, library ops only.  bf16: K and V are rounded when cached, like the oracle."""
    rnd = (lambda x: x.to(torch.float32).to(torch.bfloat16).to(torch.float64)) if bf16 else (lambda x: x)
    f32 = lambda x: x.to(torch.float32).to(torch.float64)
    w = [None if t is None else t.to(torch.float64) for t in weights]
    d, H, KH = desc["d_model"], desc["n_heads"], desc["n_kv_heads"]
    hd = d // H
    m = len(tokens)
    h = f32(F.embedding(torch.as_tensor(tokens, dtype=torch.long), w[0]))
    pos = torch.arange(m, dtype=torch.float64)
    freqs = desc["rope_theta"] ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(m, hd // 2, dtype=torch.float64), pos[:, None] * freqs[None, :])

    def rope(x):  # x [m, heads, hd]; pair (i, i + hd/2) is one complex number
        z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for L in range(desc["n_layers"]):
        an, wq, wk, wv, wo, fn, wg, wu, wd = w[1 + 9 * L: 10 + 9 * L]
        a = f32(F.rms_norm(h, (d,), an, desc["rms_eps"]))
        q = rope(f32(F.linear(a, wq)).view(m, H, hd))
        k = rnd(rope(f32(F.linear(a, wk)).view(m, KH, hd)))
        v = rnd(f32(F.linear(a, wv)).view(m, KH, hd))
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           is_causal=True, enable_gqa=True)[0].transpose(0, 1).reshape(m, d)
        h = f32(h + f32(F.linear(f32(o), wo)))
        b = f32(F.rms_norm(h, (d,), fn, desc["rms_eps"]))
        if desc["act"] == W.SWIGLU:
            act = f32(F.silu(f32(F.linear(b, wg))) * f32(F.linear(b, wu)))
        else:
            act = f32(F.gelu(f32(F.linear(b, wu))))
        h = f32(h + f32(F.linear(act, wd)))
    x = f32(F.rms_norm(h, (d,), w[-2], desc["rms_eps"]))
    return f32(F.linear(x, w[-1])).numpy()


CASES = {
    "gelu_mha_fp32": W.model_desc(2, 64, 4, 4, 128, 97, W.GELU, W.FP32),
    "swiglu_gqa_fp32": W.model_desc(3, 64, 4, 2, 96, 50, W.SWIGLU, W.FP32),
    "swiglu_gqa_bf16": W.model_desc(2, 64, 8, 2, 96, 50, W.SWIGLU, W.BF16),
}


@pytest.mark.parametrize("name", list(CASES))
def test_forward_matches_library_model(name):
    desc = CASES[name]
    w = W.gen_weights(desc, 5, std=0.08)
    toks = W.prompt_tokens(11, desc["vocab"], 2)
    M = oracle.Model(desc, W.to_numpy(w), 32)
    got = M.forward(toks, 0, "all")
    want = torch_forward(desc, w, toks, bf16=desc["dtype"] == W.BF16)
    tol = 2e-3 if desc["dtype"] == W.BF16 else 2e-5       # bf16: a K/V rounding flip moves one cache entry by 2^-8
    assert np.abs(got - want).max() < tol
    assert np.abs(want).max() > 0.1                        # the comparison is not vacuous
    if desc["dtype"] == W.BF16:
        assert np.median(np.abs(got - want)) < 2e-5


def test_block_equals_single_rows_and_cache_reuse():
    desc = CASES["swiglu_gqa_fp32"]
    w = W.to_numpy(W.gen_weights(desc, 6, std=0.08))
    toks = W.prompt_tokens(12, desc["vocab"], 4)
    A = oracle.Model(desc, w, 16)
    full = A.forward(toks, 0, "all")
    B = oracle.Model(desc, w, 16)
    part1 = B.forward(toks[:5], 0, "all")
    part2 = B.forward(toks[5:9], 5, "all")
    last = B.forward(toks[9:12], 9, "last")
    assert np.abs(np.concatenate([part1, part2]) - full[:9]).max() < 1e-5
    assert np.abs(last - full[11]).max() < 1e-5
    Cm = oracle.Model(desc, w, 16)
    rows = np.stack([Cm.forward(toks[i:i + 1], i, "last") for i in range(12)])
    assert np.abs(rows - full).max() < 1e-5
    # overwriting speculative positions: stale cache entries beyond pos0 are never read
    B.forward(W.prompt_tokens(6, desc["vocab"], 9), 6, None)
    again = B.forward(toks[5:9], 5, "all")
    assert np.abs(again - full[5:9]).max() < 1e-5
    assert np.abs(A.kv(0)[:, :, :12] - Cm.kv(0)[:, :, :12]).max() < 1e-5


def test_rope_closed_forms():
    x = np.array([0.7, -0.3], np.float32)                  # head_dim 2: one pair, frequency 1 -> rotation by pos
    for pos in (0, 1, 5, 100):
        c, s = np.cos(pos), np.sin(pos)
        assert np.allclose(oracle.rope(x, pos, 10000.0), [0.7 * c + 0.3 * s, 0.7 * s - 0.3 * c], atol=1e-6)
    y = np.array([1.0, 2.0, 3.0, 4.0], np.float32)         # head_dim 4: pairs (0,2) and (1,3), frequencies 1 and theta^-1/2
    got = oracle.rope(y, 3, 10000.0)
    a0, a1 = 3.0, 3.0 * 10000.0 ** -0.5
    want = [1 * np.cos(a0) - 3 * np.sin(a0), 2 * np.cos(a1) - 4 * np.sin(a1),
            1 * np.sin(a0) + 3 * np.cos(a0), 2 * np.sin(a1) + 4 * np.cos(a1)]
    assert np.allclose(got, want, atol=1e-6)
    assert np.array_equal(oracle.rope(y, 0, 10000.0), y)   # position 0 is the identity
    z = np.random.default_rng(0).normal(size=64).astype(np.float32)
    assert np.isclose(np.linalg.norm(oracle.rope(z, 77, 10000.0)), np.linalg.norm(z), rtol=1e-6)
    # relative-position property: <rope(a,p), rope(b,p')> depends on p - p' only
    a, b = z[:32].copy(), z[32:].copy()
    d1 = oracle.rope(a, 9, 1e4) @ oracle.rope(b, 4, 1e4)
    d2 = oracle.rope(a, 25, 1e4) @ oracle.rope(b, 20, 1e4)
    assert np.isclose(d1, d2, atol=1e-5)


def test_bf16_rounding_matches_torch():
    xs = np.random.default_rng(1).normal(size=4000).astype(np.float32) * np.float32(3.0)
    xs = np.concatenate([xs, np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.3895314e38], np.float32)])  # ties
    want = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.round_bf16(float(x)) for x in xs], np.float32)
    assert np.array_equal(got, want)


def test_bad_arguments_are_rejected():
    desc = CASES["gelu_mha_fp32"]
    M = oracle.Model(desc, W.to_numpy(W.gen_weights(desc, 1)), 8)
    with pytest.raises(ValueError):
        M.forward([desc["vocab"]], 0)
    with pytest.raises(ValueError):
        M.forward([1, 2, 3], 6)
