"""Seeded synthetic inputs for the MetaSD hot path (shared by the oracle tests, the GPU parity
tests, smoke() and bench.py).  This module only draws random numbers and lays out tensors: it
holds none of the method's arithmetic (no softmax, no sampling, no decoder math, no bandit).

Shapes follow the paper's setting: a Llama-style target (Vicuna-7B shape), 68M-parameter
Llama-style drafters (2 layers, hidden 768, 12 heads, vocabulary 32000 - Sec. 4 and App.
"Drafter training"), K = 5 drafters and N_max = 5 drafts per round.  Weights are random
(no trained checkpoints exist offline).

Tensor table of a model, in order: embed [V, d]; per layer attn_norm [d], wq [H*hd, d],
wk [KH*hd, d], wv [KH*hd, d], wo [d, H*hd], ffn_norm [d], w_gate [f, d] (None for GELU),
w_up [f, d], w_down [d, f]; final_norm [d]; lm_head [V, d].  Matrices are [out, in] row-major.
"""
from __future__ import annotations

import numpy as np
import torch

PER_LAYER = 9
GELU, SWIGLU = 0, 1
FP32, BF16 = 0, 1


def model_desc(n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab, act, dtype,
               rms_eps=1e-5, rope_theta=10000.0) -> dict:
    return dict(n_layers=n_layers, d_model=d_model, n_heads=n_heads, n_kv_heads=n_kv_heads, d_ffn=d_ffn,
                vocab=vocab, act=act, dtype=dtype, rms_eps=rms_eps, rope_theta=rope_theta)


def tensor_shapes(desc: dict) -> list:
    d, H, KH, f, V = desc["d_model"], desc["n_heads"], desc["n_kv_heads"], desc["d_ffn"], desc["vocab"]
    hd = d // H
    out = [("embed", (V, d))]
    for L in range(desc["n_layers"]):
        out += [(f"l{L}.attn_norm", (d,)), (f"l{L}.wq", (H * hd, d)), (f"l{L}.wk", (KH * hd, d)),
                (f"l{L}.wv", (KH * hd, d)), (f"l{L}.wo", (d, H * hd)), (f"l{L}.ffn_norm", (d,)),
                (f"l{L}.w_gate", (f, d) if desc["act"] == SWIGLU else None),
                (f"l{L}.w_up", (f, d)), (f"l{L}.w_down", (d, f))]
    out += [("final_norm", (d,)), ("lm_head", (V, d))]
    return out


def _torch_dtype(desc):
    return torch.bfloat16 if desc["dtype"] == BF16 else torch.float32


def _randn(shape, seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def gen_weights(desc: dict, seed: int, std: float = 0.02, device: str = "cpu") -> list:
    """Random weights: matrices N(0, std), norm gains 1 + N(0, std); stored in the model dtype.
    Tensor i draws from its own generator seeded (seed, i), so tables are reproducible per
    device type (CPU and GPU generators differ; one run uses one device for both sides)."""
    dt = _torch_dtype(desc)
    out = []
    for i, (name, shape) in enumerate(tensor_shapes(desc)):
        if shape is None:
            out.append(None)
            continue
        x = _randn(shape, seed * 1000003 + i, device) * std
        if name.endswith("norm"):
            x = x + 1.0
        out.append(x.to(dt).contiguous())
    return out


def noisy_head(head: torch.Tensor, sigma: float, seed: int, scale: float = 1.0, cols: int | None = None):
    """scale * head[:, :cols] + N(0, sigma), in head's dtype."""
    base = head if cols is None else head[:, :cols]
    x = base.float() * scale
    if sigma > 0:
        x = x + _randn(tuple(x.shape), seed, str(head.device)) * sigma
    return x.to(head.dtype).contiguous()


def early_exit_drafter(tdesc: dict, tweights: list, n_run: int, sigma: float, seed: int):
    """Drafter = first n_run target layers -> target final norm -> (target head + N(0, sigma)).
    Shares the target's tensors for the layers it runs; owns its head."""
    desc = dict(tdesc)
    desc["n_layers"] = n_run
    w = list(tweights[: 1 + PER_LAYER * n_run]) + [tweights[-2], noisy_head(tweights[-1], sigma, seed)]
    return desc, w


def feature_head_drafter(tdesc: dict, tweights: list, layer: int, eps: float, seed: int):
    """A drafter head on the target's hidden states (shape only: nothing is trained here): the target's embedding, one decoder
    layer (the tensors of target layer `layer`, shared), the target's final norm and LM head, and W_fc = [I | eps * N(0, 1)]
    ([d, 2 d]) mixing the token embedding with the previous position's feature.  With eps = 0 it is the early-exit drafter
    after one layer (when layer = 0); a small eps keeps some agreement with the target while the feature path carries weight.
    Returns (desc, weights, fc)."""
    desc = dict(tdesc)
    desc["n_layers"] = 1
    d = tdesc["d_model"]
    w = [tweights[0]] + list(tweights[1 + PER_LAYER * layer: 1 + PER_LAYER * (layer + 1)]) + [tweights[-2], tweights[-1]]
    dev = str(tweights[0].device)
    fc = torch.cat([torch.eye(d, device=dev), _randn((d, d), seed, dev) * eps], dim=1).to(_torch_dtype(tdesc)).contiguous()
    return desc, w, fc


def to_numpy(weights: list) -> list:
    """Host copies for the oracle: fp32 arrays, or uint16 bit patterns for bf16 tensors."""
    out = []
    for w in weights:
        if w is None:
            out.append(None)
        elif w.dtype == torch.bfloat16:
            out.append(w.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16))
        else:
            out.append(w.detach().cpu().contiguous().numpy())
    return out


def prompt_tokens(n: int, vocab: int, seed: int) -> np.ndarray:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return torch.randint(0, vocab, (n,), generator=g, dtype=torch.int32).numpy()


def kv_fill(desc: dict, ctx: int, seed: int, device: str = "cpu"):
    """Synthetic KV prefix: K and V ~ N(0,1) in the model dtype, shape [layer, kv_head, ctx, hd]."""
    hd = desc["d_model"] // desc["n_heads"]
    shape = (desc["n_layers"], desc["n_kv_heads"], ctx, hd)
    dt = _torch_dtype(desc)
    k = _randn(shape, seed * 7919 + 1, device).to(dt)
    v = _randn(shape, seed * 7919 + 2, device).to(dt)
    return k, v


# ------------------------------------------------------------------ configurations

def config1(device: str = "cpu") -> dict:
    """Tiny full loop, fp32: 2-layer GELU target, d=128, 4 heads, FFN 512, vocab 512; K=3
    early-exit drafters after layer 1 with head noise sigma = (0, 0.02, 0.1)."""
    td = model_desc(2, 128, 4, 4, 512, 512, GELU, FP32)
    tw = gen_weights(td, 0, device=device)
    drafters = [early_exit_drafter(td, tw, 1, s, 100 + k) for k, s in enumerate((0.0, 0.02, 0.1))]
    return dict(name="C1", target=(td, tw), drafters=drafters, gamma=4, prompt=prompt_tokens(16, 512, 0),
                n_new=64, beta=1.0, seed=1, max_ctx=16 + 64 + 16)


def config2(sigma: float, rows: int = 64, gamma: int = 5, vocab: int = 32000, seed: int = 1,
            device: str = "cpu", variant: int = 0) -> dict:
    """Accept-step microbench inputs: target logits ~ N(0, 2^2), drafter logits = target + N(0, sigma^2)."""
    s = seed * 100003 + variant * 17
    P = _randn((rows, gamma + 1, vocab), s + 1, device) * 2.0
    Q = P[:, :gamma, :] + _randn((rows, gamma, vocab), s + 2, device) * sigma
    return dict(name="C2", P=P.contiguous(), Q=Q.contiguous(), rows=rows, gamma=gamma, vocab=vocab, T=1.0,
                seed=seed, sigma=sigma)


def config3(device: str = "cpu", n_layers: int = 16) -> dict:
    """1B-shape bf16 target (GQA 32/8 heads, SwiGLU 8192, vocab 32000), K=4 early-exit drafters
    at layers {2,4,6,8} with head noise 0.01; 512-token prompt, 256 new tokens, T=1."""
    td = model_desc(n_layers, 2048, 32, 8, 8192, 32000, SWIGLU, BF16)
    tw = gen_weights(td, 0, device=device)
    drafters = [early_exit_drafter(td, tw, min(e, n_layers), 0.01, 100 + k) for k, e in enumerate((2, 4, 6, 8))]
    return dict(name="C3", target=(td, tw), drafters=drafters, gamma=5, prompt=prompt_tokens(512, 32000, 3),
                n_new=256, beta=1.0, seed=1, max_ctx=512 + 256 + 16, T=1.0)


C4_NOISE = (0.25, 0.5, 1.0, 2.0, 4.0)


def c4_noise_scale(k: int, seg: int) -> float:
    """Head-noise multiplier of drafter k in segment seg (cyclic shifts: the best arm moves)."""
    return C4_NOISE[(k + seg) % len(C4_NOISE)]


def config4(device: str = "cpu", n_layers: int = 32, ctx: int = 2048, n_new: int = 128, K: int = 5,
            d_model: int = 4096, n_heads: int = 32, d_ffn: int = 11008, vocab: int = 32000,
            dd_model: int = 768, dn_heads: int = 12, dd_ffn: int = 3072, seg_len: int = 32) -> dict:
    """7B-shape bf16 target with K separate 2-layer drafters.  Drafter k's LM head in segment s
    is 0.5 * target_head[:, :d_drafter] + c4_noise_scale(k, s) * N(0, 0.02); the segment index
    is (new tokens generated // seg_len) % 4 (non-stationary reward, cf. App. "Non-stationary
    environment").  The KV prefix of ctx positions is a seeded synthetic fill."""
    td = model_desc(n_layers, d_model, n_heads, n_heads, d_ffn, vocab, SWIGLU, BF16)
    tw = gen_weights(td, 0, device=device)
    dd = model_desc(2, dd_model, dn_heads, dn_heads, dd_ffn, vocab, SWIGLU, BF16)
    drafters, heads = [], []
    for k in range(K):
        dw = gen_weights(dd, 100 + k, device=device)
        hk = [noisy_head(tw[-1], 0.02 * c4_noise_scale(k, s), 5000 + 10 * k + s, scale=0.5, cols=dd_model)
              for s in range(4)]
        dw[-1] = hk[0]
        drafters.append((dd, dw))
        heads.append(hk)
    return dict(name="C4", target=(td, tw), drafters=drafters, heads=heads, seg_len=seg_len, gamma=5,
                prompt=prompt_tokens(ctx, vocab, 3), n_new=n_new, beta=1.0, seed=1, ctx=ctx,
                max_ctx=ctx + n_new + 16, T=1.0, kv_seed=7)


def draft_tree(kind: str = "wide") -> dict:
    """Shapes of draft trees for multi-candidate rounds (parent, rank per node; node 0 the root; breadth-first order).
    'wide': 13 nodes, depth 5 - three candidates after the root, two after the likeliest nodes of the next levels, the
    likeliest path kept to depth 5 (a small stand-in for the static trees of the multi-draft methods the paper cites;
    it gives no tree of its own).  'chain5': ordinary speculation with gamma = 5 written as a tree."""
    if kind == "chain5":
        return dict(parent=[-1, 0, 1, 2, 3, 4], rank=[0] * 6)
    if kind == "bushy":          # 16 nodes, depth 3: many siblings per level (ranks up to 4)
        return dict(parent=[-1, 0, 0, 0, 0, 0, 1, 1, 1, 2, 2, 3, 6, 6, 7, 9], rank=[0, 0, 1, 2, 3, 4, 0, 1, 2, 0, 1, 0, 0, 1, 0, 0])
    return dict(parent=[-1, 0, 0, 0, 1, 1, 2, 4, 4, 5, 7, 7, 10], rank=[0, 0, 1, 2, 0, 1, 0, 0, 1, 0, 0, 1, 0])


def config1_tree(device: str = "cpu", sigmas=(0.0, 0.005, 0.02)) -> dict:
    """The tiny fp32 configuration for multi-candidate (tree) rounds.  With random weights an early exit
    after layer 1 almost never shares the target's argmax, so depth would never be exercised; the drafters here run all
    of the target's layers and differ by the noise on their LM head, sigma = (0, 0.005, 0.02): in greedy mode always /
    often / rarely the target's choice, often as a second candidate.  Sampled rounds need more noise before the accept
    ratios leave 1 (the logits are nearly flat): the tests pass sigmas = (0, 0.05, 0.15) for them."""
    cfg = config1(device)
    td, tw = cfg["target"]
    cfg["drafters"] = [early_exit_drafter(td, tw, td["n_layers"], s, 200 + k) for k, s in enumerate(sigmas)]
    cfg["name"] = "C1-tree"
    cfg["max_ctx"] = 16 + 64 + 32
    return cfg
