"""MetaSD generation loop of the oracle: Alg. 1 (generic loop), Alg. 2 (UCB policy) and one
speculative-sampling round per Alg. 3, written step by step on top of the C primitives.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Bookkeeping.  ``hist[0:l]`` are the committed tokens.  The target's KV cache holds positions
``[0, l-1)``: the last committed token has no KV yet, it is row 0 of the next verification
block.  Drafter k's KV cache holds positions ``[0, c[k])`` with ``c[k] <= l-1``; when drafter k
is selected it first consumes every committed token it has not seen (App. "Switching costs":
the missing KV entries are recomputed when a drafter is switched in).  An early-exit drafter that
shares the target's cache (``Model(..., share_kv_with=target)``) has nothing to consume: the
target's cache already holds the K/V of its layers at every committed position but the last, so
for it ``c[k] = l-1`` at the start of every round.

Streaming drafter caches (the paper's appendix "MetaEagle-UCB with efficient KV cache strategies" replaces the
recomputation on a drafter switch by the StreamingLLM technique and states neither sink nor window size).  Reading used
here: a drafter with ``stream = (S, W)`` attends, at position p, to the first S positions (the attention sinks) and to the
last W positions up to p, at their original positions; when it is switched in it therefore needs, besides the sinks, only
the last W committed tokens, and that is all it consumes - a longer backlog is skipped, and ``a[k]`` remembers where the
contiguous tail of its cache starts so that nothing skipped is ever attended to.  (The drafter's distribution changes;
the output law does not: Alg. 3 is exact for any drafter.)

Drafter heads on the target's hidden states (the white-box drafters of Sec. 4: "Eagle" drafters; the paper gives no
formulas for them).  Reading used here, after the published design it cites: the *feature* of position p, f_p, is the
target's residual stream after its last layer at p.  A drafter head (``Model(..., fc=W_fc)``: W_fc, its own decoder
layer(s), and the target's embedding, final norm and LM head) processes position p from the token there and the feature
of the position before it: h = W_fc . [embedding(x_p) ; f_{p-1}] (f_{-1} = 0), then its layers with a KV cache of its own;
what comes out is its estimate of f_p, and the target's final norm and LM head turn that into the distribution of
x_{p+1}.  While drafting, the estimate of f_p is the feature input of the next step.  True features exist for every
position the target has processed, i.e. up to l - 2; the verification pass yields those of the block's rows, and the
accepted ones (positions l-1 .. l-1+n) are kept.  Whatever the head computed from estimated features is not kept: after
a round its cache is valid up to position l_before - 1 only (``c[k] = l_before``), and the next time it is selected it
first consumes the committed tokens since then with their true features.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class SdState:
    hist: np.ndarray                 # int32 [max_ctx]
    l: int                           # number of committed tokens
    c: list                          # per-drafter number of positions already in its KV cache
    t: int = 0                       # completed rounds (Alg. 2's t)
    log: list = field(default_factory=list)
    a: list = None                   # streaming drafters: first position of the contiguous tail of the cache (0: no gap)
    feat: np.ndarray = None          # [max_ctx, d] target features of the processed positions (only with drafter heads)


def stream_allow(max_ctx: int, positions, S: int, W: int, a: int) -> np.ndarray:
    """allow[r, p] = 1 iff row r (at positions[r]) attends to cache position p: a sink (p < S) or one of the last W positions
    up to its own that belong to the contiguous tail starting at a."""
    al = np.zeros((len(positions), max_ctx), np.uint8)
    for r, pr in enumerate(positions):
        al[r, : min(S, pr + 1)] = 1
        al[r, max(a, pr - W + 1): pr + 1] = 1
    return al


def stream_forward(drafter, hist, lo: int, hi: int, a: int):
    """Feed positions lo .. hi-1 to a streaming drafter (blocks of <= 16 rows); returns the last row's logits."""
    S, W = drafter.stream
    out = None
    for b0 in range(lo, hi, 16):
        pos = list(range(b0, min(b0 + 16, hi)))
        out = drafter.forward_rows(hist[pos[0]: pos[-1] + 1], pos, pos, stream_allow(drafter.max_ctx, pos, S, W, a))
    return None if out is None else out[-1]


def stream_catch_up(drafter, hist, c: int, l: int, a: int):
    """What a streaming drafter consumes when it is switched in with c positions cached and l tokens committed: the
    sinks it has not seen, then the last W committed tokens (a longer backlog is skipped and the tail restarts there).
    Returns (logits after the last committed token, new tail start)."""
    S, W = drafter.stream
    q = None
    if c < min(S, l):
        q = stream_forward(drafter, hist, c, min(S, l), a)
        c = min(S, l)
    start = max(c, l - W)
    if start > c:
        a = start
    if start < l:
        q = stream_forward(drafter, hist, start, l, a)
    return q, a


def sd_round(target, drafter, k: int, st: SdState, gamma: int, T: float, seed: int, seq: int = 0) -> dict:
    """One draft -> verify -> accept round (Alg. 3 body) with drafter ``k``; commits the result."""
    from . import STREAM_ACCEPT, STREAM_DRAFT, STREAM_RESIDUAL, accept, sample, uniform

    l = st.l
    V = target.desc["vocab"]
    Q = np.empty((gamma, V), np.float32)
    d = np.empty(gamma, np.int32)
    draft_margin = np.empty(gamma, np.float64)
    # --- draft: catch-up block (ends with the last committed token), then gamma-1 single steps
    if getattr(drafter, "shares_kv", False):
        st.c[k] = l - 1
    stream = getattr(drafter, "stream", None)
    head = getattr(drafter, "feature_head", False)
    f_est = None
    if head:
        # the committed tokens it has not seen, each with the true feature of the position before it
        c = st.c[k]
        D = st.feat.shape[1]
        feats = np.zeros((l - c, D), np.float32)
        lo = max(c, 1)
        feats[lo - c:] = st.feat[lo - 1: l - 1]
        Q[0], hid = drafter.forward_hidden(st.hist[c: l], c, "last", feats=feats)
        f_est = hid[-1]
    elif stream is not None:
        if st.a is None:
            st.a = [0] * len(st.c)
        Q[0], st.a[k] = stream_catch_up(drafter, st.hist, st.c[k], l, st.a[k])
    else:
        Q[0] = drafter.forward(st.hist[st.c[k]: l], st.c[k], "last")
    for j in range(gamma):
        if j > 0 and head:
            Q[j], hid = drafter.forward_hidden(st.hist[l + j - 1: l + j], l + j - 1, "last", feats=f_est[None])
            f_est = hid[-1]
        elif j > 0 and stream is not None:
            Q[j] = stream_forward(drafter, st.hist, l + j - 1, l + j, st.a[k])
        elif j > 0:
            Q[j] = drafter.forward(st.hist[l + j - 1: l + j], l + j - 1, "last")
        u = uniform(seed, seq, st.t, j, STREAM_DRAFT)
        d[j], draft_margin[j] = sample(Q[j], T, u, with_margin=True)
        st.hist[l + j] = d[j]
    # --- verify: one target pass over [x_last, d_1 .. d_gamma]
    if st.feat is not None:
        P, H = target.forward_hidden(st.hist[l - 1: l + gamma], l - 1, "all")
    else:
        P = target.forward(st.hist[l - 1: l + gamma], l - 1, "all")
    # --- accept
    u_acc = np.array([uniform(seed, seq, st.t, j, STREAM_ACCEPT) for j in range(gamma)], np.float32)
    u_res = uniform(seed, seq, st.t, 0, STREAM_RESIDUAL)
    r = accept(P, Q, d, T, u_acc, u_res)
    n = r["n_acc"]
    # --- commit: d_1..d_n stay, the emitted token follows them
    st.hist[l + n] = r["token"]
    st.l = l + n + 1
    st.c[k] = st.l - 1 if getattr(drafter, "shares_kv", False) else min(l + n, l + gamma - 1)
    if st.feat is not None:
        st.feat[l - 1: l + n] = H[: n + 1]             # the features of the committed rows of the block
    if head:
        st.c[k] = l                                    # what it computed from estimated features is not kept
    out = dict(k=k, round=st.t, l_before=l, d=d.copy(), P=P, Q=Q, u_acc=u_acc, u_res=u_res,
               draft_margin=draft_margin, **r)
    st.t += 1
    return out


def generate(target, drafters, prompt, n_new: int, gamma: int, T: float, seed: int, beta: float,
             reward: str = "BE", seq: int = 0, kv_prefilled: bool = False, policy=None,
             before_round=None, keep_logits: bool = False) -> dict:
    """MetaSD-UCB generation (Alg. 2).  Stops when ``n_new`` tokens beyond the prompt exist
    (the check ``l < B`` is made before every round, also during the initial sweep); the
    output is truncated to exactly ``n_new`` new tokens.

    policy: optional callable(round_index) -> arm overriding the bandit's choice (the bandit is
    still updated), used to test single-drafter runs.
    before_round: optional callable(state) run before each round (e.g. to swap drafter heads).
    """
    from . import Ucb, reward_bd, reward_be

    prompt = np.asarray(prompt, np.int32)
    l0 = int(prompt.shape[0])
    B = l0 + n_new
    hist = np.zeros(target.max_ctx, np.int32)
    hist[:l0] = prompt
    st = SdState(hist=hist, l=l0, c=[0] * len(drafters))
    heads = any(getattr(dr, "feature_head", False) for dr in drafters)
    if heads:
        st.feat = np.zeros((target.max_ctx, target.desc["d_model"]), np.float32)
    if kv_prefilled:
        assert not heads, "drafter heads need the features of the prefilled positions"
        st.c = [l0 - 1] * len(drafters)
    elif l0 > 1:
        if heads:
            _, st.feat[: l0 - 1] = target.forward_hidden(prompt[: l0 - 1], 0, None)
        else:
            target.forward(prompt[: l0 - 1], 0, None)
    bandit = Ucb(len(drafters), beta)
    rounds = []
    while st.l < B:
        if before_round is not None:
            before_round(st)
        k, scores = bandit.select(with_scores=True)
        if policy is not None:
            k = int(policy(st.t))
        r = sd_round(target, drafters[k], k, st, gamma, T, seed, seq)
        rew = reward_be(r["n_acc"], gamma) if reward == "BE" else reward_bd(r["bd"])
        bandit.update(k, rew)
        r["reward"] = rew
        r["scores"] = scores
        if not keep_logits:
            r.pop("P"), r.pop("Q")
        rounds.append(r)
    return dict(tokens=st.hist[l0:B].copy(), total_len=st.l, rounds=rounds, state=st,
                mu=bandit.mu, n=bandit.n, t=bandit.t)


def ar_decode(target, prompt, n_new: int, T: float = 0.0, seed: int = 0, seq: int = 0) -> np.ndarray:
    """Plain autoregressive decoding with the target alone: one token per forward pass.
    T == 0 is greedy; T > 0 draws with the residual-stream uniform of round i."""
    from . import STREAM_RESIDUAL, sample, uniform

    prompt = np.asarray(prompt, np.int32)
    l0 = int(prompt.shape[0])
    out = np.empty(n_new, np.int32)
    logits = target.forward(prompt, 0, "last")
    for i in range(n_new):
        u = uniform(seed, seq, i, 0, STREAM_RESIDUAL)
        out[i] = sample(logits, T, u)
        if i + 1 < n_new:
            logits = target.forward(out[i: i + 1], l0 + i, "last")
    return out
