"""Teacher-forced lock-step comparison of the GPU library with the oracle (test helper).

Each round the GPU runs select -> draft -> verify -> accept -> update on its own; the oracle is fed
the GPU's committed tokens, so both always see the same context, and every intermediate result
is compared:
  stage A  logits: drafter logits Q_j and target logits P_j, max-abs tolerance;
  stage B  the oracle's accept step on the GPU's own logits must give the GPU's mask / N_acc /
           token (exact, except draws the oracle itself flags as near-ties);
  stage C  the oracle's decisions from its own logits (draft tokens, accept tests, emitted token)
           against the GPU's: exact for fp32, logged for bf16 (a 3e-2 logit error moves p/q by
           several per cent, so token equality on independent logits is not a meaningful demand).
Near-ties: |u - p/q| < 1e-3 for accept tests, inverse-CDF margin < 1e-6 for draws, top-2 logit
gap < 2 x the logit tolerance for argmax.
"""
from __future__ import annotations

import numpy as np

import oracle

RATIO_TIE = 1e-3
CDF_TIE = 1e-6


def top2_gap(x: np.ndarray) -> float:
    part = np.partition(x, -2)[-2:]
    return float(part[1] - part[0])


class LockStep:
    def __init__(self, gpu, target, drafters, prompt, gamma, T, seed, beta, logit_tol, kv_prefilled=False, reward="BE", seq=0, feat_tol=None,
                 feat_prefill=None):
        self.feat_tol = logit_tol if feat_tol is None else feat_tol
        self.gpu, self.target, self.drafters = gpu, target, drafters
        self.seq = seq                                   # sequence of a batched context (its Philox sequence id)
        self.gamma, self.T, self.seed, self.tol, self.reward = gamma, T, seed, logit_tol, reward
        self.hist = np.zeros(target.max_ctx, np.int32)
        self.l = len(prompt)
        self.hist[: self.l] = prompt
        self.c = [self.l - 1 if kv_prefilled else 0] * len(drafters)
        self.a = [0] * len(drafters)                     # streaming drafter caches: start of the contiguous tail
        self.t = 0
        self.bandit = oracle.Ucb(len(drafters), beta)
        self.stats = dict(rounds=0, max_dq=0.0, max_dp=0.0, ties_shared=0, ties_own=0, mismatch_own=0, n_acc=[], arms=[],
                          alpha=[])
        # drafter heads on the target's hidden states: the table of the target's features, one row per cached position
        self.feat = None
        if any(getattr(D, "feature_head", False) for D in drafters):
            self.feat = np.zeros((target.max_ctx, target.desc["d_model"]), np.float32)
            if kv_prefilled:                             # synthetic prefix: its features are given like its K/V
                self.feat[: self.l - 1] = feat_prefill
            elif self.l > 1:
                _, self.feat[: self.l - 1] = target.forward_hidden(prompt[: self.l - 1], 0, None)
        elif not kv_prefilled and self.l > 1:
            target.forward(prompt[: self.l - 1], 0, None)

    def select(self, force_k=None):
        """Arm of this round: the GPU's bandit and the oracle's must agree."""
        k_gpu = self.gpu.bandit_select(seq=self.seq)
        k_or = self.bandit.select()
        assert k_gpu == k_or, f"seq {self.seq} round {self.t}: arm {k_gpu} vs oracle {k_or}"
        return k_gpu if force_k is None else force_k

    def round(self, force_k=None):
        g, gamma, l = self.gpu, self.gamma, self.l
        k = self.select(force_k)
        g.draft(k, gamma)
        g.verify(gamma)
        n_gpu, tok_gpu, mask_gpu, bd_gpu = g.accept(gamma)
        Pg = g.peek("P")[: gamma + 1].cpu().numpy()
        Qg = g.peek("Q")[:gamma].cpu().numpy()
        d = g.peek("draft")[:gamma].cpu().numpy().copy()
        hist_gpu = g.peek("hist")[l: l + gamma + 1].cpu().numpy()
        return self.check(k, n_gpu, tok_gpu, mask_gpu, bd_gpu, Pg, Qg, d, hist_gpu)

    def check(self, k, n_gpu, tok_gpu, mask_gpu, bd_gpu, Pg, Qg, d, hist_gpu):
        """Compare one finished GPU round of this sequence with the oracle and commit it on both sides."""
        g, T, seed, gamma, l, t, sq = self.gpu, self.T, self.seed, self.gamma, self.l, self.t, self.seq
        st = self.stats
        V = self.target.desc["vocab"]
        exact = self.tol <= 1e-3
        assert (hist_gpu[:n_gpu] == d[:n_gpu]).all() and hist_gpu[n_gpu] == tok_gpu     # committed on the device too
        # ---- oracle, teacher-forced on the GPU's draft tokens
        D = self.drafters[k]
        if getattr(D, "shares_kv", False):               # reads the target's cache: never a backlog
            self.c[k] = l - 1
        Qo = np.empty((gamma, V), np.float32)
        stream = getattr(D, "stream", None)
        head = getattr(D, "feature_head", False)
        if head:                                         # unseen committed tokens, each with the true feature before it
            c = self.c[k]
            feats = np.zeros((l - c, self.feat.shape[1]), np.float32)
            lo = max(c, 1)
            feats[lo - c:] = self.feat[lo - 1: l - 1]
            Qo[0], hid = D.forward_hidden(self.hist[c: l], c, "last", feats=feats)
            f_est = hid[-1]
        elif stream is not None:                         # sinks not seen yet + the last `window` committed tokens
            from oracle.loop import stream_catch_up, stream_forward
            Qo[0], self.a[k] = stream_catch_up(D, self.hist, self.c[k], l, self.a[k])
        else:
            Qo[0] = D.forward(self.hist[self.c[k]: l], self.c[k], "last")
        u_d = [oracle.uniform(seed, sq, t, j, oracle.STREAM_DRAFT) for j in range(gamma)]
        for j in range(gamma):       # stage B for the draft: the oracle's draw on the GPU's own logits
            tj, mg = oracle.sample(Qg[j], T, u_d[j], with_margin=True)
            if tj != d[j]:
                tie = mg < CDF_TIE if T > 0 else top2_gap(Qg[j]) < 1e-6
                assert tie, f"round {t} draft {j}: GPU token {d[j]} vs draw {tj} on its own logits (margin {mg})"
                st["ties_shared"] += 1
        for j in range(gamma):
            if j > 0:
                self.hist[l + j - 1] = d[j - 1]
                if head:                                 # the head's own estimate stands in for the unknown feature
                    Qo[j], hid = D.forward_hidden(self.hist[l + j - 1: l + j], l + j - 1, "last", feats=f_est[None])
                    f_est = hid[-1]
                elif stream is not None:
                    Qo[j] = stream_forward(D, self.hist, l + j - 1, l + j, self.a[k])
                else:
                    Qo[j] = D.forward(self.hist[l + j - 1: l + j], l + j - 1, "last")
            tj, mg = oracle.sample(Qo[j], T, u_d[j], with_margin=True)
            if tj != d[j]:
                tie = (mg < CDF_TIE) if T > 0 else top2_gap(Qo[j]) < 2 * self.tol
                if exact:
                    assert tie, f"round {t} draft {j}: oracle token {tj} vs GPU {d[j]} (margin {mg})"
                st["ties_own" if tie else "mismatch_own"] += 1
        self.hist[l + gamma - 1] = d[gamma - 1]
        if self.feat is not None:
            Po, Ho = self.target.forward_hidden(self.hist[l - 1: l + gamma], l - 1, "all")
        else:
            Po = self.target.forward(self.hist[l - 1: l + gamma], l - 1, "all")
        dq, dp = float(np.abs(Qo - Qg).max()), float(np.abs(Po - Pg).max())
        st["max_dq"], st["max_dp"] = max(st["max_dq"], dq), max(st["max_dp"], dp)
        assert dq <= self.tol and dp <= self.tol, f"round {t}: logits differ by {dq} (drafter) / {dp} (target) > {self.tol}"
        u_acc = np.array([oracle.uniform(seed, sq, t, j, oracle.STREAM_ACCEPT) for j in range(gamma)], np.float32)
        u_res = oracle.uniform(seed, sq, t, 0, oracle.STREAM_RESIDUAL)
        # ---- stage B: oracle accept on the GPU's logits
        rb = oracle.accept(Pg, Qg, d, T, u_acc, u_res)
        mask_b = sum(int(m) << j for j, m in enumerate(rb["mask"]))
        if T > 0:
            tie_mask = [j for j in range(gamma) if abs(u_acc[j] - min(1.0, rb["ratio"][j])) < RATIO_TIE]
        else:
            tie_mask = [j for j in range(gamma) if top2_gap(Pg[j]) < 1e-6]
        diff_bits = [j for j in range(gamma) if (mask_b >> j) & 1 != (mask_gpu >> j) & 1]
        assert all(j in tie_mask for j in diff_bits), f"round {t}: mask {mask_gpu:b} vs oracle-on-GPU-logits {mask_b:b}"
        if diff_bits:
            st["ties_shared"] += 1
        else:
            assert n_gpu == rb["n_acc"]
            if tok_gpu != rb["token"]:
                tie = rb["margin"] < CDF_TIE if T > 0 else top2_gap(Pg[n_gpu]) < 1e-6
                assert tie, f"round {t}: token {tok_gpu} vs oracle-on-GPU-logits {rb['token']} (margin {rb['margin']})"
                st["ties_shared"] += 1
            if T > 0:
                assert abs(bd_gpu - oracle.reward_bd(rb["bd"])) < 1e-5
        # ---- stage C: oracle accept on its own logits
        ro = oracle.accept(Po, Qo, d, T, u_acc, u_res)
        if ro["n_acc"] != n_gpu or ro["token"] != tok_gpu:
            if T > 0:
                tie = any(abs(u_acc[j] - min(1.0, ro["ratio"][j])) < RATIO_TIE for j in range(gamma)) or ro["margin"] < CDF_TIE
            else:
                tie = any(top2_gap(Po[j]) < 2 * self.tol for j in range(gamma + 1))
            if exact:
                assert tie, f"round {t}: oracle (n={ro['n_acc']}, tok={ro['token']}) vs GPU (n={n_gpu}, tok={tok_gpu})"
            st["ties_own" if tie else "mismatch_own"] += 1
        # ---- commit the GPU's outcome on both sides
        n = n_gpu
        self.hist[l: l + n] = d[:n]
        self.hist[l + n] = tok_gpu
        self.l = l + n + 1
        self.c[k] = min(l + n, l + gamma - 1)
        if self.feat is not None:                        # features of the committed rows; estimated-feature entries go
            self.feat[l - 1: l + n] = Ho[: n + 1]
            fg = g.peek("feat")[: l + n].cpu().numpy()
            df = float(np.abs(fg - self.feat[: l + n]).max())
            st["max_df"] = max(st.get("max_df", 0.0), df)
            assert df <= self.feat_tol, f"round {t}: feature table differs by {df} > {self.feat_tol}"
        if head:
            self.c[k] = l
        for i, Di in enumerate(self.drafters):
            if getattr(Di, "shares_kv", False):
                self.c[i] = self.l - 1
        self.t += 1
        rew = oracle.reward_be(n, gamma) if self.reward == "BE" else bd_gpu
        self.bandit.update(k, rew)
        g.bandit_update(k, n, gamma, bd_gpu, seq=sq)
        mu, nn, tt = g.bandit_state(seq=sq)
        assert np.allclose(mu, self.bandit.mu, atol=1e-12) and (nn == self.bandit.n).all() and tt == self.bandit.t
        lg, kvg, rg = g.state(-1, seq=sq)
        assert (lg, kvg, rg) == (self.l, self.l - 1, self.t)
        assert g.state(k, seq=sq)[1] == self.c[k]
        st["rounds"] += 1
        st["n_acc"].append(n)
        st["arms"].append(k)
        if T > 0:
            st["alpha"].append(float(np.mean(rb["bd"])))
        return n, tok_gpu


class BatchLockStep:
    """B sequences of one batched GPU context, each compared with its own oracle models (own KV caches)."""

    def __init__(self, gpu, seqs):
        self.gpu, self.seqs = gpu, seqs                  # seqs: LockStep objects with seq = 0 .. B-1, all sharing `gpu`

    def round(self, force_k=None):
        g = self.gpu
        gamma = self.seqs[0].gamma
        ks = [ls.select(None if force_k is None else force_k[b]) for b, ls in enumerate(self.seqs)]
        ls0 = [ls.l for ls in self.seqs]
        g.draft(ks, gamma)
        g.verify(gamma)
        n, tok, mask, bd = g.accept(gamma)
        P = g.peek("P", gamma).cpu().numpy()
        Q = g.peek("Q", gamma).cpu().numpy()
        D = g.peek("draft", gamma).cpu().numpy().copy()
        H = g.peek("hist").cpu().numpy()
        out = []
        for b, ls in enumerate(self.seqs):
            l = ls0[b]
            out.append(ls.check(ks[b], int(n[b]), int(tok[b]), int(mask[b]), float(bd[b]), P[b], Q[b], D[b], H[b, l: l + gamma + 1]))
        return ks, out
