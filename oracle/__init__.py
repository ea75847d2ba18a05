"""CPU oracle for the MetaSD hot path: ctypes front end of ``metasd_oracle.c``.

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The GPU library never imports it and shares no code with it.

What pins each function (all in ``tests/test_oracle_*.py``, CPU only):

* ``accept``      - brute force over a vocabulary of 8: acceptance probability = sum_v min(p, q)
                    = 1 - d_TV (Assumption 1) and output marginal = p (losslessness, Sec. 2.1 /
                    Alg. 3); special cases q = p and disjoint supports; a two-position chain.
* ``accept`` + ``uniform`` - 10^6 Philox-driven draws against the same closed forms.
* N_acc statistics - mean / variance of the accepted length against the closed forms of the
                    BE-reward lemma (App. "Proof of Theorem 1") and the printed example of the
                    stopping-time lemma (alpha = 0.1, 0.5, 0.8, N_max = 2).
* ``Ucb``         - hand-computed arm sequence for Alg. 2 stored in ``tests/golden/``.
* ``Model.forward`` - library-routine model (torch SDPA / rms_norm / linear) on random weights,
                    block-vs-single-row consistency, RoPE closed forms on head_dim 2 and 4.
* ``generate``    - greedy speculative decoding equals target-only greedy decoding token for
                    token (Alg. 3 is lossless); accounting identity B = tau + sum N_acc.
* ``Model.forward_rows`` / ``tree_round`` - tree attention and greedy tree acceptance: a chain-shaped tree equals
                    ``Model.forward`` / ``sd_round`` bit for bit; a branching tree attends exactly like a chain along each
                    root-to-node path; greedy tree decoding equals target-only greedy decoding token for token for good
                    and bad drafters; the caches after compaction equal those of a model fed the committed tokens
                    (``tests/test_oracle_tree.py``).
* ``policies``    - discounted / sliding-window UCB, sequential halving, EXP3, uniform random (the
                    paper's appendix "Extensions"): hand-worked runs in ``tests/golden/policies_hand.txt``,
                    reductions to Alg. 2, EXP3 closed forms (``tests/test_oracle_policies.py``).
* ``philox``      - word-for-word equality with rocRAND's Philox4x32-10 host generator for counters
                    (c0, c1, 0, 0) under several keys (``tests/test_gpu_philox_pin.py``, needs a device for
                    rocRAND's allocations); bijection / avalanche / moment tests on the CPU.
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "metasd_oracle.c")
_LIB = os.path.join(_HERE, "libmetasd_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


class _Desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("act", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class _UcbState(C.Structure):
    _fields_ = [("K", C.c_int32), ("t", C.c_int32), ("beta", C.c_double),
                ("mu", C.c_double * 64), ("n", C.c_int32 * 64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.om_model_create.restype = C.c_void_p
        L.om_model_create.argtypes = [C.POINTER(_Desc), C.POINTER(C.c_void_p), C.c_int32]
        L.om_model_create_shared.restype = C.c_void_p
        L.om_model_create_shared.argtypes = [C.POINTER(_Desc), C.POINTER(C.c_void_p), C.c_void_p]
        L.om_model_free.argtypes = [C.c_void_p]
        L.om_model_kv.restype = C.POINTER(C.c_float)
        L.om_model_kv.argtypes = [C.c_void_p, C.c_int]
        L.om_forward.restype = C.c_int
        L.om_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int]
        L.om_forward_ex.restype = C.c_int
        L.om_forward_ex.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.om_forward_rows_ex.restype = C.c_int
        L.om_forward_rows_ex.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p]
        L.om_forward_rows.restype = C.c_int
        L.om_forward_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.om_philox.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        L.om_uniform.restype = C.c_float
        L.om_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        L.om_uniform_batch.argtypes = [C.c_uint64, C.c_uint32, C.c_int, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        L.om_sample_batch.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
        L.om_softmax.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_void_p]
        L.om_argmax.restype = C.c_int
        L.om_argmax.argtypes = [C.c_void_p, C.c_int]
        L.om_sample.restype = C.c_int
        L.om_sample.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_float, C.c_void_p]
        L.om_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float,
                                C.c_void_p, C.c_float] + [C.c_void_p] * 6
        L.om_accept_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                      C.c_void_p, C.c_void_p] + [C.c_void_p] * 6
        L.om_rope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float]
        L.om_round_bf16.restype = C.c_float
        L.om_round_bf16.argtypes = [C.c_float]
        L.om_ucb_init.argtypes = [C.POINTER(_UcbState), C.c_int, C.c_double]
        L.om_ucb_select.restype = C.c_int
        L.om_ucb_select.argtypes = [C.POINTER(_UcbState), C.c_void_p]
        L.om_ucb_update.argtypes = [C.POINTER(_UcbState), C.c_int, C.c_double]
        L.om_reward_be.restype = C.c_double
        L.om_reward_be.argtypes = [C.c_int, C.c_int]
        L.om_reward_bd.restype = C.c_double
        L.om_reward_bd.argtypes = [C.c_void_p, C.c_int]
        L.om_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().om_num_threads())


# ------------------------------------------------------------------ model

class Model:
    """Decoder with a KV cache.  ``weights`` is the flat tensor table in the order
    embed, per layer (attn_norm, wq, wk, wv, wo, ffn_norm, w_gate | None, w_up, w_down),
    final_norm, lm_head; fp32 arrays for dtype 0, uint16 bf16 bit patterns for dtype 1.

    share_kv_with: another Model (the target) whose first ``desc["n_layers"]`` layers are this model's layers - an
    early-exit drafter.  The new model then keeps no cache of its own: it reads and writes the owner's (the
    no-recomputation strategy for drafter switches, cf. the paper's appendix on switching costs); ``shares_kv`` is set."""

    def __init__(self, desc: dict, weights: list, max_ctx: int, share_kv_with: "Model | None" = None, stream=None, fc=None):
        """fc (optional, [d, 2 d] in the model's dtype): the model is a drafter head on the target's hidden states - its rows start
        from W_fc . [embedding(token) ; feature] instead of the embedding (``forward_feat``)."""
        self.desc = dict(desc)
        self.max_ctx = int(max_ctx)
        self.fc = fc
        self.feature_head = fc is not None
        if fc is not None:
            want_fc = np.uint16 if desc["dtype"] == 1 else np.float32
            assert isinstance(fc, np.ndarray) and fc.dtype == want_fc and fc.shape == (desc["d_model"], 2 * desc["d_model"]) and fc.flags["C_CONTIGUOUS"]
        self.stream = None if stream is None else (int(stream[0]), int(stream[1]))   # (sinks, window) of a streaming drafter cache
        assert self.stream is None or (share_kv_with is None and self.stream[0] >= 0 and self.stream[1] >= 1)
        self.shares_kv = share_kv_with is not None
        self._owner = share_kv_with                  # keeps the owner (and its arrays) alive
        want = np.uint16 if desc["dtype"] == 1 else np.float32
        self._keep = []
        ptrs = (C.c_void_p * len(weights))()
        assert len(weights) == 1 + 9 * desc["n_layers"] + 2, "weight table length"
        for i, w in enumerate(weights):
            if w is None:
                ptrs[i] = None
                continue
            assert isinstance(w, np.ndarray) and w.dtype == want and w.flags["C_CONTIGUOUS"], (i, w.dtype)
            self._keep.append(w)
            ptrs[i] = w.ctypes.data
        d = _Desc(desc["n_layers"], desc["d_model"], desc["n_heads"], desc["n_kv_heads"], desc["d_ffn"],
                  desc["vocab"], desc["act"], desc["dtype"], desc.get("rms_eps", 1e-5), desc.get("rope_theta", 1e4))
        if share_kv_with is None:
            self._h = lib().om_model_create(C.byref(d), ptrs, self.max_ctx)
        else:
            assert self.max_ctx == share_kv_with.max_ctx
            self._h = lib().om_model_create_shared(C.byref(d), ptrs, share_kv_with._h)
        if not self._h:
            raise MemoryError("om_model_create failed (or the shapes of a shared-cache drafter do not match its owner's)")
        self.hd = desc["d_model"] // desc["n_heads"]

    def close(self):
        if getattr(self, "_h", None):
            lib().om_model_free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def kv(self, which: int) -> np.ndarray:
        """View of the K (0) or V (1) cache, shape [layer][kv_head][max_ctx][head_dim]."""
        p = lib().om_model_kv(self._h, which)
        shape = (self.desc["n_layers"], self.desc["n_kv_heads"], self.max_ctx, self.hd)
        return np.ctypeslib.as_array(p, shape=shape)

    def forward(self, tokens, pos0: int, want: str | None = "all"):
        """Block forward at positions pos0.. ; want = 'all' | 'last' | None."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        m = tok.shape[0]
        V = self.desc["vocab"]
        if want == "all":
            out = np.empty((m, V), np.float32)
            rc = lib().om_forward(self._h, _ptr(tok), m, pos0, _ptr(out), 0)
        elif want == "last":
            out = np.empty((V,), np.float32)
            rc = lib().om_forward(self._h, _ptr(tok), m, pos0, _ptr(out), 1)
        else:
            out = None
            rc = lib().om_forward(self._h, _ptr(tok), m, pos0, None, 0)
        if rc != 0:
            raise ValueError("om_forward: bad arguments (tokens / positions out of range)")
        return out

    def forward_hidden(self, tokens, pos0: int, want: str | None = "all", feats=None):
        """``forward`` that also returns the residual stream after the last layer of every row ([m, d]: the features of
        those positions).  feats [m, d] (drafter heads only, ``fc`` given): row r starts from W_fc . [embedding ; feats[r]]."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        m = tok.shape[0]
        V, D = self.desc["vocab"], self.desc["d_model"]
        hid = np.empty((m, D), np.float32)
        out = None if want is None else np.empty((m, V) if want == "all" else (V,), np.float32)
        if self.feature_head:
            f = np.ascontiguousarray(feats, np.float32)
            assert f.shape == (m, D)
            fcp, fp = _ptr(self.fc), _ptr(f)
        else:
            assert feats is None
            fcp, fp = None, None
        rc = lib().om_forward_ex(self._h, _ptr(tok), m, pos0, None if out is None else _ptr(out), 1 if want == "last" else 0, fcp, fp, _ptr(hid))
        if rc != 0:
            raise ValueError("om_forward_ex: bad arguments (tokens / positions out of range)")
        return out, hid

    def forward_rows(self, tokens, slots, positions, allow, want_logits: bool = True):
        """Rows that need not form a chain (tree attention): row r writes its K/V to cache slot slots[r], is rotated for
        positions[r] and attends to the slots p with allow[r, p] != 0.  Returns logits [m, V] (or None)."""
        tok = np.ascontiguousarray(tokens, np.int32)
        sl = np.ascontiguousarray(slots, np.int32)
        ps = np.ascontiguousarray(positions, np.int32)
        al = np.ascontiguousarray(allow, np.uint8)
        m = tok.shape[0]
        assert sl.shape == (m,) and ps.shape == (m,) and al.shape == (m, self.max_ctx)
        out = np.empty((m, self.desc["vocab"]), np.float32) if want_logits else None
        rc = lib().om_forward_rows(self._h, _ptr(tok), m, _ptr(sl), _ptr(ps), _ptr(al), _ptr(out) if want_logits else None)
        if rc != 0:
            raise ValueError("om_forward_rows: bad arguments")
        return out

    def forward_rows_hidden(self, tokens, slots, positions, allow, feats=None):
        """forward_rows that also returns the residual stream after the last layer of every row; a drafter head (fc given
        at construction) takes feats [m, D], the feature input of every row.  Returns (logits [m, V], hidden [m, D])."""
        tok = np.ascontiguousarray(tokens, np.int32)
        sl = np.ascontiguousarray(slots, np.int32)
        ps = np.ascontiguousarray(positions, np.int32)
        al = np.ascontiguousarray(allow, np.uint8)
        m, D = tok.shape[0], self.desc["d_model"]
        assert sl.shape == (m,) and ps.shape == (m,) and al.shape == (m, self.max_ctx)
        out = np.empty((m, self.desc["vocab"]), np.float32)
        hid = np.empty((m, D), np.float32)
        if self.feature_head:
            f = np.ascontiguousarray(feats, np.float32)
            assert f.shape == (m, D)
            fcp, fp = _ptr(self.fc), _ptr(f)
        else:
            assert feats is None
            fcp, fp = None, None
        rc = lib().om_forward_rows_ex(self._h, _ptr(tok), m, _ptr(sl), _ptr(ps), _ptr(al), _ptr(out), fcp, fp, _ptr(hid))
        if rc != 0:
            raise ValueError("om_forward_rows_ex: bad arguments")
        return out, hid


# ------------------------------------------------------------------ randomness

STREAM_ACCEPT, STREAM_RESIDUAL, STREAM_DRAFT = 0, 1, 2


def philox(seed: int, c0: int, c1: int, c2: int, c3: int) -> np.ndarray:
    out = np.empty(4, np.uint32)
    lib().om_philox(seed, c0, c1, c2, c3, _ptr(out))
    return out


def uniform(seed: int, seq: int, rnd: int, pos: int, stream: int) -> float:
    return float(lib().om_uniform(seed, seq, rnd, pos, stream))


def uniform_batch(seed: int, seq0: int, n: int, rnd: int, pos: int, stream: int) -> np.ndarray:
    """Uniforms of sequences seq0 .. seq0+n-1 at one (round, pos, stream)."""
    out = np.empty(n, np.float32)
    lib().om_uniform_batch(seed, seq0, n, rnd, pos, stream, _ptr(out))
    return out


# ------------------------------------------------------------------ sampling / accept

def sample_batch(logits, T: float, u, with_margin: bool = False):
    x = np.ascontiguousarray(logits, np.float32)
    u = np.ascontiguousarray(u, np.float32)
    rows, V = x.shape
    tok = np.empty(rows, np.int32)
    mg = np.empty(rows, np.float64)
    lib().om_sample_batch(_ptr(x), rows, V, T, _ptr(u), _ptr(tok), _ptr(mg))
    return (tok, mg) if with_margin else tok


def softmax(logits: np.ndarray, T: float) -> np.ndarray:
    x = np.ascontiguousarray(logits, np.float32)
    out = np.empty(x.shape[0], np.float64)
    lib().om_softmax(_ptr(x), x.shape[0], T, _ptr(out))
    return out


def argmax(x: np.ndarray) -> int:
    x = np.ascontiguousarray(x, np.float32)
    return int(lib().om_argmax(_ptr(x), x.shape[0]))


def sample(logits: np.ndarray, T: float, u: float, with_margin: bool = False):
    x = np.ascontiguousarray(logits, np.float32)
    mg = C.c_double(0.0)
    t = int(lib().om_sample(_ptr(x), x.shape[0], T, u, C.byref(mg)))
    return (t, mg.value) if with_margin else t


def accept(P, Q, d, T: float, u_acc, u_res: float) -> dict:
    """Alg. 3 accept step for one sequence.  P [gamma+1, V], Q [gamma, V], d [gamma]."""
    P = np.ascontiguousarray(P, np.float32)
    Q = np.ascontiguousarray(Q, np.float32)
    d = np.ascontiguousarray(d, np.int32)
    u_acc = np.ascontiguousarray(u_acc, np.float32)
    gamma, V = Q.shape
    assert P.shape == (gamma + 1, V) and d.shape == (gamma,) and u_acc.shape == (gamma,)
    mask = np.zeros(gamma, np.int32)
    n_acc = C.c_int32(0)
    token = C.c_int32(0)
    bd = np.zeros(gamma, np.float64)
    ratio = np.zeros(gamma, np.float64)
    margin = C.c_double(0.0)
    lib().om_accept(_ptr(P), _ptr(Q), _ptr(d), gamma, V, T, _ptr(u_acc), u_res,
                    _ptr(mask), C.byref(n_acc), C.byref(token), _ptr(bd), _ptr(ratio), C.byref(margin))
    return dict(mask=mask, n_acc=int(n_acc.value), token=int(token.value), bd=bd, ratio=ratio,
                margin=float(margin.value))


def accept_batch(P, Q, d, T: float, u_acc, u_res) -> dict:
    """Rows of ``accept``: P [rows, gamma+1, V], Q [rows, gamma, V], d, u_acc [rows, gamma], u_res [rows]."""
    P = np.ascontiguousarray(P, np.float32)
    Q = np.ascontiguousarray(Q, np.float32)
    d = np.ascontiguousarray(d, np.int32)
    u_acc = np.ascontiguousarray(u_acc, np.float32)
    u_res = np.ascontiguousarray(u_res, np.float32)
    rows, gamma, V = Q.shape
    assert P.shape == (rows, gamma + 1, V) and d.shape == (rows, gamma)
    mask = np.zeros((rows, gamma), np.int32)
    n_acc = np.zeros(rows, np.int32)
    token = np.zeros(rows, np.int32)
    bd = np.zeros((rows, gamma), np.float64)
    ratio = np.zeros((rows, gamma), np.float64)
    margin = np.zeros(rows, np.float64)
    lib().om_accept_batch(_ptr(P), _ptr(Q), _ptr(d), rows, gamma, V, T, _ptr(u_acc), _ptr(u_res),
                          _ptr(mask), _ptr(n_acc), _ptr(token), _ptr(bd), _ptr(ratio), _ptr(margin))
    return dict(mask=mask, n_acc=n_acc, token=token, bd=bd, ratio=ratio, margin=margin)


def rope(v: np.ndarray, pos: int, theta: float) -> np.ndarray:
    x = np.array(v, np.float32, copy=True)
    lib().om_rope(_ptr(x), x.shape[0], pos, theta)
    return x


def round_bf16(x: float) -> float:
    return float(lib().om_round_bf16(x))


# ------------------------------------------------------------------ bandit

class Ucb:
    """MetaSD-UCB (Alg. 2): per-query state mu_i, n_i, t."""

    def __init__(self, K: int, beta: float):
        assert 1 <= K <= 64
        self.K = K
        self._s = _UcbState()
        lib().om_ucb_init(C.byref(self._s), K, beta)

    def select(self, with_scores: bool = False):
        sc = np.empty(self.K, np.float64)
        a = int(lib().om_ucb_select(C.byref(self._s), _ptr(sc)))
        return (a, sc) if with_scores else a

    def update(self, arm: int, reward: float):
        lib().om_ucb_update(C.byref(self._s), arm, reward)

    @property
    def mu(self):
        return np.array(self._s.mu[: self.K])

    @property
    def n(self):
        return np.array(self._s.n[: self.K])

    @property
    def t(self):
        return int(self._s.t)


def reward_be(n_acc: int, gamma: int) -> float:
    return float(lib().om_reward_be(n_acc, gamma))


def reward_bd(bd: np.ndarray) -> float:
    b = np.ascontiguousarray(bd, np.float64)
    return float(lib().om_reward_bd(_ptr(b), b.shape[0]))


from .loop import SdState, sd_round, generate, ar_decode  # noqa: E402,F401
from .tree import Tree, tree_round, generate_tree  # noqa: E402,F401
from . import policies  # noqa: E402,F401
