"""ctypes binding of include/metasd.h.  Names follow the C ABI; argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
PER_LAYER = 9
MATRIX_SLOTS = (1, 2, 3, 4, 6, 7, 8)          # wq wk wv wo w_gate w_up w_down within a layer

EXPORTS = ["metasd_kv_bytes", "metasd_workspace_bytes", "metasd_pack_weight", "metasd_create", "metasd_destroy",
           "metasd_set_context", "metasd_swap_weight", "metasd_bandit_select", "metasd_bandit_update",
           "metasd_bandit_state", "metasd_draft", "metasd_verify", "metasd_accept", "metasd_draft_tree", "metasd_verify_tree", "metasd_accept_tree", "metasd_accept_logits",
           "metasd_accept_logits_noalloc", "metasd_sample_logits", "metasd_philox_words", "metasd_stream_read", "metasd_profile", "metasd_profile_read", "metasd_profile_shapes", "metasd_peek", "metasd_state", "metasd_state_seq", "metasd_accept_fallbacks", "metasd_set_drafter_head", "metasd_last_error"]


class MetaSDError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"metasd error {code}: {msg}")
        self.code = code


class _Desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("act", C.c_int32), ("dtype", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class _Config(C.Structure):
    _fields_ = [("K", C.c_int32), ("gamma_max", C.c_int32), ("batch", C.c_int32), ("max_ctx", C.c_int32),
                ("temperature", C.c_float), ("reward", C.c_int32), ("ucb_beta", C.c_double), ("seed", C.c_uint64),
                ("policy", C.c_int32), ("policy_window", C.c_int32), ("policy_param", C.c_double),
                ("stream_sink", C.c_int32), ("stream_window", C.c_int32), ("feature_heads", C.c_int32)]


class _Tree(C.Structure):
    _fields_ = [("n", C.c_int32), ("parent", C.c_int32 * 16), ("rank", C.c_int32 * 16)]


def lib_path() -> str:
    return os.path.join(HERE, "libmetasd.so")


_lib = None


def load_library():
    """Load libmetasd.so (built by ``paper_2604_05417_amd.build`` / ``__graft_entry__.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python -m paper_2604_05417_amd.build` (hipcc, gfx950) first")
    L = C.CDLL(path)
    vp, i32, u32, u64, f32, f64, sz = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_float, C.c_double, C.c_size_t
    sig = {
        "metasd_kv_bytes": [C.POINTER(_Desc), i32, C.POINTER(sz)],
        "metasd_workspace_bytes": [C.POINTER(_Config), C.POINTER(_Desc), C.POINTER(_Desc), C.POINTER(sz)],
        "metasd_pack_weight": [vp, vp, i32, i32, i32, vp],
        "metasd_create": [C.POINTER(vp), C.POINTER(_Config), C.POINTER(_Desc), C.POINTER(_Desc), C.POINTER(vp),
                          C.POINTER(C.POINTER(vp)), vp, C.POINTER(vp), vp, sz, vp],
        "metasd_destroy": [vp],
        "metasd_set_context": [vp, i32, vp, i32, i32],
        "metasd_swap_weight": [vp, i32, i32, vp],
        "metasd_bandit_select": [vp, i32, C.POINTER(i32)],
        "metasd_bandit_update": [vp, i32, i32, i32, i32, f64],
        "metasd_bandit_state": [vp, i32, vp, vp, C.POINTER(i32)],
        "metasd_set_drafter_head": [vp, i32, vp],
        "metasd_draft": [vp, C.POINTER(i32), i32],
        "metasd_verify": [vp, i32],
        "metasd_accept": [vp, i32, vp, vp, vp, vp],
        "metasd_draft_tree": [vp, i32, C.POINTER(_Tree)],
        "metasd_verify_tree": [vp],
        "metasd_accept_tree": [vp, C.POINTER(i32), C.POINTER(i32), vp],
        "metasd_accept_logits": [vp, vp, vp, i32, i32, i32, f32, u64, u32, u32, vp, vp, vp, vp, vp, vp],
        "metasd_accept_logits_noalloc": [vp, vp, vp, i32, i32, i32, f32, u64, u32, u32, vp, vp, vp, vp, vp],
        "metasd_sample_logits": [vp, i32, i32, f32, u64, u32, u32, u32, vp, vp],
        "metasd_philox_words": [u64, u32, i32, u32, u32, u32, vp, vp],
        "metasd_stream_read": [vp, C.c_size_t, vp, vp],
        "metasd_profile": [vp, i32],
        "metasd_profile_read": [vp, i32, C.POINTER(f64), C.POINTER(C.c_int64), C.POINTER(f64)],
        "metasd_profile_shapes": [vp, i32, i32, vp, vp, vp, vp, vp, vp, C.POINTER(i32)],
        "metasd_peek": [vp, i32, C.POINTER(vp), C.POINTER(sz)],
        "metasd_state": [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)],
        "metasd_state_seq": [vp, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)],
        "metasd_accept_fallbacks": [vp, C.POINTER(C.c_int64)],
    }
    for name, args in sig.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = i32
    L.metasd_last_error.argtypes = [vp]
    L.metasd_last_error.restype = C.c_char_p
    _lib = L
    return L


def _check(rc: int, ctx=None):
    if rc != 0:
        raise MetaSDError(rc, load_library().metasd_last_error(ctx).decode())


def _require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("the MetaSD library needs a GPU (MI355X); there is no CPU fallback")


def _stream_ptr(stream=None) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _desc(d: dict) -> _Desc:
    return _Desc(d["n_layers"], d["d_model"], d["n_heads"], d["n_kv_heads"], d["d_ffn"], d["vocab"], d["act"], d["dtype"],
                 d.get("rms_eps", 1e-5), d.get("rope_theta", 10000.0))


def pack_weight(w: torch.Tensor, rope_head_dim: int = 0, stream=None) -> torch.Tensor:
    """Row-major bf16 matrix [n_out, n_in] on the GPU -> streaming-tile order (same shape container).
    rope_head_dim: the head dimension for the q and k projections, 0 for every other matrix."""
    _require_gpu()
    assert w.is_cuda and w.dtype == torch.bfloat16 and w.dim() == 2 and w.is_contiguous()
    out = torch.empty_like(w)
    _check(load_library().metasd_pack_weight(out.data_ptr(), w.data_ptr(), w.shape[0], w.shape[1], rope_head_dim,
                                             _stream_ptr(stream)))
    return out


POLICIES = {"ucb": 0, "ducb": 1, "swucb": 2, "exp3": 3, "sh": 4, "random": 5}


class MetaSD:
    """One MetaSD context: a target, K drafters, their KV caches and the workspace (all torch-owned)."""

    def __init__(self, target, drafters, gamma_max: int, max_ctx: int, temperature: float, seed: int,
                 ucb_beta: float = 1.0, reward: str = "BE", device: str = "cuda:0", policy: str = "ucb",
                 policy_param: float = 0.0, policy_window: int = 0, batch: int = 1, share_target_kv: bool = False,
                 stream=None, heads=None):
        """stream = (sinks, window): drafters with caches of their own keep a streaming cache (metasd_config.stream_*).
        heads = {k: W_fc [d, 2 d]}: drafter k is a head on the target's hidden states (metasd_set_drafter_head)."""
        _require_gpu()
        self.L = load_library()
        self.device = torch.device(device)
        self.K = len(drafters)
        self.gamma_max = gamma_max
        self.max_ctx = max_ctx
        self.batch = batch
        self._packed = {}       # data_ptr of a row-major matrix -> packed tensor (early-exit drafters share the target's)
        self._keep = []
        tdesc, tw = target
        self.tdesc = dict(tdesc)
        self.ddescs = [dict(d) for d, _ in drafters]
        self.cfg = _Config(self.K, gamma_max, batch, max_ctx, temperature, 1 if reward == "BD" else 0, ucb_beta, seed,
                           POLICIES[policy], policy_window, policy_param, 0 if stream is None else int(stream[0]),
                           0 if stream is None else int(stream[1]), 1 if heads else 0)
        self._tdesc_c = _desc(tdesc)
        self._ddesc_c = (_Desc * self.K)(*[_desc(d) for d in self.ddescs])
        self._tw = self._table(tdesc, tw)
        self._dw = [self._table(d, w) for d, w in drafters]
        self.kv_target = self._alloc_kv(self._tdesc_c, tdesc)
        # share_target_kv: a drafter whose layer tensors ARE the target's first layers (early exit) gets the target's cache
        # itself (metasd.h, "shared" strategy); every other drafter gets a cache of its own
        self.kv_shared = [share_target_kv and d["n_layers"] <= tdesc["n_layers"] and
                          all(a is b for a, b in zip(w[: 1 + PER_LAYER * d["n_layers"]], tw)) for d, w in drafters]
        self.kv_drafters = [self.kv_target if self.kv_shared[k] else self._alloc_kv(self._ddesc_c[k], self.ddescs[k]) for k in range(self.K)]
        nbytes = C.c_size_t(0)
        _check(self.L.metasd_workspace_bytes(C.byref(self.cfg), C.byref(self._tdesc_c), self._ddesc_c, C.byref(nbytes)))
        self.workspace = torch.zeros(nbytes.value, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        tptr = (C.c_void_p * len(self._tw))(*self._tw)
        dptrs = [(C.c_void_p * len(t))(*t) for t in self._dw]
        dtab = (C.POINTER(C.c_void_p) * self.K)(*[C.cast(p, C.POINTER(C.c_void_p)) for p in dptrs])
        dkv = (C.c_void_p * self.K)(*[t.data_ptr() for t in self.kv_drafters])
        h = C.c_void_p()
        torch.cuda.synchronize(self.device)
        _check(self.L.metasd_create(C.byref(h), C.byref(self.cfg), C.byref(self._tdesc_c), self._ddesc_c, tptr, dtab,
                                    self.kv_target.data_ptr(), dkv, self.workspace.data_ptr(), nbytes.value,
                                    _stream_ptr(self.stream)))
        self._h = h
        for k, fc in (heads or {}).items():
            want = torch.bfloat16 if tdesc["dtype"] == 1 else torch.float32
            assert fc.dtype == want and tuple(fc.shape) == (tdesc["d_model"], 2 * tdesc["d_model"])
            t = fc.to(self.device).contiguous()
            if tdesc["dtype"] == 1:
                t = pack_weight(t)
            self._keep.append(t)
            _check(self.L.metasd_set_drafter_head(self._h, int(k), t.data_ptr()), self._h)

    # ---- construction helpers
    def _prepare(self, desc, index, w):
        """Device tensor for weight-table entry `index`.  Tensors shared between tables (early-exit
        drafters reuse the target's) are uploaded, and bf16 matrices packed, once."""
        if w is None:
            return None
        want = torch.bfloat16 if desc["dtype"] == 1 else torch.float32
        assert w.dtype == want, (index, w.dtype)
        nl = desc["n_layers"]
        is_matrix = (index == 2 + PER_LAYER * nl) or (1 <= index <= PER_LAYER * nl and (index - 1) % PER_LAYER in MATRIX_SLOTS)
        pack = desc["dtype"] == 1 and is_matrix
        is_qk = 1 <= index <= PER_LAYER * nl and (index - 1) % PER_LAYER in (1, 2)
        rope_hd = desc["d_model"] // desc["n_heads"] if (pack and is_qk) else 0
        key = (w.data_ptr(), tuple(w.shape), pack, rope_hd)
        if key not in self._packed:
            dev = w.to(self.device).contiguous()
            self._packed[key] = (pack_weight(dev, rope_hd) if pack else dev, w)   # keep the source alive: the key stays unique
        return self._packed[key][0]

    def _table(self, desc, weights):
        assert len(weights) == 1 + PER_LAYER * desc["n_layers"] + 2
        out = []
        for i, w in enumerate(weights):
            t = self._prepare(desc, i, w)
            self._keep.append(t)
            out.append(None if t is None else t.data_ptr())
        return out

    def _alloc_kv(self, desc_c, desc):
        nbytes = C.c_size_t(0)
        _check(self.L.metasd_kv_bytes(C.byref(desc_c), self.max_ctx, C.byref(nbytes)))
        dt = torch.bfloat16 if desc["dtype"] == 1 else torch.float32
        hd = desc["d_model"] // desc["n_heads"]
        t = torch.zeros((self.batch, desc["n_layers"], 2, desc["n_kv_heads"], self.max_ctx, hd), dtype=dt, device=self.device)
        assert t.numel() * t.element_size() == nbytes.value * self.batch
        return t[0] if self.batch == 1 else t

    # ---- C ABI, same names
    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize(self.device)
            self.L.metasd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_context(self, tokens, kv_prefilled: bool = False, seq: int = 0):
        tok = np.ascontiguousarray(tokens, np.int32)
        _check(self.L.metasd_set_context(self._h, seq, tok.ctypes.data_as(C.c_void_p), tok.shape[0], int(kv_prefilled)), self._h)

    def swap_weight(self, model: int, index: int, tensor: torch.Tensor):
        """tensor must already be in device layout (bf16 matrices: packed with pack_weight)."""
        self._keep.append(tensor)
        _check(self.L.metasd_swap_weight(self._h, model, index, tensor.data_ptr()), self._h)

    def bandit_select(self, seq: int = 0) -> int:
        k = C.c_int32(-1)
        _check(self.L.metasd_bandit_select(self._h, seq, C.byref(k)), self._h)
        return int(k.value)

    def bandit_update(self, k: int, n_acc: int, gamma: int, bd_reward: float = float("nan"), seq: int = 0):
        _check(self.L.metasd_bandit_update(self._h, seq, k, n_acc, gamma, bd_reward), self._h)

    def bandit_state(self, seq: int = 0):
        mu = np.zeros(self.K, np.float64)
        n = np.zeros(self.K, np.int32)
        t = C.c_int32(0)
        _check(self.L.metasd_bandit_state(self._h, seq, mu.ctypes.data_as(C.c_void_p), n.ctypes.data_as(C.c_void_p), C.byref(t)))
        return mu, n, int(t.value)

    def draft(self, k, gamma: int):
        """k: the arm (batch 1) or one arm per sequence."""
        ks = [k] * self.batch if np.isscalar(k) else list(k)
        assert len(ks) == self.batch
        kk = (C.c_int32 * self.batch)(*[int(v) for v in ks])
        _check(self.L.metasd_draft(self._h, kk, gamma), self._h)

    def verify(self, gamma: int):
        _check(self.L.metasd_verify(self._h, gamma), self._h)

    def accept(self, gamma: int):
        """batch 1: (n_acc, token, mask, bd); otherwise four arrays of `batch` entries."""
        B = self.batch
        n, tok, mask, bd = np.zeros(B, np.int32), np.zeros(B, np.int32), np.zeros(B, np.uint32), np.zeros(B, np.float64)
        _check(self.L.metasd_accept(self._h, gamma, n.ctypes.data_as(C.c_void_p), tok.ctypes.data_as(C.c_void_p),
                                    mask.ctypes.data_as(C.c_void_p), bd.ctypes.data_as(C.c_void_p)), self._h)
        if B == 1:
            return int(n[0]), int(tok[0]), int(mask[0]), float(bd[0])
        return n, tok, mask, bd

    # ---- tree rounds (greedy for temperature 0, sampled otherwise): parent[i], rank[i] per node, node 0 the root
    def draft_tree(self, k: int, parent, rank):
        n = len(parent)
        assert len(rank) == n and n <= 16
        t = _Tree(n, (C.c_int32 * 16)(*[int(v) for v in parent]), (C.c_int32 * 16)(*[int(v) for v in rank]))
        _check(self.L.metasd_draft_tree(self._h, k, C.byref(t)), self._h)

    def verify_tree(self):
        _check(self.L.metasd_verify_tree(self._h), self._h)

    def accept_tree(self):
        """(n_acc, token, path): path = the accepted nodes."""
        n, tok = C.c_int32(0), C.c_int32(0)
        path = np.zeros(16, np.int32)
        _check(self.L.metasd_accept_tree(self._h, C.byref(n), C.byref(tok), path.ctypes.data_as(C.c_void_p)), self._h)
        return int(n.value), int(tok.value), [int(v) for v in path[: n.value]]

    def peek(self, what: str, gamma: int | None = None) -> torch.Tensor:
        """View of an internal device buffer: 'P' [gamma_max+1, V], 'Q' [gamma_max, V], 'hist' [max_ctx], 'bd' [gamma_max],
        'draft' [gamma_max].  batch > 1: pass the gamma of the last round; the views are P [batch, gamma+1, V],
        Q [batch, gamma, V], hist [batch, max_ctx], bd / draft [batch, gamma]."""
        code = {"P": 0, "Q": 1, "hist": 2, "bd": 3, "draft": 4, "feat": 5}[what]
        p, n = C.c_void_p(), C.c_size_t(0)
        _check(self.L.metasd_peek(self._h, code, C.byref(p), C.byref(n)), self._h)
        off = p.value - self.workspace.data_ptr()
        raw = self.workspace[off: off + n.value]
        V = self.tdesc["vocab"]
        if what == "feat":
            return raw.view(torch.float32).view(self.max_ctx, self.tdesc["d_model"])
        if self.batch > 1:
            B, g = self.batch, gamma
            if what == "hist":
                return raw.view(torch.int32).view(B, self.max_ctx)
            assert g is not None
            if what == "P":
                return raw.view(torch.float32)[: B * (g + 1) * V].view(B, g + 1, V)
            if what == "Q":
                return raw.view(torch.float32)[: B * g * V].view(B, g, V)
            if what == "draft":
                return raw.view(torch.int32)[: B * g].view(B, g)
            return raw.view(torch.float64)[: B * g].view(B, g)
        if what == "P":
            return raw.view(torch.float32).view(self.gamma_max + 1, V)
        if what == "Q":
            return raw.view(torch.float32).view(self.gamma_max, V)
        if what in ("hist", "draft"):
            return raw.view(torch.int32)
        return raw.view(torch.float64)

    def profile(self, max_records: int):
        _check(self.L.metasd_profile(self._h, max_records), self._h)

    def profile_read(self, kind: str) -> dict:
        ms, n, by = C.c_double(0), C.c_int64(0), C.c_double(0)
        _check(self.L.metasd_profile_read(self._h, {"gemm": 0, "attn": 1, "accept": 2}[kind], C.byref(ms), C.byref(n), C.byref(by)), self._h)
        return dict(ms=ms.value, launches=n.value, bytes=by.value)

    def profile_shapes(self, target_only: bool = True, max_rows: int = 64) -> list:
        """Recorded GEMM launches by shape: dicts N, K, m, launches, avg_us, bytes_per_launch, GBs."""
        n, k, m = (np.zeros(max_rows, np.int32) for _ in range(3))
        ms, by, cnt = np.zeros(max_rows, np.float64), np.zeros(max_rows, np.float64), np.zeros(max_rows, np.int64)
        rows = C.c_int32(0)
        vp = lambda a: a.ctypes.data_as(C.c_void_p)
        _check(self.L.metasd_profile_shapes(self._h, int(target_only), max_rows, vp(n), vp(k), vp(m), vp(ms), vp(cnt), vp(by), C.byref(rows)), self._h)
        out = []
        for i in range(rows.value):
            out.append(dict(N=int(n[i]), K=int(k[i]), m=int(m[i]), launches=int(cnt[i]), avg_us=ms[i] / cnt[i] * 1e3,
                            bytes_per_launch=by[i] / cnt[i], GBs=by[i] / (ms[i] * 1e-3) / 1e9 if ms[i] > 0 else 0.0))
        return out

    def state(self, model: int = -1, seq: int = 0):
        l, kv, r = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        _check(self.L.metasd_state_seq(self._h, seq, model, C.byref(l), C.byref(kv), C.byref(r)))
        return int(l.value), int(kv.value), int(r.value)

    def accept_fallbacks(self) -> int:
        n = C.c_int64(0)
        _check(self.L.metasd_accept_fallbacks(self._h, C.byref(n)))
        return int(n.value)

    # ---- convenience: one full round (select -> draft -> verify -> accept -> update)
    def round(self, gamma: int, k: int | None = None):
        kk = self.bandit_select()
        if k is not None:
            kk = k
        self.draft(kk, gamma)
        self.verify(gamma)
        n, tok, mask, bd = self.accept(gamma)
        self.bandit_update(kk, n, gamma, bd)
        return kk, n, tok, mask, bd


# ---- stand-alone kernels on caller-supplied logits

def accept_logits(P: torch.Tensor, Q: torch.Tensor, d: torch.Tensor, T: float, seed: int, rnd: int = 0, seq0: int = 0,
                  out=None, stream=None) -> dict:
    """P [rows, gamma+1, V], Q [rows, gamma, V] fp32, d [rows, gamma] int32 (all CUDA, contiguous)."""
    _require_gpu()
    rows, gamma, V = Q.shape
    assert P.shape == (rows, gamma + 1, V) and d.shape == (rows, gamma)
    assert P.is_cuda and Q.is_cuda and d.is_cuda and P.is_contiguous() and Q.is_contiguous() and d.is_contiguous()
    assert P.dtype == torch.float32 and Q.dtype == torch.float32 and d.dtype == torch.int32
    if out is None:
        dev = P.device
        out = dict(n_acc=torch.empty(rows, dtype=torch.int32, device=dev), token=torch.empty(rows, dtype=torch.int32, device=dev),
                   mask=torch.empty(rows, dtype=torch.int32, device=dev), bd=torch.empty((rows, gamma), dtype=torch.float64, device=dev),
                   scratch=torch.zeros(rows * (gamma + 1) * 336, dtype=torch.uint8, device=dev))   # zero-filled once, reusable
    _check(load_library().metasd_accept_logits(P.data_ptr(), Q.data_ptr(), d.data_ptr(), rows, gamma, V, T, seed, rnd, seq0,
                                               out["n_acc"].data_ptr(), out["token"].data_ptr(), out["mask"].data_ptr(),
                                               out["bd"].data_ptr(), out["scratch"].data_ptr(), _stream_ptr(stream)))
    return out


ACCEPT_NOALLOC_MAX_ITEMS = 4096


def accept_logits_noalloc(P: torch.Tensor, Q: torch.Tensor, d: torch.Tensor, T: float, seed: int, rnd: int, seq0: int, out: dict,
                          stream=None) -> dict:
    """metasd_accept_logits_noalloc: the caller passes inputs and the output tensors (out: n_acc, token, mask int32 [rows],
    bd float64 [rows, gamma]); the binding allocates nothing either."""
    _require_gpu()
    rows, gamma, V = Q.shape
    assert P.shape == (rows, gamma + 1, V) and d.shape == (rows, gamma)
    assert P.is_cuda and Q.is_cuda and d.is_cuda and P.is_contiguous() and Q.is_contiguous() and d.is_contiguous()
    assert P.dtype == torch.float32 and Q.dtype == torch.float32 and d.dtype == torch.int32
    _check(load_library().metasd_accept_logits_noalloc(P.data_ptr(), Q.data_ptr(), d.data_ptr(), rows, gamma, V, T, seed, rnd, seq0,
                                                       out["n_acc"].data_ptr(), out["token"].data_ptr(), out["mask"].data_ptr(),
                                                       out["bd"].data_ptr(), _stream_ptr(stream)))
    return out


def sample_logits(logits: torch.Tensor, T: float, seed: int, rnd: int = 0, pos: int = 0, seq0: int = 0, stream=None):
    _require_gpu()
    rows, V = logits.shape
    assert logits.is_cuda and logits.is_contiguous() and logits.dtype == torch.float32
    tok = torch.empty(rows, dtype=torch.int32, device=logits.device)
    _check(load_library().metasd_sample_logits(logits.data_ptr(), rows, V, T, seed, rnd, pos, seq0, tok.data_ptr(), _stream_ptr(stream)))
    return tok


STREAM_READ_SINK_WORDS = 8192


def stream_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """One plain streaming read of `src` (CUDA, contiguous) on the current stream; `sink`: int32 tensor of at least
    STREAM_READ_SINK_WORDS elements.  Asynchronous: time it with events."""
    _require_gpu()
    assert src.is_cuda and src.is_contiguous() and sink.is_cuda and sink.is_contiguous()
    assert sink.numel() * sink.element_size() >= 4 * STREAM_READ_SINK_WORDS
    _check(load_library().metasd_stream_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream_ptr()))


def philox_words(seed: int, c0_start: int, n: int, c1: int, c2: int, c3: int, device="cuda:0") -> torch.Tensor:
    _require_gpu()
    out = torch.empty((n, 4), dtype=torch.int32, device=device)
    _check(load_library().metasd_philox_words(seed, c0_start, n, c1, c2, c3, out.data_ptr(), _stream_ptr()))
    return out
