"""The C-ABI library loads and exports every symbol include/metasd.h declares; host-only entry
points (sizes, argument validation) behave as documented.  No GPU work is launched here."""
import ctypes as C
import os
import re

import pytest

import paper_2604_05417_amd as M
from paper_2604_05417_amd import binding as B
from paper_2604_05417_amd.build import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    build(force=False)
    return M.load_library()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "metasd.h")).read()
    declared = sorted(set(re.findall(r"\b(metasd_[a-z_]+)\s*\(", hdr)))
    assert len(declared) >= 19
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(M.EXPORTS) == declared


def desc(**kw):
    d = dict(n_layers=2, d_model=128, n_heads=4, n_kv_heads=4, d_ffn=512, vocab=512, act=0, dtype=0)
    d.update(kw)
    return B._desc(d)


def test_sizes_and_validation(lib):
    n = C.c_size_t(0)
    assert lib.metasd_kv_bytes(C.byref(desc()), 96, C.byref(n)) == 0
    assert n.value == 2 * 2 * 4 * 96 * 32 * 4
    assert lib.metasd_kv_bytes(C.byref(desc(dtype=1, d_model=4096, n_heads=32, n_kv_heads=32, d_ffn=11008, vocab=32000, n_layers=32)), 2048, C.byref(n)) == 0
    assert n.value == 2048 * 524288                       # 512 KiB per token for the 7B shape
    assert lib.metasd_kv_bytes(C.byref(desc(n_heads=3)), 96, C.byref(n)) == -1
    assert b"n_heads" in lib.metasd_last_error(None)
    assert lib.metasd_kv_bytes(C.byref(desc(vocab=40000)), 96, C.byref(n)) == -1
    assert lib.metasd_kv_bytes(None, 96, C.byref(n)) == -1
    cfg = B._Config(3, 4, 1, 96, 1.0, 0, 1.0, 1)
    dr = (B._Desc * 3)(desc(n_layers=1), desc(n_layers=1), desc(n_layers=1))
    assert lib.metasd_workspace_bytes(C.byref(cfg), C.byref(desc()), dr, C.byref(n)) == 0 and n.value > 0
    bad = B._Config(3, 16, 1, 96, 1.0, 0, 1.0, 1)
    assert lib.metasd_workspace_bytes(C.byref(bad), C.byref(desc()), dr, C.byref(n)) == -1
    one = n.value
    two = B._Config(3, 4, 2, 96, 1.0, 0, 1.0, 1)            # a batch of two sequences needs a larger workspace
    assert lib.metasd_workspace_bytes(C.byref(two), C.byref(desc()), dr, C.byref(n)) == 0 and n.value > one
    for batch in (0, 33):
        bad = B._Config(3, 4, batch, 96, 1.0, 0, 1.0, 1)
        assert lib.metasd_workspace_bytes(C.byref(bad), C.byref(desc()), dr, C.byref(n)) == -1
    assert b"batch" in lib.metasd_last_error(None)
    # drafter heads: the feature table (max_ctx x d_model fp32) and one estimate row per tree node come on top; one sequence only;
    # streaming caches: one sequence only, sizes not negative
    heads = B._Config(3, 4, 1, 96, 1.0, 0, 1.0, 1)
    heads.feature_heads = 1
    assert lib.metasd_workspace_bytes(C.byref(heads), C.byref(desc()), dr, C.byref(n)) == 0
    d_model = desc().d_model
    assert (96 + 16) * d_model * 4 <= n.value - one <= (96 + 16) * d_model * 4 + 2 * 256
    heads.batch = 2
    assert lib.metasd_workspace_bytes(C.byref(heads), C.byref(desc()), dr, C.byref(n)) == -1
    heads.batch, heads.feature_heads = 1, 2
    assert lib.metasd_workspace_bytes(C.byref(heads), C.byref(desc()), dr, C.byref(n)) == -1
    stream = B._Config(3, 4, 2, 96, 1.0, 0, 1.0, 1)
    stream.stream_window = 8
    assert lib.metasd_workspace_bytes(C.byref(stream), C.byref(desc()), dr, C.byref(n)) == -1
    stream.batch, stream.stream_sink = 1, -1
    assert lib.metasd_workspace_bytes(C.byref(stream), C.byref(desc()), dr, C.byref(n)) == -1
    assert lib.metasd_set_drafter_head(None, 0, None) == -1
    dr2 = (B._Desc * 3)(desc(n_layers=1), desc(n_layers=1, vocab=256), desc(n_layers=1))
    assert lib.metasd_workspace_bytes(C.byref(cfg), C.byref(desc()), dr2, C.byref(n)) == -1
    h = C.c_void_p()
    assert lib.metasd_create(C.byref(h), C.byref(cfg), C.byref(desc()), dr, None, None, None, None, None, 0, None) == -1
    assert lib.metasd_pack_weight(None, None, 16, 32, 0, None) == -1
    assert lib.metasd_accept_logits(None, None, None, 1, 1, 8, 1.0, 0, 0, 0, None, None, None, None, None, None) == -1
    assert lib.metasd_sample_logits(None, 1, 8, 1.0, 0, 0, 0, 0, None, None) == -1
    assert lib.metasd_destroy(None) == 0
    assert lib.metasd_draft(None, None, 1) == -1 and lib.metasd_verify(None, 1) == -1
    assert lib.metasd_last_error(None) is not None


def test_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        M.accept_logits(torch.zeros(1, 2, 8), torch.zeros(1, 1, 8), torch.zeros(1, 1, dtype=torch.int32), 1.0, 1)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: --gpus N with N > 1 exits with a message and starts nothing."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
