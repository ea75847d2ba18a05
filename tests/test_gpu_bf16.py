"""GPU parity of the bf16 path (MFMA skinny GEMMs on packed weights, bf16 KV cache) against the
oracle: odd shapes spanning several tiles / attention chunks with ragged tails, then the
1B-shape and 7B-shape configurations at full size on a synthetic KV prefix."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_05417_amd as M
import workloads as W
from lockstep import LockStep

pytestmark = pytest.mark.gpu
TOL = 3e-2


def oracle_models(cfg, share_kv=False, stream=None):
    """share_kv: early-exit drafters (their layer tensors are the target's) read the target's cache on the oracle side too.
    stream = (sinks, window): drafters with caches of their own keep a streaming cache."""
    td, tw = cfg["target"]
    tw_np = W.to_numpy(tw)
    cache = {id(t): a for t, a in zip(tw, tw_np) if t is not None}
    ot = oracle.Model(td, tw_np, cfg["max_ctx"])
    od = []
    for dd, dw in cfg["drafters"]:
        arrs = [None if t is None else (cache[id(t)] if id(t) in cache else W.to_numpy([t])[0]) for t in dw]
        early_exit = all(a is b for a, b in zip(dw[: 1 + 9 * dd["n_layers"]], tw))
        shared = share_kv and early_exit
        od.append(oracle.Model(dd, arrs, cfg["max_ctx"], share_kv_with=ot if shared else None, stream=None if shared else stream))
    return ot, od


def fill_kv(cfg, g, ot, od, ctx, device):
    """Same seeded synthetic KV prefix on both sides (positions [0, ctx)); drafters that share the target's cache have none."""
    models = [(cfg["target"][0], g.kv_target, ot)] + [(dd, g.kv_drafters[k], od[k]) for k, (dd, _) in enumerate(cfg["drafters"])
                                                       if not g.kv_shared[k]]
    for i, (desc, kv_gpu, om) in enumerate(models):
        k, v = W.kv_fill(desc, ctx, cfg["kv_seed"] + i, device=device)
        kv_gpu[:, 0, :, :ctx] = k.to(kv_gpu.device)
        kv_gpu[:, 1, :, :ctx] = v.to(kv_gpu.device)
        om.kv(0)[:, :, :ctx] = k.float().cpu().numpy()
        om.kv(1)[:, :, :ctx] = v.float().cpu().numpy()


def run_lockstep(cfg, T, rounds, kv_prefilled, device="cpu", swap_heads=False, share_kv=False, force_arms=None, stream=None):
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=cfg["gamma"], max_ctx=cfg["max_ctx"], temperature=T, seed=cfg["seed"],
                 ucb_beta=cfg["beta"], share_target_kv=share_kv, stream=stream)
    ot, od = oracle_models(cfg, share_kv, stream)
    if kv_prefilled:
        fill_kv(cfg, g, ot, od, len(cfg["prompt"]) - 1, device)
    g.set_context(cfg["prompt"], kv_prefilled=kv_prefilled)
    ls = LockStep(g, ot, od, cfg["prompt"], cfg["gamma"], T, cfg["seed"], cfg["beta"], logit_tol=TOL, kv_prefilled=kv_prefilled)
    for r in range(rounds):
        if swap_heads and r == rounds // 2:                # second half: the next head variant of every drafter
            for k, (dd, dw) in enumerate(cfg["drafters"]):
                hk = cfg["heads"][k][1]
                g.swap_weight(k, 2 + 9 * dd["n_layers"], M.pack_weight(hk.cuda().contiguous()))
                old = od[k]
                od[k] = oracle.Model(dd, W.to_numpy(dw[:-1]) + W.to_numpy([hk]), cfg["max_ctx"])
                od[k].kv(0)[:] = old.kv(0)                 # the head does not enter the KV cache
                od[k].kv(1)[:] = old.kv(1)
        ls.round(None if force_arms is None else force_arms[r])
    g.close()
    return ls.stats


SMALL = [
    # (target d, heads, kv heads, ffn, layers, vocab, prompt, gamma): head_dim 64/32/128, GQA, ragged everything
    dict(d_model=256, n_heads=4, d_ffn=736, n_layers=2, vocab=1040, prompt=45, gamma=5, dd_model=128, dn_heads=2, dd_ffn=160),
    dict(d_model=192, n_heads=6, d_ffn=352, n_layers=3, vocab=528, prompt=150, gamma=3, dd_model=96, dn_heads=3, dd_ffn=96),
    dict(d_model=512, n_heads=4, d_ffn=1056, n_layers=2, vocab=2000 + 16, prompt=270, gamma=7, dd_model=256, dn_heads=2, dd_ffn=288),
]


@pytest.mark.parametrize("i", range(len(SMALL)))
@pytest.mark.parametrize("T", [0.0, 1.0])
def test_small_bf16_models_real_prefill(i, T):
    s = SMALL[i]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = s["gamma"]
    cfg["max_ctx"] = s["prompt"] + 80
    st = run_lockstep(cfg, T, rounds=6, kv_prefilled=False, swap_heads=True)
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL, st
    assert st["ties_shared"] <= 1, st


def test_gqa_early_exit_drafters_real_prefill():
    """1B-shape structure (GQA 4:1, SwiGLU, early-exit drafters sharing the target's tensors), reduced width."""
    td = W.model_desc(4, 256, 8, 2, 512, 1024, W.SWIGLU, W.BF16)
    tw = W.gen_weights(td, 0)
    drafters = [W.early_exit_drafter(td, tw, e, 0.01, 100 + k) for k, e in enumerate((1, 2, 3))]
    cfg = dict(target=(td, tw), drafters=drafters, gamma=5, prompt=W.prompt_tokens(131, 1024, 3), beta=1.0, seed=1,
               max_ctx=131 + 64)
    st = run_lockstep(cfg, 1.0, rounds=6, kv_prefilled=False)
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


@pytest.mark.parametrize("T", [1.0, 0.0])
def test_config3_1b_shape_full_size(T):
    """1B-shape target at full size (16 layers, d 2048, 32/8 heads, FFN 8192, vocab 32000), K = 4
    early-exit drafters; 512-position synthetic KV prefix instead of a CPU prefill; 3 rounds, T = 1 and greedy."""
    cfg = W.config3(device="cuda")
    cfg["kv_seed"] = 7
    st = run_lockstep(cfg, T, rounds=3, kv_prefilled=True, device="cuda")
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_gqa_early_exit_drafters_share_the_target_cache(T):
    """The same structure with the drafters reading the target's cache (no cache of their own, nothing recomputed when
    the bandit switches drafters): real prefill by the target only, then rounds in which the arm changes every round,
    including a return to a drafter that sat out; 3-row, 6-row and 1-row catch-ups never happen (every drafter step is
    one row).  Compared with oracle drafters that share the oracle target's cache."""
    td = W.model_desc(4, 256, 8, 2, 512, 1024, W.SWIGLU, W.BF16)
    tw = W.gen_weights(td, 0)
    drafters = [W.early_exit_drafter(td, tw, e, 0.01, 100 + k) for k, e in enumerate((1, 2, 3))]
    cfg = dict(target=(td, tw), drafters=drafters, gamma=5, prompt=W.prompt_tokens(131, 1024, 3), beta=1.0, seed=1,
               max_ctx=131 + 80)
    st = run_lockstep(cfg, T, rounds=8, kv_prefilled=False, share_kv=True, force_arms=[None, None, None, 0, 2, 2, 1, 0])
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


def test_shared_cache_needs_the_targets_own_layers():
    """drafter_kv[k] == target_kv is only accepted for a drafter whose layer tensors are the target's first layers."""
    cfg = W.config4(n_layers=2, ctx=20, n_new=16, K=1, d_model=256, n_heads=4, d_ffn=512, vocab=1024, dd_model=256, dn_heads=4, dd_ffn=512)
    td, tw = cfg["target"]
    import ctypes as C
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=3, max_ctx=64, temperature=1.0, seed=1)      # same shapes, own weights, own cache: fine
    L = g.L
    tptr = (C.c_void_p * len(g._tw))(*g._tw)
    dptr = (C.c_void_p * len(g._dw[0]))(*g._dw[0])
    dtab = (C.POINTER(C.c_void_p) * 1)(C.cast(dptr, C.POINTER(C.c_void_p)))
    dkv = (C.c_void_p * 1)(g.kv_target.data_ptr())                                                   # ... but on the target's cache: refused
    h = C.c_void_p()
    rc = L.metasd_create(C.byref(h), C.byref(g.cfg), C.byref(g._tdesc_c), g._ddesc_c, tptr, dtab, g.kv_target.data_ptr(), dkv,
                         g.workspace.data_ptr(), g.workspace.numel(), 0)
    assert rc == -1 and b"first" in L.metasd_last_error(None)
    g.close()


def test_config3_1b_shape_shared_cache():
    """1B-shape configuration at full size with the four early-exit drafters on the target's cache (512-position synthetic
    prefix in the target's cache only: the drafters have none of their own), 5 rounds at T = 1: one per drafter and a
    return to the first."""
    cfg = W.config3(device="cuda")
    cfg["kv_seed"] = 7
    st = run_lockstep(cfg, 1.0, rounds=5, kv_prefilled=True, device="cuda", share_kv=True)
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


def test_config3_1b_shape_real_prefill():
    """The 1B-shape configuration as it is stated: the 512-token prompt is prefilled by the library
    (metasd_set_context with kv_prefilled = 0: 31 blocks of 16 rows and a ragged last one through the target;
    every drafter catches up over the whole prompt the first time it is selected) and by the oracle, then
    4 rounds at T = 1 - one per drafter - compared logit by logit."""
    cfg = W.config3(device="cuda")
    st = run_lockstep(cfg, 1.0, rounds=4, kv_prefilled=False, device="cuda")
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


def test_config4_7b_shape_full_size_across_segment_switch():
    """7B-shape target at full size (32 layers, d 4096, FFN 11008, vocab 32000, KV context 2048), K = 5
    two-layer drafters, T = 1, in the launch configuration bench.py times, run the way bench.py runs it: the
    drafters' heads are exchanged (metasd_swap_weight, all five) when the number of generated tokens crosses a
    multiple of 32.  Runs until 36 tokens are out, i.e. across the first switch; every round is compared."""
    cfg = W.config4(device="cuda")
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=cfg["gamma"], max_ctx=cfg["max_ctx"], temperature=1.0, seed=cfg["seed"],
                 ucb_beta=cfg["beta"])
    ot, od = oracle_models(cfg)
    fill_kv(cfg, g, ot, od, len(cfg["prompt"]) - 1, "cuda")
    g.set_context(cfg["prompt"], kv_prefilled=True)
    ls = LockStep(g, ot, od, cfg["prompt"], cfg["gamma"], 1.0, cfg["seed"], cfg["beta"], logit_tol=TOL, kv_prefilled=True)
    head_index = 2 + 9 * cfg["drafters"][0][0]["n_layers"]
    seg, new_tokens, switches = 0, 0, 0
    while new_tokens < 36:
        s = (new_tokens // cfg["seg_len"]) % 4
        if s != seg:
            for k, (dd, dw) in enumerate(cfg["drafters"]):
                hk = cfg["heads"][k][s]
                g.swap_weight(k, head_index, M.pack_weight(hk.cuda().contiguous()))
                old = od[k]
                od[k] = oracle.Model(dd, W.to_numpy(dw[:-1]) + W.to_numpy([hk]), cfg["max_ctx"])
                od[k].kv(0)[:] = old.kv(0)                 # the head does not enter the KV cache
                od[k].kv(1)[:] = old.kv(1)
            seg, switches = s, switches + 1
        n, tok = ls.round()
        new_tokens += n + 1
    st = ls.stats
    g.close()
    assert switches >= 1 and st["rounds"] >= 7, (switches, st["rounds"])
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


def test_config4_7b_shape_full_size_greedy():
    """The same configuration in greedy mode (T = 0: accept iff the draft token is the target's argmax), 3 rounds."""
    cfg = W.config4(device="cuda")
    st = run_lockstep(cfg, 0.0, rounds=3, kv_prefilled=True, device="cuda")
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


def test_tall_prefill_blocks_with_many_split_k_siblings():
    """A narrow model with a very wide FFN (d 256, FFN 11008): the down projection of a 16-row prefill block
    needs 12 split-K siblings for its activations to fit in LDS - more than the 8 the launch plan asks for on
    its own - so the siblings' exchange area has to be sized from the split really taken.  Real prefill of a
    40-token prompt (two full 16-row blocks and a ragged one), then rounds at gamma = 15 (16-row verification)."""
    cfg = W.config4(n_layers=1, ctx=40, n_new=64, K=2, d_model=256, n_heads=4, d_ffn=11008, vocab=1024, dd_model=128, dn_heads=2,
                    dd_ffn=160)
    cfg["gamma"] = 15
    cfg["max_ctx"] = 40 + 80
    st = run_lockstep(cfg, 1.0, rounds=3, kv_prefilled=False)
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


def test_accept_exchange_timeout_falls_back_to_one_workgroup_per_position(monkeypatch):
    """With the accept kernel's bounded wait forced to zero from the host its four workgroups per position never
    meet; the context then takes the step again with one workgroup per position: same outcome as an undisturbed
    run (same seed, prompt, round), the fallback is counted, nothing is lost."""
    s = SMALL[0]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=5, max_ctx=s["prompt"] + 80, temperature=1.0, seed=3)
    g.set_context(cfg["prompt"])
    want = [g.round(5) for _ in range(3)]
    assert g.accept_fallbacks() == 0
    g.set_context(cfg["prompt"])
    monkeypatch.setenv("METASD_ACCEPT_SPIN_LIMIT", "0")
    got = [g.round(5) for _ in range(3)]
    monkeypatch.delenv("METASD_ACCEPT_SPIN_LIMIT")
    assert g.accept_fallbacks() == 3
    for a, b in zip(want, got):
        assert a[:4] == b[:4] and abs(a[4] - b[4]) < 1e-6, (a, b)
    g.close()


@pytest.mark.skip(reason="the cooperative one-launch forward was taken out of the library: it was 2.2x slower than the "
                         "step-by-step kernels for a 7B-shape verification pass and 2.5x slower for a drafter step")
@pytest.mark.parametrize("i", [0, 2])
def test_one_launch_forward_opt_in(i, monkeypatch):
    """The cooperative one-launch forward (opt-in by environment) gives the same parity as the
    step-by-step kernels: small ragged shapes with a real prefill, T = 1."""
    monkeypatch.setenv("METASD_PERSISTENT", "1")
    s = SMALL[i]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = s["gamma"]
    cfg["max_ctx"] = s["prompt"] + 80
    st = run_lockstep(cfg, 1.0, rounds=4, kv_prefilled=False)
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


def test_long_context_small_models():
    """More than 32 attention chunks (context 4300): the fused attention-combine prologue of the drafters'
    output projection walks the chunk records beyond its first batch; synthetic KV prefix, T = 1."""
    s = SMALL[0]
    cfg = W.config4(n_layers=s["n_layers"], ctx=4300, n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"], device="cuda")
    cfg["gamma"] = 3                       # verify blocks of 4 rows: the target takes the fused-prologue path too
    cfg["max_ctx"] = 4300 + 64
    st = run_lockstep(cfg, 1.0, rounds=4, kv_prefilled=True, device="cuda")
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


def test_split_k_reduction_bounded_wait_reports_failure(monkeypatch):
    """The sibling workgroups of a residual GEMM meet through memory with bounded polls.  With the bound
    forced to zero from the host the last sibling gives up at once: every wave exits, accept reports the
    failure (-4), and after set_context the same context works again."""
    s = SMALL[0]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=5, max_ctx=s["prompt"] + 80, temperature=1.0, seed=3)
    g.set_context(cfg["prompt"])
    k, n, tok, mask, bd = g.round(5)
    assert 0 <= n <= 5
    monkeypatch.setenv("METASD_GEMM_SPIN_LIMIT", "0")
    k = g.bandit_select()
    g.draft(k, 5)
    g.verify(5)                                   # 6 rows: the general bf16 path with the reducing GEMMs
    with pytest.raises(M.MetaSDError) as e:
        g.accept(5)
    assert e.value.code == -4
    monkeypatch.delenv("METASD_GEMM_SPIN_LIMIT")
    g.set_context(cfg["prompt"])
    k, n2, tok2, mask2, bd2 = g.round(5)
    assert (n2, tok2) == (n, tok)                 # same seed, same prompt, same round index: the same outcome as the first time
    g.close()


@pytest.mark.parametrize("env", ["METASD_GEMM_REDUCE", "METASD_FUSE_SMALL", "METASD_ACCEPT_SPLIT"])
def test_step_by_step_variants_stay_in_parity(env, monkeypatch):
    """Each fused variant can be switched off from the environment (the plain kernels then run); the plain
    variants keep the same parity."""
    monkeypatch.setenv(env, "0")
    s = SMALL[0]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = s["gamma"]
    cfg["max_ctx"] = s["prompt"] + 80
    st = run_lockstep(cfg, 1.0, rounds=4, kv_prefilled=False)
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


@pytest.mark.parametrize("gamma,roll", [(3, "1"), (5, "1"), (7, "1"), (7, "0")])
def test_wide_shallow_target_residual_projections(gamma, roll, monkeypatch):
    """A target wide enough (d 3072 = 192 tiles, FFN 4096) for the residual projections without split-K -
    output projection with its input block in LDS, down projection with rolling staging - at 4, 6 and 8
    verification rows (both staging widths), and the same shape through the split-K sibling reduction."""
    monkeypatch.setenv("METASD_GEMM_ROLL", roll)
    cfg = W.config4(n_layers=2, ctx=70, n_new=64, K=2, d_model=3072, n_heads=24, d_ffn=4096, vocab=1024, dd_model=128, dn_heads=2,
                    dd_ffn=160)
    cfg["gamma"] = gamma
    cfg["max_ctx"] = 70 + 64
    st = run_lockstep(cfg, 1.0, rounds=3, kv_prefilled=False)
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st


# ---------------------------------------------------------------- streaming drafter caches (sinks + window)

@pytest.mark.parametrize("i,stream,prompt", [(0, (4, 16), None), (1, (0, 40), None), (2, (3, 100), None), (2, (130, 20), None), (2, (3, 50), 420), (0, (1, 30), 300)])
@pytest.mark.parametrize("T", [0.0, 1.0])
def test_small_bf16_streaming_drafter_caches(i, stream, prompt, T):
    """Drafters that attend to their first `sinks` positions and the last `window` positions only, and consume no more than
    that when they are switched in (real prefill: the first switch-in skips most of the prompt; arms forced so that each
    drafter sits out longer than its window and returns).  head_dim 64 / 32 / 128: the MFMA attention kernels with empty
    chunks skipped and the plain kernel; sinks inside the first chunk and reaching into the second; with the longer prompts
    one or two whole chunks lie between the sinks and the window.  Every drafter logit is
    compared with the oracle's, which masks the same way; the rest of the round as in the other lock-step tests."""
    s = dict(SMALL[i])
    if prompt:
        s["prompt"] = prompt
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = s["gamma"]
    cfg["max_ctx"] = s["prompt"] + 120
    st = run_lockstep(cfg, T, rounds=12, kv_prefilled=False, stream=stream, force_arms=[0, 0, 1, 1, 1, 1, 1, 1, 0, 0, 1, 0])
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL, st
    assert st["ties_shared"] <= 1, st


def test_streaming_caches_are_refused_for_batches_and_trees():
    cfg = W.config1_tree()
    td, tw = cfg["target"]
    with pytest.raises(M.MetaSDError) as e:
        M.MetaSD((td, tw), cfg["drafters"], gamma_max=4, max_ctx=cfg["max_ctx"], temperature=0.0, seed=1, batch=2, stream=(2, 8))
    assert e.value.code == -1
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=15, max_ctx=cfg["max_ctx"], temperature=0.0, seed=1, stream=(2, 8))
    g.set_context(cfg["prompt"])
    t = W.draft_tree("wide")
    with pytest.raises(M.MetaSDError) as e:
        g.draft_tree(0, t["parent"], t["rank"])
    assert e.value.code == -1
    g.close()
