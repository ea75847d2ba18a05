"""GPU parity of batched contexts (several independent sequences per context, each with its own
bandit, drafter choice, KV caches and Philox sequence id) against the oracle: every sequence is
compared round by round with its own oracle models (see lockstep.py).  Prompts have different
lengths, so blocks are ragged; the arms differ between sequences, so drafters run on subsets."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_05417_amd as M
import workloads as W
from lockstep import BatchLockStep, LockStep
from test_gpu_bf16 import SMALL, TOL, oracle_models

pytestmark = pytest.mark.gpu


def batch_pair(cfg, T, prompts, logit_tol, reward="BE", kv_prefilled=False, policy="ucb", share_kv=False, **kw):
    td, tw = cfg["target"]
    B = len(prompts)
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=cfg["gamma"], max_ctx=cfg["max_ctx"], temperature=T, seed=cfg["seed"],
                 ucb_beta=cfg["beta"], reward=reward, batch=B, policy=policy, share_target_kv=share_kv, **kw)
    seqs = []
    for b, p in enumerate(prompts):
        ot, od = oracle_models(cfg, share_kv)           # own KV caches per sequence
        seqs.append((ot, od))
    return g, seqs


def make_lockstep(g, cfg, seqs, prompts, T, tol, reward="BE", kv_prefilled=False):
    out = []
    for b, (p, (ot, od)) in enumerate(zip(prompts, seqs)):
        g.set_context(p, kv_prefilled=kv_prefilled, seq=b)
        out.append(LockStep(g, ot, od, p, cfg["gamma"], T, cfg["seed"], cfg["beta"], logit_tol=tol, kv_prefilled=kv_prefilled,
                            reward=reward, seq=b))
    return BatchLockStep(g, out)


def test_new_query_for_one_sequence_between_rounds():
    """One sequence of a batch gets a new query (metasd_set_context) after four rounds while the others carry on:
    its bandit and its round counter - the round word of its Philox counters - restart, those of the other
    sequences do not, so no sequence ever re-uses a counter.  Every sequence stays in lock-step with its oracle
    (which counts its own rounds).  Between draft and accept a new context is refused."""
    cfg = W.config1()
    prompts = [cfg["prompt"], W.prompt_tokens(9, 512, 11), W.prompt_tokens(23, 512, 12)]
    g, seqs = batch_pair(cfg, 1.0, prompts, 1e-4)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, 1e-4)
    for r in range(4):
        bl.round()
    ks = [g.bandit_select(seq=b) for b in range(3)]
    g.draft(ks, cfg["gamma"])
    with pytest.raises(M.MetaSDError) as e:                 # a round is in flight
        g.set_context(prompts[0], seq=0)
    assert e.value.code == -3
    g.verify(cfg["gamma"])
    n, tok, mask, bd = g.accept(cfg["gamma"])
    g.close()
    # the same again, this time with the new query placed between two rounds
    g, seqs = batch_pair(cfg, 1.0, prompts, 1e-4)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, 1e-4)
    for r in range(4):
        bl.round()
    p_new = W.prompt_tokens(14, 512, 77)
    ot, od = oracle_models(cfg)
    g.set_context(p_new, seq=1)
    bl.seqs[1] = LockStep(g, ot, od, p_new, cfg["gamma"], 1.0, cfg["seed"], cfg["beta"], logit_tol=1e-4, seq=1)
    assert g.state(-1, seq=1)[2] == 0 and g.state(-1, seq=0)[2] == 4 and g.state(-1, seq=2)[2] == 4
    for r in range(5):
        ks, _ = bl.round()
        if r < 3:
            assert ks[1] == r                                # the re-set sequence sweeps its arms again (Alg. 2)
    for ls in bl.seqs:
        st = ls.stats
        assert st["mismatch_own"] == 0 and st["ties_own"] + st["ties_shared"] <= 1, st
    g.close()


@pytest.mark.parametrize("T,reward", [(0.0, "BE"), (1.0, "BD")])
def test_fp32_batch_of_three(T, reward):
    """Tiny fp32 configuration, three sequences with prompts of 16, 9 and 23 tokens, real prefill."""
    cfg = W.config1()
    prompts = [cfg["prompt"], W.prompt_tokens(9, 512, 11), W.prompt_tokens(23, 512, 12)]
    g, seqs = batch_pair(cfg, T, prompts, 1e-4, reward)
    bl = make_lockstep(g, cfg, seqs, prompts, T, 1e-4, reward)
    arms = []
    for r in range(10):
        force = None if r < 5 else [(r + b) % 3 for b in range(3)]       # later rounds: three different arms in one round
        ks, _ = bl.round(force)
        arms.append(ks)
    for ls in bl.seqs:
        st = ls.stats
        assert st["mismatch_own"] == 0 and st["ties_own"] + st["ties_shared"] <= 1, st
        assert st["max_dp"] <= 1e-4 and st["max_dq"] <= 1e-4
    assert arms[0] == [0, 0, 0] and arms[1] == [1, 1, 1] and arms[2] == [2, 2, 2]       # Alg. 2's initial sweep, per sequence
    if T == 0.0:                                                                         # lossless, sequence by sequence
        for b, ls in enumerate(bl.seqs):
            ref = oracle.ar_decode(oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"]), prompts[b], 10, T=0.0)
            assert np.array_equal(ls.hist[len(prompts[b]): len(prompts[b]) + 10], ref)
    g.close()


def test_fp32_batch_of_six_more_than_sixteen_rows():
    """fp32 models with a verification block of 6 x 5 = 30 rows (the fp32 GEMM runs per 16-row block)."""
    cfg = W.config1()
    prompts = [W.prompt_tokens(5 + 3 * b, 512, 20 + b) for b in range(6)]
    g, seqs = batch_pair(cfg, 1.0, prompts, 1e-4)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, 1e-4)
    for r in range(5):
        bl.round()
    for ls in bl.seqs:
        st = ls.stats
        assert st["mismatch_own"] == 0 and st["ties_own"] + st["ties_shared"] <= 1, st
        assert st["max_dp"] <= 1e-4 and st["max_dq"] <= 1e-4
    g.close()


@pytest.mark.parametrize("share_kv", [False, True])
def test_bf16_gqa_early_exit_batch(share_kv):
    """Grouped-query attention (8 query heads on 2 KV heads) and early-exit drafters that share the target's
    tensors, 5 sequences x 6 rows, real prefill of prompts of different lengths; with caches of their own, and
    reading the target's (each sequence's drafter reads that sequence's target cache)."""
    td = W.model_desc(4, 256, 8, 2, 512, 1024, W.SWIGLU, W.BF16)
    tw = W.gen_weights(td, 0)
    drafters = [W.early_exit_drafter(td, tw, e, 0.01, 100 + k) for k, e in enumerate((1, 2, 3))]
    cfg = dict(target=(td, tw), drafters=drafters, gamma=5, beta=1.0, seed=1, max_ctx=150 + 64)
    prompts = [W.prompt_tokens(150 - 29 * b, 1024, 40 + b) for b in range(5)]
    g, seqs = batch_pair(cfg, 1.0, prompts, TOL, share_kv=share_kv)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, TOL)
    for r in range(5):
        bl.round(None if r < 3 else [(b + r) % 3 for b in range(5)])
    for ls in bl.seqs:
        st = ls.stats
        assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st
    g.close()


@pytest.mark.parametrize("B,i", [(2, 0), (5, 0), (12, 1), (7, 2)])
def test_bf16_batches_span_the_gemm_variants(B, i):
    """Small bf16 models: 2 x 6 = 12 rows (single-tile GEMM), 5 x 6 = 30 and 7 x 8 = 56 rows (64-row variant),
    12 x 4 = 48; prompts of different lengths (ragged catch-up blocks, several attention chunks)."""
    s = SMALL[i]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = s["gamma"]
    cfg["max_ctx"] = s["prompt"] + 80
    prompts = [W.prompt_tokens(max(2, s["prompt"] - 17 * b), s["vocab"], 30 + b) for b in range(B)]
    g, seqs = batch_pair(cfg, 1.0, prompts, TOL)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, TOL)
    for r in range(4):
        force = None if r < 2 else [(b + r) % 2 for b in range(B)]      # after the sweep: mixed arms in one round
        bl.round(force)
    for ls in bl.seqs:
        st = ls.stats
        assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st
    g.close()


@pytest.mark.parametrize("rows", [(11, 6), (20, 7), (32, 8)])
def test_bf16_wide_blocks(rows):
    """More rows than one 64-row workgroup tile holds: 11 x 7 = 77 rows (128-row variant), 20 x 8 = 160 rows
    (256-row variant) and the largest batch, 32 x 9 = 288 rows (two passes of the 256-row variant); real prefill."""
    B, gamma = rows
    s = SMALL[0]
    cfg = W.config4(n_layers=2, ctx=140, n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"], d_ffn=s["d_ffn"], vocab=s["vocab"],
                    dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = gamma
    cfg["max_ctx"] = 140 + 40
    prompts = [W.prompt_tokens(140 - (b % 3), s["vocab"], 50 + b) for b in range(B)]
    g, seqs = batch_pair(cfg, 1.0, prompts, TOL)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, TOL)
    for r in range(2):
        bl.round()
    for ls in bl.seqs:
        st = ls.stats
        assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st
    g.close()


@pytest.mark.parametrize("tpb", [4, 6, 12])
def test_bf16_wide_blocks_other_tile_counts(tpb, monkeypatch):
    """The 256-row GEMM variant with 4, 6 and 12 feature tiles per workgroup (12: the form whose activations go straight from memory into LDS) (the cost model picks them for the 7B shapes;
    here forced at context creation): 20 x 8 = 160 rows, tile counts that are no multiple of 4 or 6 (ragged last group)."""
    monkeypatch.setenv("METASD_ROWS_TPB", str(tpb))
    s = SMALL[0]
    cfg = W.config4(n_layers=2, ctx=140, n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"], d_ffn=s["d_ffn"], vocab=s["vocab"],
                    dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = 7
    cfg["max_ctx"] = 140 + 40
    prompts = [W.prompt_tokens(140 - (b % 3), s["vocab"], 50 + b) for b in range(20)]
    g, seqs = batch_pair(cfg, 1.0, prompts, TOL)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, TOL)
    for r in range(2):
        bl.round()
    for ls in bl.seqs:
        st = ls.stats
        assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st
    g.close()


@pytest.mark.parametrize("i,cpw", [(2, 2), (1, 3), (0, 4)])
def test_bf16_attention_several_chunks_per_workgroup(i, cpw, monkeypatch):
    """The batched attention kernel walking several 128-position chunks per workgroup with a running softmax state
    (used for large batches of long contexts; here forced at context creation): head_dim 128 / 32 / 64, prompts of
    270, 150 and 45 tokens and shorter ones, so sequences end in different chunk groups and the last group is ragged."""
    monkeypatch.setenv("METASD_ATT_CPW", str(cpw))
    s = SMALL[i]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = s["gamma"]
    cfg["max_ctx"] = s["prompt"] + 80
    prompts = [W.prompt_tokens(max(2, s["prompt"] - 61 * b), s["vocab"], 70 + b) for b in range(4)]
    g, seqs = batch_pair(cfg, 1.0, prompts, TOL)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, TOL)
    for r in range(3):
        bl.round()
    for ls in bl.seqs:
        st = ls.stats
        assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st
    g.close()


@pytest.mark.parametrize("grouped", ["0", "1"])
def test_bf16_mixed_arms_grouped_and_per_arm_drafting(grouped, monkeypatch):
    """Sequences on different drafters in the same round: with drafters of one shape (bf16, head_dim >= 64) a draft step
    is one forward for all arms (weights and caches picked per segment), otherwise - or with the switch off - one
    forward per arm.  Both against the oracle, arms forced so that 2 and 3 arms share a round and drafters that sat
    out a round have several tokens to catch up on."""
    monkeypatch.setenv("METASD_DRAFT_GROUPED", grouped)
    s = SMALL[0]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=3, d_model=s["d_model"], n_heads=s["n_heads"],
                    d_ffn=s["d_ffn"], vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["gamma"] = 4
    cfg["max_ctx"] = s["prompt"] + 80
    B = 7
    prompts = [W.prompt_tokens(max(2, s["prompt"] - 5 * b), s["vocab"], 90 + b) for b in range(B)]
    g, seqs = batch_pair(cfg, 1.0, prompts, TOL)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, TOL)
    plans = [[b % 3 for b in range(B)], [(b // 2) % 3 for b in range(B)], [b % 2 for b in range(B)], [2 - b % 3 for b in range(B)],
             [(b + 1) % 3 for b in range(B)]]
    for plan in plans:
        bl.round(plan)
    for ls in bl.seqs:
        st = ls.stats
        assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st
    g.close()


def test_batch_limits_and_errors():
    cfg = W.config1()
    td, tw = cfg["target"]
    with pytest.raises(M.MetaSDError) as e:
        M.MetaSD((td, tw), cfg["drafters"], gamma_max=4, max_ctx=64, temperature=1.0, seed=1, batch=33)
    assert e.value.code == -1
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=4, max_ctx=64, temperature=1.0, seed=1, batch=2)
    g.set_context(cfg["prompt"], seq=0)
    with pytest.raises(M.MetaSDError) as e:
        g.draft([0, 0], 4)                                 # sequence 1 has no context yet
    assert e.value.code == -3
    with pytest.raises(M.MetaSDError) as e:
        g.set_context(cfg["prompt"], seq=2)
    assert e.value.code == -1
    g.set_context(cfg["prompt"][:5], seq=1)
    with pytest.raises(M.MetaSDError) as e:
        g.draft([0, 3], 4)                                 # K = 3
    assert e.value.code == -1
    g.draft([2, 1], 3)
    g.verify(3)
    n, tok, mask, bd = g.accept(3)
    assert n.shape == (2,) and ((0 <= n) & (n <= 3)).all() and ((0 <= tok) & (tok < 512)).all()
    assert g.state(-1, seq=0)[0] == 16 + n[0] + 1 and g.state(-1, seq=1)[0] == 5 + n[1] + 1
    # identical sequences in one batch differ only by their Philox sequence id: same logits, independent draws
    g.close()


def test_identical_prompts_share_logits_not_draws():
    """Two sequences with the same prompt and arm see the same drafter and target logits in round 0
    (bit for bit: the rows go through the same kernels) but draw with different uniforms."""
    cfg = W.config1()
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=4, max_ctx=96, temperature=1.0, seed=5, batch=2)
    for b in range(2):
        g.set_context(cfg["prompt"], seq=b)
    g.draft([1, 1], 4)
    Q = g.peek("Q", 4).cpu().numpy()
    d = g.peek("draft", 4).cpu().numpy()
    assert np.array_equal(Q[0, 0], Q[1, 0])                # first step: same context on both
    assert not np.array_equal(d[0], d[1])                  # sequence ids 0 and 1 give different uniforms
    g.verify(4)
    g.accept(4)
    g.close()


def test_config5_full_size_sampled_sequences():
    """The batched configuration at full size - 7B-shape target, 32 sequences, KV context 4096 (synthetic
    prefix, different per sequence), gamma = 7, T = 0.7, 256 verification rows, in the launch
    configuration `bench.py --workload c5` times - with eight of the 32 sequences (the first, the last and six
    spread over the row range) followed by the oracle: drafter and target logits, accept outcome, commit.
    The oracle models of the followed sequences share one copy of the weights; each has its own caches."""
    B, gamma, ctx, T = 32, 7, 4096, 0.7
    cfg = W.config4(device="cuda", ctx=ctx)
    cfg["gamma"], cfg["max_ctx"] = gamma, ctx + 2 * (gamma + 1) + 8
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=gamma, max_ctx=cfg["max_ctx"], temperature=T, seed=cfg["seed"],
                 ucb_beta=cfg["beta"], batch=B)
    sampled = (0, 5, 9, 14, 18, 23, 27, 31)
    tw_np = W.to_numpy(tw)                                  # shared by the oracle models of both sampled sequences
    dw_np = [W.to_numpy(dw) for _, dw in cfg["drafters"]]
    models = [(td, g.kv_target)] + [(dd, g.kv_drafters[k]) for k, (dd, _) in enumerate(cfg["drafters"])]
    seqs = {}
    for b in range(B):
        prompt = W.prompt_tokens(ctx, td["vocab"], 3 + b)
        om = None
        if b in sampled:
            om = [oracle.Model(td, tw_np, cfg["max_ctx"])] + [oracle.Model(dd, dw_np[k], cfg["max_ctx"]) for k, (dd, _) in enumerate(cfg["drafters"])]
        for i, (desc, kv) in enumerate(models):
            k, v = W.kv_fill(desc, ctx - 1, cfg["kv_seed"] + 16 * b + i, device="cuda")
            kv[b, :, 0, :, : ctx - 1] = k
            kv[b, :, 1, :, : ctx - 1] = v
            if om is not None:
                om[i].kv(0)[:, :, : ctx - 1] = k.float().cpu().numpy()
                om[i].kv(1)[:, :, : ctx - 1] = v.float().cpu().numpy()
        g.set_context(prompt, kv_prefilled=True, seq=b)
        if om is not None:
            seqs[b] = LockStep(g, om[0], om[1:], prompt, gamma, T, cfg["seed"], cfg["beta"], logit_tol=TOL, kv_prefilled=True, seq=b)
    for r in range(2):
        ks = [seqs[b].select() if b in seqs else g.bandit_select(seq=b) for b in range(B)]
        if r == 1:                                          # second round: the sequences of a batch use different drafters
            ks = [(k + b) % g.K for b, k in enumerate(ks)]
        l0 = {b: ls.l for b, ls in seqs.items()}
        g.draft(ks, gamma)
        g.verify(gamma)
        n, tok, mask, bd = g.accept(gamma)
        P, Q = g.peek("P", gamma), g.peek("Q", gamma)
        D, H = g.peek("draft", gamma).cpu().numpy().copy(), g.peek("hist").cpu().numpy()
        for b in range(B):
            if b in seqs:
                l = l0[b]
                seqs[b].check(ks[b], int(n[b]), int(tok[b]), int(mask[b]), float(bd[b]), P[b].cpu().numpy(), Q[b].cpu().numpy(), D[b],
                              H[b, l: l + gamma + 1])
            else:
                assert 0 <= n[b] <= gamma and 0 <= tok[b] < td["vocab"]
                g.bandit_update(ks[b], int(n[b]), gamma, float(bd[b]), seq=b)
    for ls in seqs.values():
        st = ls.stats
        print("C5 sampled sequence", ls.seq, {k: st[k] for k in ("max_dp", "max_dq", "ties_shared", "ties_own", "mismatch_own")})
        assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st
    g.close()


def test_largest_batch_and_draft_length():
    """The upper ends of the ranges at a shape the oracle follows in seconds: 32 sequences (METASD_MAX_BATCH) with
    gamma = 15 (METASD_MAX_GAMMA): 512 verification rows - two passes of the many-row GEMM - ragged prompts, every
    sequence followed by its own oracle for three rounds, the third with three different arms in flight."""
    cfg = W.config4(n_layers=2, ctx=40, n_new=64, K=3, d_model=256, n_heads=4, d_ffn=512, vocab=1024, dd_model=128, dn_heads=2, dd_ffn=256)
    cfg["gamma"], cfg["max_ctx"] = 15, 40 + 64
    prompts = [W.prompt_tokens(40 - b, 1024, 90 + b) for b in range(32)]
    g, seqs = batch_pair(cfg, 1.0, prompts, TOL)
    bl = make_lockstep(g, cfg, seqs, prompts, 1.0, TOL)
    for r in range(3):
        bl.round(None if r < 2 else [(b + r) % 3 for b in range(32)])
    for ls in bl.seqs:
        st = ls.stats
        assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties_shared"] <= 1, st
    g.close()
