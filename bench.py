#!/usr/bin/env python3
"""MetaSD hot-path benchmark on one MI355X.

A step is one MetaSD round - bandit select, draft (gamma tokens from the chosen drafter), verify
(one target pass over gamma+1 rows against the KV cache), accept, commit, bandit update - on the
7B-shape configuration: bf16 target (32 layers, d 4096, FFN 11008, vocab 32000, KV context 2048),
K = 5 two-layer drafters with segment-switching heads, gamma = 5, batch 1, T = 1.  All inputs are
seeded synthetic tensors resident in HBM before the timed region.

Prints ONE JSON line: verified tokens/s (sum of N_acc + 1 over the timed rounds / wall clock),
the roofline of the dominant kernel (the bf16 weight-streaming GEMMs: algorithmic bytes per launch
/ mean launch duration from HIP events attached to each dispatch on the library's stream), and the CPU oracle timed on a
bounded sample of the same workload on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic():
    """HBM bytes per GEMM launch from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "gemm_bf16_kernel_c4_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get("hbm_bytes_per_launch")
    except Exception:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--ctx", type=int, default=2048)
    ap.add_argument("--layers", type=int, default=32, help="target layers (32 = the 7B shape; fewer is NOT the benchmark)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rounds", type=int, default=8)
    ap.add_argument("--workload", default="c4", choices=["c4", "c5", "c3", "c2", "c4tree", "c4heads", "c4policies"],
                    help="c4 (default): the headline benchmark; c5: the batched configuration (32 sequences, gamma 7, KV context 4096); "
                         "c3: the 1B-shape GQA target with four early-exit drafters, real 512-token prefill; "
                         "c2: the accept kernel alone (64 rows x gamma 5 x vocab 32000); c4tree: the C4 models with multi-candidate "
                         "(tree) rounds next to chain rounds of the same depth; all but c4 are side measurements")
    ap.add_argument("--tree", default="wide", choices=["wide", "bushy"], help="c4tree: the draft tree (workloads.draft_tree)")
    ap.add_argument("--temperature", type=float, default=1.0, help="c4tree: 0 = greedy trees, otherwise sampled trees")
    ap.add_argument("--batch", type=int, default=32, help="sequences of the c5 workload")
    ap.add_argument("--stream-cache", default=None, metavar="SINKS,WINDOW",
                    help="c4 / c3 (with --own-kv): drafters keep a streaming cache (attention sinks + window; metasd_config.stream_*) "
                         "- a side measurement, not the default workload")
    ap.add_argument("--own-kv", action="store_true", help="c3: give every early-exit drafter a KV cache of its own (recomputed when it is "
                                                           "switched in) instead of letting it read the target's")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU (one process, no collectives); use --gpus 1")
    if args.workload == "c5":
        return bench_c5(args)
    if args.workload == "c2":
        return bench_c2(args)
    if args.workload == "c3":
        return bench_c3(args)
    if args.workload == "c4heads":
        return bench_c4_heads(args)
    if args.workload == "c4policies":
        return bench_c4_policies(args)
    if args.workload == "c4tree":
        return bench_c4_tree(args)

    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU available; the MetaSD library has no CPU path")
    import paper_2604_05417_amd as M
    import workloads as W

    K_steps, Wm = args.steps, args.warmup
    gamma = 5
    dev = "cuda"
    t0 = time.time()
    cfg = W.config4(device=dev, n_layers=args.layers, ctx=args.ctx)
    total_rounds = 3 * K_steps + Wm                              # timed pass + phase pass + per-launch pass
    cfg["max_ctx"] = args.ctx + (gamma + 1) * total_rounds + 16
    td, tw = cfg["target"]
    stream = tuple(int(v) for v in args.stream_cache.split(",")) if args.stream_cache else None
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=gamma, max_ctx=cfg["max_ctx"], temperature=cfg["T"],
                 seed=cfg["seed"], ucb_beta=cfg["beta"], stream=stream)
    heads = [[M.pack_weight(h.contiguous()) for h in hk] for hk in cfg["heads"]]
    head_index = 2 + 9 * cfg["drafters"][0][0]["n_layers"]

    def fill_kv(ctx):
        models = [(td, g.kv_target)] + [(dd, g.kv_drafters[k]) for k, (dd, _) in enumerate(cfg["drafters"])]
        for i, (desc, kv) in enumerate(models):
            k, v = W.kv_fill(desc, ctx, cfg["kv_seed"] + i, device=dev)
            kv[:, 0, :, :ctx] = k
            kv[:, 1, :, :ctx] = v

    fill_kv(args.ctx - 1)
    g.set_context(cfg["prompt"], kv_prefilled=True)
    # one device-to-device copy of exactly 256 MiB: the known-size kernel that the HBM counters
    # (FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc) of this same command are scaled by
    cal = torch.empty(2, 64 << 20, dtype=torch.float32, device=dev)
    cal[0].fill_(1.0)
    cal[1].copy_(cal[0])
    torch.cuda.synchronize()
    del cal
    log(f"[bench] setup {time.time() - t0:.1f}s; weights {sum(t.numel() * 2 for t in tw if t is not None) / 1e9:.2f} GB")

    state = dict(seg=0, new_tokens=0)

    def one_round():
        seg = (state["new_tokens"] // cfg["seg_len"]) % 4       # non-stationary drafters: head variant per segment
        if seg != state["seg"]:
            for k in range(g.K):
                g.swap_weight(k, head_index, heads[k][seg])
            state["seg"] = seg
        k = g.bandit_select()
        g.draft(k, gamma)
        g.verify(gamma)
        n, tok, mask, bd = g.accept(gamma)
        g.bandit_update(k, n, gamma, bd)
        state["new_tokens"] += n + 1
        return k, n, bd

    for _ in range(Wm):
        one_round()
    torch.cuda.synchronize()
    # ---- timed region: exactly K steps
    t1 = time.perf_counter()
    toks, accs, bds, arms = 0, [], [], []
    for _ in range(K_steps):
        k, n, bd = one_round()
        toks += n + 1
        accs.append(n); bds.append(bd); arms.append(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    value = toks / dt
    ms_per_step = dt / K_steps * 1e3

    # ---- phase pass: the same kind of steps with events between the three phases (no per-launch timing)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K_steps)]
    host = np.zeros((K_steps, 2))                 # seconds the host spends inside the draft and verify calls (enqueueing their launches)
    for i in range(K_steps):
        k = g.bandit_select()
        ev[i][0].record(); h0 = time.perf_counter(); g.draft(k, gamma); h1 = time.perf_counter()
        ev[i][1].record(); h2 = time.perf_counter(); g.verify(gamma); h3 = time.perf_counter()
        ev[i][2].record(); n, tok, mask, bd = g.accept(gamma)
        ev[i][3].record()
        g.bandit_update(k, n, gamma, bd)
        host[i] = (h1 - h0, h3 - h2)
    torch.cuda.synchronize()
    phase_all = np.array([[ev[i][j].elapsed_time(ev[i][j + 1]) for j in range(3)] for i in range(K_steps)])
    phase = [float(np.median(phase_all[:, j])) for j in range(3)]
    phase_p10_p90 = [[float(np.percentile(phase_all[:, j], q)) for q in (10, 90)] for j in range(3)]
    # ---- per-launch pass: HIP events attached to every dispatch of the bandwidth-bound kernels
    # (begin/end of the kernel itself, on the library's stream)
    g.profile(4096 * 4)
    for i in range(K_steps):
        one_round()
    torch.cuda.synchronize()
    pg, pa, pc = g.profile_read("gemm"), g.profile_read("attn"), g.profile_read("accept")
    shapes_target, shapes_all = g.profile_shapes(True), g.profile_shapes(False)
    g.profile(0)

    def roof(p):
        if not p["launches"]:
            return None
        per_launch_bytes = p["bytes"] / p["launches"]
        avg_ms = p["ms"] / p["launches"]
        gbs = per_launch_bytes / (avg_ms * 1e-3) / 1e9
        return dict(launches=p["launches"], avg_us=avg_ms * 1e3, bytes_per_launch=per_launch_bytes, GBs=gbs)

    rg, ra, rc = roof(pg), roof(pa), roof(pc)
    # dominant kernels: the bf16 weight-streaming GEMMs
    dom, dom_name = rg, "gemm_bf16_kernel<*> + gemm_fullk_residual_kernel + gemm_fullk_roll_residual_kernel (weight-streaming GEMMs)"
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": dom["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dom["GBs"] / HBM_PEAK_GBS, "traffic": read_traffic(),
                "avg_launch_us": dom["avg_us"], "algorithmic_bytes_per_launch": dom["bytes_per_launch"],
                "launches_per_step": dom["launches"] / K_steps}
    # verify pass as a whole against its algorithmic bytes (weights once + KV read + KV write + logits)
    n_params = sum(t.numel() for i, t in enumerate(tw) if t is not None and i != 0)
    kv_tok = 2 * td["n_layers"] * td["n_kv_heads"] * (td["d_model"] // td["n_heads"]) * 2
    l_mid = args.ctx + (Wm + 1.5 * K_steps) * (np.mean(accs) + 1)
    verify_bytes = n_params * 2 + kv_tok * l_mid + kv_tok * (gamma + 1) + (gamma + 1) * td["vocab"] * 4
    extra = {
        "verify_ms": phase[1], "draft_ms": phase[0], "accept_ms": phase[2],
        # host time inside the two asynchronous calls (median): below the GPU time of the phase means the GPU, not the host's
        # launch rate, bounds the phase
        "draft_host_ms": float(np.median(host[:, 0]) * 1e3), "verify_host_ms": float(np.median(host[:, 1]) * 1e3),
        "phase_ms_p10_p90": {"draft": phase_p10_p90[0], "verify": phase_p10_p90[1], "accept": phase_p10_p90[2]},
        "verify_hbm_frac": verify_bytes / (phase[1] * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "verify_algorithmic_GB": verify_bytes / 1e9,
        "verify_positions_per_s": (gamma + 1) / (phase[1] * 1e-3),
        "gemm_kernel": rg, "attn_kernel": ra, "accept_kernel": rc,
        # the weight-streaming GEMM launches by shape (N x K at m rows): the target's, then the drafters' (all minus the target's)
        "gemm_shapes_target": shapes_target,
        "gemm_shapes_drafters": [s for s in shapes_all if not any((s["N"], s["K"], s["m"]) == (t["N"], t["K"], t["m"]) for t in shapes_target)],
        "mean_n_acc": float(np.mean(accs)), "alpha_mean_bd": float(np.mean(bds)),
        "arm_counts": [int(x) for x in np.bincount(arms, minlength=g.K)],
    }

    try:
        # the read rate a plain streaming kernel reaches on this machine, and the dominant kernel / the verify pass against it
        ceil_gbs = read_ceiling(M, torch, dev)
        extra["read_ceiling_GBs"] = ceil_gbs
        extra["roofline_frac_of_read_ceiling"] = dom["GBs"] / ceil_gbs
        extra["verify_frac_of_read_ceiling"] = verify_bytes / (phase[1] * 1e-3) / 1e9 / ceil_gbs
    except Exception as e:
        log(f"[bench] read ceiling measurement failed: {e!r}")
    try:
        extra["accept_c2"] = accept_c2_microbench(M, W, torch, dev)
        # the same kernel on four times as many rows: the fixed tail of the dependent chain amortises
        extra["accept_c2_256rows"] = accept_c2_microbench(M, W, torch, dev, iters=100, rows=256, nsets=2)
    except Exception as e:           # a side measurement; never blocks the headline
        log(f"[bench] accept C2 microbench failed: {e!r}")
    # ---- CPU oracle on a bounded sample of the same workload (same seeded tensors, same host)
    cpu = None
    if not args.no_cpu_baseline:
        try:
            cpu = cpu_baseline(cfg, args, gamma, W)
        except Exception as e:       # the baseline is context; it never blocks the GPU result
            log(f"[bench] cpu_baseline failed: {e!r}")
    out = {
        "metric": "verified tokens/sec @1 GPU (7B-shape, gamma=5)", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": K_steps, "warmup": Wm, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"C4: 7B-shape bf16 target ({td['n_layers']} layers, d {td['d_model']}, FFN {td['d_ffn']}, "
                               f"vocab {td['vocab']}), KV context {args.ctx}, K=5 two-layer d=768 drafters with "
                               "segment-switching heads, gamma=5, batch 1, T=1, UCB beta=1, BE reward" +
                               (f"; side measurement: streaming drafter caches ({args.stream_cache} sinks,window)" if args.stream_cache else ""),
                   "gamma": gamma, "batch": 1, "ctx": args.ctx, "K": g.K},
        "roofline": roofline, "cpu_baseline": cpu, "detail": extra,
    }
    g.close()
    print(json.dumps(out), flush=True)


def bench_c5(args):
    """The batched configuration: 7B-shape target, `batch` independent sequences (own bandit, arm, KV caches) at KV
    context 4096 (unless --ctx is given), gamma = 7, T = 0.7; a step is one round of all sequences.  One JSON line."""
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU available; the MetaSD library has no CPU path")
    import paper_2604_05417_amd as M
    import workloads as W
    dev, gamma, B = "cuda", 7, args.batch
    ctx = args.ctx if args.ctx != 2048 else 4096
    K_steps, Wm = args.steps if args.steps != 64 else 6, min(args.warmup, 2)
    t0 = time.time()
    cfg = W.config4(device=dev, n_layers=args.layers, ctx=ctx)
    total = 3 * K_steps + Wm
    max_ctx = ctx + (gamma + 1) * total + 16
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=gamma, max_ctx=max_ctx, temperature=0.7, seed=cfg["seed"], ucb_beta=cfg["beta"],
                 batch=B)
    models = [(td, g.kv_target)] + [(dd, g.kv_drafters[k]) for k, (dd, _) in enumerate(cfg["drafters"])]
    for b in range(B):                                           # seeded synthetic KV prefix, different per sequence
        for i, (desc, kv) in enumerate(models):
            k, v = W.kv_fill(desc, ctx - 1, cfg["kv_seed"] + 16 * b + i, device=dev)
            kv[b, :, 0, :, : ctx - 1] = k
            kv[b, :, 1, :, : ctx - 1] = v
        g.set_context(W.prompt_tokens(ctx, td["vocab"], 3 + b), kv_prefilled=True, seq=b)
    torch.cuda.synchronize()
    log(f"[bench c5] setup {time.time() - t0:.1f}s; batch {B}, ctx {ctx}, KV {g.kv_target.numel() * 2 / 1e9:.1f} GB")

    def one_round():
        ks = [g.bandit_select(seq=b) for b in range(B)]
        g.draft(ks, gamma)
        g.verify(gamma)
        n, tok, mask, bd = g.accept(gamma)
        for b in range(B):
            g.bandit_update(ks[b], int(n[b]), gamma, float(bd[b]), seq=b)
        return n

    for _ in range(Wm):
        one_round()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    toks, accs = 0, []
    for _ in range(K_steps):
        n = one_round()
        toks += int(n.sum()) + B
        accs.append(float(n.mean()))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K_steps)]
    for i in range(K_steps):
        ks = [g.bandit_select(seq=b) for b in range(B)]
        ev[i][0].record(); g.draft(ks, gamma)
        ev[i][1].record(); g.verify(gamma)
        ev[i][2].record(); n, tok, mask, bd = g.accept(gamma)
        ev[i][3].record()
        for b in range(B):
            g.bandit_update(ks[b], int(n[b]), gamma, float(bd[b]), seq=b)
    torch.cuda.synchronize()
    phase = [float(np.median([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(K_steps)])) for j in range(3)]
    g.profile(1 << 16)
    for _ in range(K_steps):
        one_round()
    torch.cuda.synchronize()
    pg, pa, pc = g.profile_read("gemm"), g.profile_read("attn"), g.profile_read("accept")
    g.profile(0)

    def roof(p):
        if not p["launches"]:
            return None
        return dict(launches=p["launches"], avg_us=p["ms"] / p["launches"] * 1e3, bytes_per_launch=p["bytes"] / p["launches"],
                    GBs=p["bytes"] / (p["ms"] * 1e-3) / 1e9, ms_per_step=p["ms"] / K_steps)

    n_params = sum(t.numel() for i, t in enumerate(tw) if t is not None and i != 0)
    kv_tok = 2 * td["n_layers"] * td["n_kv_heads"] * (td["d_model"] // td["n_heads"]) * 2
    l_mid = ctx + (Wm + 1.5 * K_steps) * (np.mean(accs) + 1)
    verify_bytes = n_params * 2 + B * (kv_tok * l_mid + kv_tok * (gamma + 1) + (gamma + 1) * td["vocab"] * 4)
    R = B * (gamma + 1)
    out = {
        "metric": "verified tokens/sec @1 GPU (7B-shape, batched)", "value": toks / dt, "unit": "tokens/s", "n_gpus": 1,
        "steps": K_steps, "warmup": Wm, "ms_per_step": dt / K_steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"C5: 7B-shape bf16 target ({td['n_layers']} layers), {B} independent sequences with their own UCB "
                               f"bandit over K=5 two-layer drafters, KV context {ctx}, gamma=7, T=0.7; {R} verification rows",
                   "gamma": gamma, "batch": B, "ctx": ctx, "K": g.K},
        "detail": {"draft_ms": phase[0], "verify_ms": phase[1], "accept_ms": phase[2], "verify_algorithmic_GB": verify_bytes / 1e9,
                   "verify_hbm_frac": verify_bytes / (phase[1] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "verify_gemm_TFLOPs": 2.0 * R * n_params / (phase[1] * 1e-3) / 1e12,
                   "gemm_kernel": roof(pg), "attn_kernel": roof(pa), "accept_kernel": roof(pc), "mean_n_acc": float(np.mean(accs))},
    }
    g.close()
    print(json.dumps(out), flush=True)


def bench_c3(args):
    """Configuration C3: 1B-shape bf16 target (16 layers, d 2048, 32 query / 8 KV heads, FFN 8192), K = 4 early-exit
    drafters (target layers [0, l) + their own noisy head, own KV), gamma 5, T = 1; the 512-token prompt is prefilled by
    the library (first draft / verify calls).  A step is one MetaSD round.  One JSON line."""
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU available; the MetaSD library has no CPU path")
    import paper_2604_05417_amd as M
    import workloads as W
    dev = "cuda"
    K_steps, Wm = args.steps, max(args.warmup, 5)                 # the warm-up covers the prefill and the bandit's sweep
    cfg = W.config3(device=dev)
    gamma = cfg["gamma"]
    total = 3 * K_steps + Wm
    cfg["max_ctx"] = len(cfg["prompt"]) + (gamma + 1) * total + 16
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=gamma, max_ctx=cfg["max_ctx"], temperature=cfg["T"], seed=cfg["seed"],
                 ucb_beta=cfg["beta"], share_target_kv=not args.own_kv,
                 stream=tuple(int(v) for v in args.stream_cache.split(",")) if args.stream_cache else None)
    g.set_context(cfg["prompt"], kv_prefilled=False)

    def one_round():
        k = g.bandit_select()
        g.draft(k, gamma)
        g.verify(gamma)
        n, tok, mask, bd = g.accept(gamma)
        g.bandit_update(k, n, gamma, bd)
        return k, n

    for _ in range(Wm):
        one_round()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    toks, accs, arms = 0, [], []
    for _ in range(K_steps):
        k, n = one_round()
        toks += n + 1
        accs.append(n); arms.append(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K_steps)]
    for i in range(K_steps):
        k = g.bandit_select()
        ev[i][0].record(); g.draft(k, gamma)
        ev[i][1].record(); g.verify(gamma)
        ev[i][2].record(); n, tok, mask, bd = g.accept(gamma)
        ev[i][3].record()
        g.bandit_update(k, n, gamma, bd)
    torch.cuda.synchronize()
    phase = [float(np.median([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(K_steps)])) for j in range(3)]
    g.profile(1 << 16)
    for _ in range(K_steps):
        one_round()
    torch.cuda.synchronize()
    pg, pa = g.profile_read("gemm"), g.profile_read("attn")
    g.profile(0)
    n_params = sum(t.numel() for i, t in enumerate(tw) if t is not None and i != 0)
    kv_tok = 2 * td["n_layers"] * td["n_kv_heads"] * (td["d_model"] // td["n_heads"]) * 2
    l_mid = len(cfg["prompt"]) + (Wm + 1.5 * K_steps) * (np.mean(accs) + 1)
    verify_bytes = n_params * 2 + kv_tok * l_mid + kv_tok * (gamma + 1) + (gamma + 1) * td["vocab"] * 4
    gbs = pg["bytes"] / (pg["ms"] * 1e-3) / 1e9 if pg["launches"] else 0.0
    out = {"metric": "verified tokens/sec @1 GPU (1B-shape, gamma=5)", "value": toks / dt, "unit": "tokens/s", "n_gpus": 1, "steps": K_steps,
           "warmup": Wm, "ms_per_step": dt / K_steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "C3: 1B-shape bf16 target (16 layers, d 2048, 32/8 heads, FFN 8192, vocab 32000), K=4 early-exit drafters "
                                  "at layers 2/4/6/8" + (" with KV caches of their own" if args.own_kv else " reading the target's KV cache") +
                                  (f" (streaming: {args.stream_cache} sinks,window)" if args.stream_cache else "") +
                                  ", 512-token prompt prefilled on the GPU, gamma=5, T=1", "gamma": gamma, "batch": 1, "K": g.K},
           "roofline": {"bound": "hbm", "kernel": "weight-streaming GEMMs (target and drafters)", "achieved": gbs, "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None},
           "cpu_baseline": None,
           "detail": {"draft_ms": phase[0], "verify_ms": phase[1], "accept_ms": phase[2],
                      "verify_algorithmic_GB": verify_bytes / 1e9, "verify_hbm_frac": verify_bytes / (phase[1] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "gemm_launches": pg["launches"], "gemm_avg_us": pg["ms"] / max(pg["launches"], 1) * 1e3,
                      "attn_avg_us": pa["ms"] / max(pa["launches"], 1) * 1e3, "mean_n_acc": float(np.mean(accs)),
                      "arm_counts": [int(x) for x in np.bincount(arms, minlength=g.K)]}}
    g.close()
    print(json.dumps(out), flush=True)


def bench_c4_tree(args):
    """Side measurement: the C4 models (7B-shape target, five two-layer drafters, KV context 2048, heads switching per segment)
    with multi-candidate rounds over a token tree, next to chain rounds of the tree's depth in the same context."""
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU available; the MetaSD library has no CPU path")
    import paper_2604_05417_amd as M
    import workloads as W
    dev = "cuda:0"
    K_steps, Wm = args.steps, max(args.warmup, 5)
    tree = W.draft_tree(args.tree)
    n = len(tree["parent"])
    depth = [0] * n
    for i in range(1, n):
        depth[i] = depth[tree["parent"][i]] + 1
    D = max(depth)
    cfg = W.config4(device=dev, n_layers=args.layers, ctx=args.ctx)
    cfg["max_ctx"] = args.ctx + (D + 1) * 2 * (K_steps + Wm + 8) + n + 16
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=15, max_ctx=cfg["max_ctx"], temperature=args.temperature, seed=cfg["seed"],
                 ucb_beta=cfg["beta"])
    heads = [[M.pack_weight(h.contiguous()) for h in hk] for hk in cfg["heads"]]
    head_index = 2 + 9 * cfg["drafters"][0][0]["n_layers"]
    models = [(td, g.kv_target)] + [(dd, g.kv_drafters[k]) for k, (dd, _) in enumerate(cfg["drafters"])]
    for i, (desc, kv) in enumerate(models):
        k, v = W.kv_fill(desc, args.ctx - 1, cfg["kv_seed"] + i, device=dev)
        kv[:, 0, :, : args.ctx - 1] = k
        kv[:, 1, :, : args.ctx - 1] = v
    g.set_context(cfg["prompt"], kv_prefilled=True)
    state = dict(seg=0, new_tokens=0)

    def one_round(use_tree):
        seg = (state["new_tokens"] // cfg["seg_len"]) % 4
        if seg != state["seg"]:
            for k in range(g.K):
                g.swap_weight(k, head_index, heads[k][seg])
            state["seg"] = seg
        k = g.bandit_select()
        if use_tree:
            g.draft_tree(k, tree["parent"], tree["rank"])
            g.verify_tree()
            na, tok, path = g.accept_tree()
        else:
            g.draft(k, D)
            g.verify(D)
            na, tok, mask, bd = g.accept(D)
        g.bandit_update(k, na, D)
        state["new_tokens"] += na + 1
        return na

    res = {}
    for name, use_tree in (("chain", False), ("tree", True)):
        for _ in range(Wm):
            one_round(use_tree)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        accs = [one_round(use_tree) for _ in range(K_steps)]
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        res[name] = {"tokens_per_s": (sum(accs) + len(accs)) / dt, "ms_per_round": dt / K_steps * 1e3, "mean_n_acc": float(np.mean(accs))}
        # phases of a few more rounds (events between the calls)
        ph = []
        for _ in range(8):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            k = g.bandit_select()
            ev[0].record()
            if use_tree:
                g.draft_tree(k, tree["parent"], tree["rank"]); ev[1].record()
                g.verify_tree(); ev[2].record()
                na, tok, path = g.accept_tree()
            else:
                g.draft(k, D); ev[1].record()
                g.verify(D); ev[2].record()
                na, tok, mask, bd = g.accept(D)
            ev[3].record()
            g.bandit_update(k, na, D)
            torch.cuda.synchronize()
            ph.append([ev[j].elapsed_time(ev[j + 1]) for j in range(3)])
        med = np.median(np.array(ph), axis=0)
        res[name].update(draft_ms=float(med[0]), verify_ms=float(med[1]), accept_ms=float(med[2]))
    out = {"metric": "verified tokens/sec @1 GPU (7B-shape, tree rounds)", "value": res["tree"]["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
           "steps": K_steps, "warmup": Wm, "ms_per_step": res["tree"]["ms_per_round"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"C4 models, KV context {args.ctx}, batch 1, T={args.temperature}: rounds over the '{args.tree}' draft tree "
                                  f"({n} nodes, depth {D}) against chain rounds with gamma = {D}", "tree": args.tree, "nodes": n, "depth": D},
           "roofline": None, "cpu_baseline": None, "detail": res}
    print(json.dumps(out))
    g.close()
    return 0


def bench_c4_heads(args):
    """Side measurement: the C4 target (7B shape, KV context 2048, T = 1) with K = 5 one-layer drafter heads on its hidden states
    (the white-box setting of the paper's Sec. 4): head k runs the tensors of target layer k behind a W_fc of its own; chain
    rounds with gamma = 5 and rounds over the draft tree (--tree) in the same context; K/V prefix and feature prefix are seeded
    synthetic fills."""
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU available; the MetaSD library has no CPU path")
    import paper_2604_05417_amd as M
    import workloads as W
    dev = "cuda:0"
    K_steps, Wm = args.steps, max(args.warmup, 5)
    tree = W.draft_tree(args.tree)
    n = len(tree["parent"])
    depth = [0] * n
    for i in range(1, n):
        depth[i] = depth[tree["parent"][i]] + 1
    D = max(depth)
    cfg = W.config4(device=dev, n_layers=args.layers, ctx=args.ctx, K=1)
    cfg["max_ctx"] = args.ctx + (D + 1) * 2 * (K_steps + Wm + 8) + n + 16
    td, tw = cfg["target"]
    drafters, heads = [], {}
    for k in range(5):
        dd, dw, fc = W.feature_head_drafter(td, tw, k % td["n_layers"], 0.01 * W.c4_noise_scale(k, 0), 300 + k)
        drafters.append((dd, dw))
        heads[k] = fc
    g = M.MetaSD((td, tw), drafters, gamma_max=15, max_ctx=cfg["max_ctx"], temperature=1.0, seed=cfg["seed"], ucb_beta=cfg["beta"],
                 heads=heads)
    n0 = args.ctx - 1
    for i, (desc, kv) in enumerate([(td, g.kv_target)] + [(dd, g.kv_drafters[k]) for k, (dd, _) in enumerate(drafters)]):
        kk, vv = W.kv_fill(desc, n0, cfg["kv_seed"] + i, device=dev)
        kv[:, 0, :, :n0] = kk
        kv[:, 1, :, :n0] = vv
    g.set_context(cfg["prompt"], kv_prefilled=True)
    gen = torch.Generator(device="cpu").manual_seed(77)
    g.peek("feat")[:n0] = (torch.randn((n0, td["d_model"]), generator=gen) * 0.05).to(dev)

    def one_round(use_tree, ev=None):
        k = g.bandit_select()
        if ev: ev[0].record()
        if use_tree:
            g.draft_tree(k, tree["parent"], tree["rank"])
            if ev: ev[1].record()
            g.verify_tree()
            if ev: ev[2].record()
            na, tok, path = g.accept_tree()
        else:
            g.draft(k, D)
            if ev: ev[1].record()
            g.verify(D)
            if ev: ev[2].record()
            na, tok, mask, bd = g.accept(D)
        if ev: ev[3].record()
        g.bandit_update(k, na, D)
        return na

    res = {}
    for name, use_tree in (("chain", False), ("tree", True)):
        for _ in range(Wm):
            one_round(use_tree)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        accs = [one_round(use_tree) for _ in range(K_steps)]
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        ph = []
        for _ in range(8):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            one_round(use_tree, ev)
            torch.cuda.synchronize()
            ph.append([ev[j].elapsed_time(ev[j + 1]) for j in range(3)])
        med = np.median(np.array(ph), axis=0)
        res[name] = {"tokens_per_s": (sum(accs) + len(accs)) / dt, "ms_per_round": dt / K_steps * 1e3, "mean_n_acc": float(np.mean(accs)),
                     "draft_ms": float(med[0]), "verify_ms": float(med[1]), "accept_ms": float(med[2])}
    out = {"metric": "verified tokens/sec @1 GPU (7B-shape, drafter heads on hidden states)", "value": res["chain"]["tokens_per_s"],
           "unit": "tokens/s", "n_gpus": 1, "steps": K_steps, "warmup": Wm, "ms_per_step": res["chain"]["ms_per_round"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"C4 target, KV context {args.ctx}, batch 1, T=1, K=5 one-layer heads on the target's hidden states (W_fc "
                                  f"[4096, 8192] each, layer tensors shared with the target): chain rounds with gamma = {D} (value) and rounds "
                                  f"over the '{args.tree}' tree ({n} nodes, depth {D})"},
           "roofline": None, "cpu_baseline": None, "detail": res}
    print(json.dumps(out))
    g.close()
    return 0


def bench_c4_policies(args):
    """Side measurement: what the bandit is for.  The C4 workload (drafter heads exchanged every 32 generated tokens, so the
    best drafter moves) run with every drafter fixed and with each selection policy of the library, same seed, same prompt,
    same number of rounds: verified tokens/s and mean accepted length per policy."""
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU available; the MetaSD library has no CPU path")
    import paper_2604_05417_amd as M
    import workloads as W
    dev = "cuda:0"
    rounds = args.steps if args.steps != 64 else 192
    cfg = W.config4(device=dev, n_layers=args.layers, ctx=args.ctx)
    gamma = cfg["gamma"]
    cfg["max_ctx"] = args.ctx + (gamma + 1) * (rounds + 8) + 16
    td, tw = cfg["target"]
    K = len(cfg["drafters"])
    heads = [[M.pack_weight(h.contiguous()) for h in hk] for hk in cfg["heads"]]
    head_index = 2 + 9 * cfg["drafters"][0][0]["n_layers"]
    runs = [("fixed %d" % k, "ucb", k, {}) for k in range(K)] + [
        ("ucb", "ucb", None, {}), ("ducb", "ducb", None, dict(policy_param=0.95)), ("swucb", "swucb", None, dict(policy_window=32)),
        ("exp3", "exp3", None, dict(policy_param=0.1)), ("random", "random", None, {})]
    res = {}
    for name, policy, fixed, extra in runs:
        g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=gamma, max_ctx=cfg["max_ctx"], temperature=cfg["T"], seed=cfg["seed"],
                     ucb_beta=cfg["beta"], policy=policy, **extra)
        for i, (desc, kv) in enumerate([(td, g.kv_target)] + [(dd, g.kv_drafters[k]) for k, (dd, _) in enumerate(cfg["drafters"])]):
            kk, vv = W.kv_fill(desc, args.ctx - 1, cfg["kv_seed"] + i, device=dev)
            kv[:, 0, :, : args.ctx - 1] = kk
            kv[:, 1, :, : args.ctx - 1] = vv
        for k in range(K):
            g.swap_weight(k, head_index, heads[k][0])
        g.set_context(cfg["prompt"], kv_prefilled=True)
        seg, new_tokens, accs, arms = 0, 0, [], [0] * K
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(rounds):
            s_now = (new_tokens // cfg["seg_len"]) % 4
            if s_now != seg:
                for k in range(K):
                    g.swap_weight(k, head_index, heads[k][s_now])
                seg = s_now
            k = g.bandit_select()
            if fixed is not None:
                k = fixed
            g.draft(k, gamma)
            g.verify(gamma)
            n, tok, mask, bd = g.accept(gamma)
            g.bandit_update(k, n, gamma, bd)
            new_tokens += n + 1
            accs.append(n)
            arms[k] += 1
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        res[name] = {"tokens_per_s": new_tokens / dt, "mean_n_acc": float(np.mean(accs)), "ms_per_round": dt / rounds * 1e3, "arm_counts": arms}
        log(f"[bench c4policies] {name:8s} {res[name]['tokens_per_s']:7.1f} tokens/s  mean N_acc {res[name]['mean_n_acc']:.3f}  arms {arms}")
        g.close()
        del g
        torch.cuda.empty_cache()
    best_fixed = max(res["fixed %d" % k]["tokens_per_s"] for k in range(K))
    out = {"metric": "verified tokens/sec @1 GPU (7B-shape, per selection policy)", "value": res["ucb"]["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
           "steps": rounds, "warmup": 0, "ms_per_step": res["ucb"]["ms_per_round"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"C4 models, KV context {args.ctx}, batch 1, gamma {gamma}, T={cfg['T']}, {rounds} rounds per policy from the same state; "
                                  "drafter heads exchanged every 32 generated tokens (the best drafter moves)"},
           "roofline": None, "cpu_baseline": None, "detail": {"per_policy": res, "best_fixed_tokens_per_s": best_fixed}}
    print(json.dumps(out))
    return 0


def bench_c2(args):
    """The accept step alone on the C2 shape; a step = one call over 64 rows.  One JSON line; value = rows per second."""
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU available; the MetaSD library has no CPU path")
    import paper_2604_05417_amd as M
    import workloads as W
    iters = max(args.steps, 1)
    r = accept_c2_microbench(M, W, torch, "cuda", iters=iters, rows=64, nsets=4)
    ceil_gbs = read_ceiling(M, torch, "cuda")
    cpu = None
    if not args.no_cpu_baseline:
        try:                                         # the oracle's accept step on one of the input sets, same host
            import numpy as np
            import oracle
            c = W.config2(1.0, rows=64, device="cuda", variant=0)
            Ph, Qh = c["P"].cpu().numpy(), c["Q"].cpu().numpy()
            rows, gamma, V = Qh.shape
            d = np.stack([oracle.sample_batch(Qh[:, j], 1.0, oracle.uniform_batch(c["seed"], 0, rows, 0, j, 2)) for j in range(gamma)], 1).astype(np.int32)
            ua = np.stack([oracle.uniform_batch(c["seed"], 0, rows, 0, j, 0) for j in range(gamma)], 1)
            ur = oracle.uniform_batch(c["seed"], 0, rows, 0, 0, 1)
            oracle.accept_batch(Ph, Qh, d, 1.0, ua, ur)
            reps, t1 = 5, time.perf_counter()
            for _ in range(reps):
                oracle.accept_batch(Ph, Qh, d, 1.0, ua, ur)
            dt = (time.perf_counter() - t1) / reps
            cpu = {"value": rows / dt, "unit": "rows/s", "cores": oracle.num_threads(), "kind": "oracle",
                   "sample": f"the oracle's accept step on one C2 input set (64 rows), mean of {reps} calls: {dt * 1e3:.1f} ms per call"}
        except Exception as e:
            log(f"[bench c2] cpu_baseline failed: {e!r}")
    out = {"metric": "accept rows/sec @1 GPU (64 rows x gamma 5 x vocab 32000)", "value": 64 / (r["us_per_call"] * 1e-6), "unit": "rows/s",
           "n_gpus": 1, "steps": iters, "warmup": 4, "ms_per_step": r["us_per_call"] * 1e-3, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic", "config": {"workload": r["workload"]},
           "roofline": {"bound": "hbm", "kernel": "accept_split_kernel", "achieved": r["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": r["hbm_frac"], "traffic": None},
           "cpu_baseline": cpu, "detail": {"accept_c2": r, "read_ceiling_GBs": ceil_gbs, "frac_of_read_ceiling": r["GBs"] / ceil_gbs}}
    print(json.dumps(out), flush=True)


def read_ceiling(M, torch, dev, nbytes=1 << 30, iters=12):
    """Read rate of a plain streaming-read kernel on this machine (GB/s): two 1 GiB buffers read alternately, so that no
    cache holds the data; the figure the fractions of the 8 TB/s nominal peak can be set against."""
    bufs = [torch.full((nbytes // 4,), float(i + 1), dtype=torch.float32, device=dev) for i in range(2)]
    sink = torch.zeros(M.STREAM_READ_SINK_WORDS, dtype=torch.int32, device=dev)
    for b in bufs:
        M.stream_read(b, sink)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    ev[0].record()
    for i in range(iters):
        M.stream_read(bufs[i & 1], sink)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(iters))
    return nbytes / (ms[len(ms) // 2] * 1e-3) / 1e9


def accept_c2_microbench(M, W, torch, dev, iters=200, rows=64, nsets=4):
    """Accept step alone on the C2 shape (64 rows x gamma 5 x vocab 32000, fp32 logits, T = 1): four seeded
    input sets (361 MB, more than the 256 MB Infinity Cache) used in rotation; time per call = accept
    kernel + finalize kernel, from events around `iters` back-to-back calls on the current stream."""
    sets = []
    for v in range(nsets):
        c = W.config2(1.0, rows=rows, device=dev, variant=v)
        d = torch.stack([M.sample_logits(c["Q"][:, j].contiguous(), 1.0, c["seed"], v, j, 0) for j in range(c["gamma"])], 1).contiguous()
        sets.append((c["P"], c["Q"], d, M.accept_logits(c["P"], c["Q"], d, 1.0, c["seed"], v, 0)))
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        P, Q, d, out = sets[i % nsets]
        M.accept_logits(P, Q, d, 1.0, 1, i, 0, out=out)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / iters * 1e3
    # a token below 0 reports that the workgroups of a position gave up waiting for each other: such a call did not do
    # the work that is being timed (each set keeps the outputs of its last timed call)
    for v, (_, _, _, out) in enumerate(sets):
        bad = int((out["token"] < 0).sum())
        if bad:
            sys.exit(f"bench.py: accept microbenchmark invalid: {bad} of {rows} rows of input set {v} report a timed-out exchange (token < 0)")
    rows, gamma, V = sets[0][1].shape
    nbytes = rows * (2 * gamma + 1) * V * 4
    return {"workload": f"C2: {rows} rows x gamma 5 x vocab 32000 fp32, sigma 1, T 1", "us_per_call": us, "algorithmic_MB": nbytes / 1e6,
            "GBs": nbytes / us / 1e3, "hbm_frac": nbytes / us / 1e3 / HBM_PEAK_GBS, "mean_n_acc": float(sets[0][3]["n_acc"].float().mean())}


def cpu_baseline(cfg, args, gamma, W):
    """The oracle as it stands, timed on this host for a few rounds of the same configuration."""
    import numpy as np
    import oracle
    t0 = time.time()
    td, tw = cfg["target"]
    ctx = args.ctx
    max_ctx = ctx + (gamma + 1) * (args.cpu_rounds + 1) + 8
    ot = oracle.Model(td, W.to_numpy(tw), max_ctx)
    od = [oracle.Model(dd, W.to_numpy(dw), max_ctx) for dd, dw in cfg["drafters"]]
    models = [(td, ot)] + [(dd, od[k]) for k, (dd, _) in enumerate(cfg["drafters"])]
    for i, (desc, om) in enumerate(models):
        k, v = W.kv_fill(desc, ctx - 1, cfg["kv_seed"] + i, device="cuda")
        om.kv(0)[:, :, : ctx - 1] = k.float().cpu().numpy()
        om.kv(1)[:, :, : ctx - 1] = v.float().cpu().numpy()
    log(f"[bench] cpu_baseline setup {time.time() - t0:.1f}s")
    K = len(od)
    hist = np.zeros(max_ctx, np.int32)
    hist[:ctx] = cfg["prompt"]
    st = oracle.SdState(hist=hist, l=ctx, c=[ctx - 1] * K)
    bandit = oracle.Ucb(K, cfg["beta"])
    t1 = time.perf_counter()
    toks = 0
    for _ in range(args.cpu_rounds):
        k = bandit.select()
        r = oracle.sd_round(ot, od[k], k, st, gamma, cfg["T"], cfg["seed"])
        bandit.update(k, oracle.reward_be(r["n_acc"], gamma))
        toks += r["n_acc"] + 1
    dt = time.perf_counter() - t1
    return {"value": toks / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{args.cpu_rounds} MetaSD rounds of the same C4 workload (same seeded weights and KV prefix): "
                      f"{toks} tokens in {dt:.1f} s"}


if __name__ == "__main__":
    main()
