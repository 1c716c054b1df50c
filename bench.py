#!/usr/bin/env python3
"""Benchmark of the EESD hot path on one MI355X.

A *step* is one whole `eesd_generate` call: prefill of the prompt, then decoding rounds
(K draft steps chosen by the Beta-posterior controller, one (K+1)-token verification,
accept / resample, KV rollback) until `max_new` tokens exist.  Inputs (random bf16 weights
of the named LLaMA-2 shape, a uniform-random prompt) are resident in HBM before the timed
region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 70b|13b|13b-long|tiny]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: (shape key, weight seed, prompt tokens, new tokens, k_cap)
    "70b": ("LLAMA70B", 2, 512, 256, 10),
    "13b": ("LLAMA13B", 1, 256, 256, 10),
    "13b-long": ("LLAMA13B", 1, 3840, 256, 10),
    "tiny": ("TINY", 0, 32, 64, 5),
}
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def pass_bytes(shape, n_layers_run, with_head, kv_tokens, si):
    """Algorithmic bytes of one pass: every weight of the layers it runs once, its LM head,
    and the cached keys/values it attends over."""
    b = n_layers_run * si.layer_bytes(shape) + (si.head_bytes(shape) if with_head else 0)
    b += n_layers_run * kv_tokens * si.kv_bytes_per_token_layer(shape)
    return b


def oracle_sample_weights(w_gpu, shape, si):
    """Host copy (fp32 numpy, row-major) of what the CPU baseline runs on: the first 2 layers, the early-exit
    layer, the heads.  Taken before the GPU copy is rearranged."""
    sh = si.reduced_depth(shape, 2, 1)
    sub = dict(shape=sh, tok_emb=w_gpu["tok_emb"], layers=w_gpu["layers"][:2], final_norm=w_gpu["final_norm"],
               lm_head=w_gpu["lm_head"], ee_layer=w_gpu["ee_layer"], ee_norm=w_gpu["ee_norm"], ee_head=w_gpu["ee_head"])
    return si.weights_to_numpy(sub)


def _oracle_rounds(w, temperature, si, budget_s, max_rounds):
    """A few rounds (1 draft step + 1 two-row verify) of the oracle on the depth-reduced weights: mean seconds per pass."""
    from oracle import eesd_oracle as orc
    sh = w["shape"]
    o = orc.OracleEESD(w, max_seq=64, temperature=temperature, seed=0, k_cap=4)
    o.prefill(si.make_prompt(4, sh["vocab"], 0))
    t_d, t_v, rounds = 0.0, 0.0, 0
    t_start = time.perf_counter()
    while rounds < 2 or (time.perf_counter() - t_start < budget_s and rounds < max_rounds):
        t0 = time.perf_counter()
        o.draft_step()
        t1 = time.perf_counter()
        o.verify()
        t2 = time.perf_counter()
        a, y = o.accept()
        o.rollback(a, y)
        t_d += t1 - t0
        t_v += t2 - t1
        rounds += 1
    return t_d / rounds, t_v / rounds, rounds


def cpu_baseline(w, shape, temperature, mean_k, mean_commit, si):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample: the same
    weights at depth L=2, N=1, a few rounds; per-parameter time scaled to the full depth.  Two legs: the
    threads numpy's BLAS takes by itself, and one thread."""
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        cores = os.cpu_count() or 1
    try:
        import psutil
        ram_gb = psutil.virtual_memory().total / 2 ** 30
    except Exception:
        ram_gb = None
    sh = w["shape"]
    p_layer, p_head = si.layer_param_count(sh), sh["vocab"] * sh["d_model"]
    p_kv = 2 * sh["n_kv_heads"] * sh["head_dim"] * sh["d_model"]
    L, N = shape["n_layers"], shape["n_draft_layers"]

    def scale(td, tv):
        c1 = td / (2 * p_layer + p_head)              # seconds per parameter, one row
        c2 = tv / (2 * p_layer + p_kv + p_head)       # seconds per parameter, two rows
        t_draft_full = c1 * ((N + 1) * p_layer + p_head)
        t_verify_full = c2 * (L * p_layer + p_kv + p_head)
        return mean_commit / (mean_k * t_draft_full + t_verify_full), t_draft_full, t_verify_full

    td, tv, rounds = _oracle_rounds(w, temperature, si, 10.0, 6)
    tok_s, t_draft_full, t_verify_full = scale(td, tv)
    out = dict(value=tok_s, unit="tokens/s", cores=int(cores), kind="oracle",
               sample=f"{rounds} rounds (1 draft step + 1 two-row verify) of the fp64 numpy oracle on the first 2 layers "
                      f"+ early-exit layer + heads of the same weights; seconds per parameter scaled to L={L}, N={N} "
                      f"with the GPU run's mean K={mean_k:.2f} and {mean_commit:.2f} tokens per round (depth-reduced because an fp64 "
                      f"pass over all {L} layers takes minutes per token on the host; host RAM {ram_gb:.0f} GiB)" if ram_gb else "",
               draft_step_s=t_draft_full, verify_s=t_verify_full, host_ram_GiB=ram_gb)
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            td1, tv1, r1 = _oracle_rounds(w, temperature, si, 8.0, 2)
        tok1, d1, v1 = scale(td1, tv1)
        out["single_thread"] = dict(value=tok1, unit="tokens/s", cores=1, draft_step_s=d1, verify_s=v1, sample=f"{r1} rounds, same scaling")
    return out


def latency_sweep(ctx, torch, cache_tokens, ks, shape, si, pk=None):
    """Draft-step, verify-pass and accept latency for fixed K over a cache of `cache_tokens` positions
    (filled with a deterministic pattern: attention cost depends on the shape only)."""
    res = {}
    L = shape["n_layers"]
    for K in ks:
        td = tv = ta = 0.0
        reps = 5
        for r in range(reps + 1):
            ctx.fill_cache(cache_tokens, 1)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            ev[0].record()
            for _ in range(K):
                ctx.draft_step(sync=False)
            ev[1].record()
            ctx.verify()
            ev[2].record()
            ctx.accept()
            ev[3].record()
            torch.cuda.synchronize()
            ctx.rollback_forced(0, 1)
            if r:
                td += ev[0].elapsed_time(ev[1])
                tv += ev[1].elapsed_time(ev[2])
                ta += ev[2].elapsed_time(ev[3])
        b_verify = pass_bytes(shape, L, True, cache_tokens, si)
        res[str(K + 1)] = {"verify_rows": K + 1, "verify_ms": tv / reps, "verify_GBps": b_verify / (tv / reps * 1e-3) / 1e9,
                           "verify_frac_of_peak": b_verify / (tv / reps * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "accept_us": ta / reps * 1e3, "draft_step_ms": (td / reps / K) if K else None}
        if pk is not None:
            res[str(K + 1)]["accept_all_rows_us"] = accept_walk_us(pk, torch, K, shape["vocab"])
    return res


def accept_walk_us(pk, torch, K, vocab, reps=5):
    """The verification tail when every draft is accepted (all K + 1 rows are walked; `accept_us` above is the run's own
    decision, which with random weights stops at the first row): the library's accept on synthetic bf16 logit rows whose
    draft distribution equals the target's, so that u q < p holds for every draft.  Host-timed, includes the call's
    synchronisation."""
    g = torch.Generator(device="cpu").manual_seed(K)
    logits = (torch.randn(K + 1, vocab, generator=g) * 2.0).to(torch.bfloat16).cuda()
    q_rows = torch.softmax(logits[:max(K, 1)].float(), dim=-1).contiguous()
    p_rows = torch.empty(K + 1, vocab, device="cuda")
    drafts = torch.randint(0, vocab, (K,), generator=g).to(torch.int32).cuda()
    u = [0.5] * (K + 1)
    a, _ = pk.op_accept_logits(logits, p_rows, q_rows, drafts, u, 1.0)
    assert a == K, "synthetic rows were meant to accept every draft"
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        pk.op_accept_logits(logits, p_rows, q_rows, drafts, u, 1.0)
    return (time.perf_counter() - t0) / reps * 1e6


def summarise(stats, shape, n_prompt, max_new, bf16, si):
    """Per-pass figures of a list of eesd_generate statistics."""
    st = stats[-1]
    rounds = sum(s.rounds for s in stats)
    drafted = sum(s.drafted for s in stats)
    accepted = sum(s.accepted for s in stats)
    mean_k = drafted / max(1, rounds)
    mean_commit = (accepted + rounds) / max(1, rounds)
    v_d = accepted / max(1, drafted)       # Section 4.1 "Metrics", over all steps
    r_d = accepted / max(1, sum(s.generated for s in stats))
    ms_draft = sum(s.ms_draft for s in stats) / max(1, drafted)
    ms_verify = sum(s.ms_verify for s in stats) / max(1, rounds)
    ms_accept = sum(s.ms_accept for s in stats) / max(1, rounds)
    ms_other = sum(s.ms_other for s in stats) / max(1, rounds)       # host turn-around between rounds
    N, L = shape["n_draft_layers"], shape["n_layers"]
    ctx_mid = n_prompt + max_new // 2      # bytes are taken at the middle of the generation
    b_draft = pass_bytes(shape, N + 1, True, ctx_mid, si)
    b_verify = pass_bytes(shape, L, True, ctx_mid, si) + 2 * shape["n_kv_heads"] * shape["head_dim"] * shape["d_model"] * (2 if bf16 else 4)
    out = {"draft_step_ms": ms_draft, "verify_ms": ms_verify, "accept_ms": ms_accept, "host_gap_ms_per_round": ms_other,
           "draft_step_GBps": b_draft / (ms_draft * 1e-3) / 1e9 if ms_draft else None,
           "verify_GBps": b_verify / (ms_verify * 1e-3) / 1e9 if ms_verify else None,
           "draft_step_bytes": b_draft, "verify_bytes": b_verify, "bytes_note": "weights of the layers a pass runs + its LM head + cached keys/values at mid-generation context",
           "mean_K": mean_k, "tokens_per_round": mean_commit, "v_d": v_d, "r_d": r_d,
           "hm": 200.0 * v_d * r_d / (v_d + r_d) if v_d + r_d else 0.0,
           "ts_alpha": st.alpha, "ts_beta": st.beta}
    # context only: the speed model of the paper's Appendix D, speedup = v_d / ((alpha - v_d) r_d + v_d) with
    # alpha = T_draft / T_target, at the acceptance the paper reports for its TRAINED early-exit layers
    # (Gsm8k, Beta-TS) and at this run's measured pass times (T_target taken as one verify pass)
    if ms_draft and ms_verify:
        alpha = ms_draft / ms_verify
        vd_p, rd_p = (0.52, 0.68) if shape["d_model"] >= 8192 else (0.50, 0.67)
        out["alpha_Td_over_Tt"] = alpha
        out["speed_model_at_paper_acceptance"] = {"v_d": vd_p, "r_d": rd_p, "speedup_vs_autoregressive": vd_p / ((alpha - vd_p) * rd_p + vd_p)}
    return out, mean_k, mean_commit


def time_prefill(ctx, torch, prompt, shape, si, reps=3):
    """eesd_prefill alone (it is part of every timed step): milliseconds, and the rate of its products against the
    bf16 MFMA peak (2 flop per weight of the L layers and token; attention and the one-row LM head not counted)."""
    ctx.prefill(prompt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        ctx.prefill(prompt)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / reps * 1e3
    flops = 2.0 * len(prompt) * shape["n_layers"] * si.layer_param_count(shape)
    tf = flops / (ms * 1e-3) / 1e12
    return {"tokens": len(prompt), "ms": ms, "ms_per_layer": ms / shape["n_layers"], "TFLOPs": tf, "bound": "mfma", "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
            "frac": tf / MFMA_BF16_PEAK_TFLOPS}


def side_generation(pk, si, torch, w, shape, n_prompt, max_new, k_cap, temperature, tiled, steps, ar_tokens=0, warmup_s=0.0):
    """A short untimed-by-the-headline generation run on given weights: tokens/s and per-pass figures."""
    max_seq = (n_prompt + max_new + k_cap + 2 + 63) // 64 * 64
    ctx = pk.EESD(w, max_seq=max_seq, temperature=temperature, seed=0, k_cap=k_cap, kv_page=64,
                  weight_layout=pk.WEIGHTS_TILED if tiled else pk.WEIGHTS_ROW_MAJOR)
    prompts = [si.make_prompt(n_prompt, shape["vocab"], 100 + i) for i in range(steps)]
    # untimed warm-up: one generation, or as many as fill warmup_s seconds (for the seconds after a large free, see the caller)
    t_warm = time.perf_counter()
    ctx.generate(prompts[-1], max_new)
    while time.perf_counter() - t_warm < warmup_s:
        ctx.generate(prompts[-1], max_new)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stats = [ctx.generate(prompts[i], max_new)[1] for i in range(steps)]
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    passes, _, _ = summarise(stats, shape, n_prompt, max_new, shape["dtype"] == "bf16", si)
    passes["tokens_per_s"] = steps * max_new / dt
    passes["steps"] = steps
    passes["temperature"] = temperature
    if shape["dtype"] == "bf16":
        passes["prefill"] = time_prefill(ctx, torch, prompts[0], shape, si)
    if ar_tokens:
        passes["autoregressive"] = autoregressive(ctx, torch, prompts[0], ar_tokens, passes["tokens_per_s"])
    ctx.close()
    return passes


def autoregressive(ctx, torch, prompt, n_tokens, eesd_tokens_per_s):
    """Plain auto-regressive decoding with the target model on the same context (the baseline of the paper's speed-up
    figures, Section 4.1): every token is one single-row target pass and one draw from its distribution - a round with
    no draft, driven call by call (verify, accept, rollback).  The ratio to the speculative rate is this run's speed-up,
    at the acceptance the synthetic draft happens to have (random weights: 15-22 %), not the paper's."""
    ctx.prefill(prompt)
    for _ in range(4):
        ctx.verify(); a, _ = ctx.accept(); ctx.rollback(a)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_tokens):
        ctx.verify()
        a, _ = ctx.accept()
        ctx.rollback(a)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    rate = n_tokens / dt
    return {"tokens_per_s": rate, "ms_per_token": dt / n_tokens * 1e3, "tokens": n_tokens, "prefill": "not in the rate",
            "eesd_over_autoregressive": eesd_tokens_per_s / rate,
            "note": "EESD rate: whole generations incl. prefill, acceptance of the synthetic draft"}


def progress(msg):
    """One line on stderr when a phase or a step has finished: the run prints its JSON line only at the end, and a
    harness that watches the output would take minutes of silence for a hang."""
    print(f"bench.py: {msg}", file=sys.stderr, flush=True)


def stored_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed hardware-counter summary
    (profiles/hbm_traffic.json, written from two rocprofv3 --pmc runs), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f).get(workload, {}).get("bytes_per_launch")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="70b", choices=sorted(WORKLOADS))
    ap.add_argument("--temperature", type=float, default=1.0)
    ap.add_argument("--tree-width", type=int, default=0,
                    help="2..4: candidate-tree verification (greedy decoding; temperature is set to 0 and K is capped so that 1 + K * width <= 16)")
    ap.add_argument("--row-major-weights", action="store_true",
                    help="keep the bf16 matrices row-major instead of the tile-major layout of eesd_pack_weight")
    ap.add_argument("--verify-reuse", action="store_true",
                    help="verify takes the drafted rows' layer-N hidden states from the draft steps instead of recomputing them")
    ap.add_argument("--controller", default="beta", choices=["beta", "cali"],
                    help="beta: Beta-posterior Thompson sampling (Algorithm 2); cali: the calibrated controller "
                         "(Algorithm 3) with a random predictor - measures its cost, not the paper's gain")
    ap.add_argument("--draft-correlation", type=float, default=None,
                    help="gamma of synth_inputs.make_weights(correlated_draft=gamma): a synthetic draft model that agrees with the "
                         "target often (independent random weights almost never do under greedy decoding)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip what the default run reports beside the timed steps: the greedy run, latency versus verify rows, the 13B-shape passes")
    ap.add_argument("--latency-sweep", action="store_true",
                    help="(non-default workloads) also report draft-step and verify-pass latency versus K over a pre-filled cache")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run the library's 1 GiB copy kernel a few times (reference for hardware-counter runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (batch-1 decoding does not shard across GPUs here); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth_inputs as si
    import paper_2406_03853_amd as pk

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    pk.lib()  # fails loudly if libeesd.so is not built
    shape_key, wseed, n_prompt, max_new, k_cap = WORKLOADS[args.workload]
    shape = getattr(si, shape_key)
    if args.tree_width >= 2:
        args.temperature = 0.0
        k_cap = min(k_cap, 15 // args.tree_width)
    extras = args.workload == "70b" and not args.headline_only and args.tree_width < 2 and args.controller == "beta" \
        and args.draft_correlation is None and not args.row_major_weights
    t0 = time.perf_counter()
    w = si.make_weights(shape, seed=wseed, device="cuda", correlated_draft=args.draft_correlation)
    torch.cuda.synchronize()
    t_weights = time.perf_counter() - t0
    progress(f"weights of the {shape['name']} drawn in {t_weights:.1f} s")
    cpu_w = None if args.no_cpu_baseline else oracle_sample_weights(w, shape, si)
    bf16 = shape["dtype"] == "bf16"
    tiled = bf16 and not args.row_major_weights
    if tiled:      # one-off rearrangement by the library's own kernel, matrix by matrix
        w = pk.pack_weights(w)
        torch.cuda.synchronize()
    layout = pk.WEIGHTS_TILED if tiled else pk.WEIGHTS_ROW_MAJOR
    max_seq = n_prompt + max_new + k_cap * max(1, args.tree_width) + 2
    sweep_tokens = 2048 if args.workload == "70b" else n_prompt       # cache length of the latency sweep
    if args.latency_sweep:
        max_seq = max(max_seq, sweep_tokens + k_cap + 2)
    max_seq = (max_seq + 63) // 64 * 64
    ctx = pk.EESD(w, max_seq=max_seq, temperature=args.temperature, seed=0, k_cap=k_cap, kv_page=64, tree_width=args.tree_width, verify_reuse=int(args.verify_reuse),
                  weight_layout=layout, ts_mode=pk.TS_CALI if args.controller == "cali" else pk.TS_BETA)
    if args.controller == "cali":
        cw = si.make_cali_weights(shape, wseed, device="cuda")
        ctx.set_calibration(pk.pack_calibration(cw) if tiled else cw, 0.2, 0.5, 0.5)
    # one prompt per step: with random weights the acceptance of a single stream is a matter of luck
    # (14-21 % here), so the steps run different streams and the rate is their mean
    prompts = [si.make_prompt(n_prompt, shape["vocab"], i) for i in range(max(1, args.steps))]

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(7)
        dst = torch.empty_like(src)
        for _ in range(3):
            pk.calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        ctx.generate(prompts[-1], max_new)
        progress(f"warm-up step {i + 1} of {args.warmup} done")
    torch.cuda.synchronize()
    # ---- the timed region: exactly `steps` whole generations, nothing else on the stream ----
    t0 = time.perf_counter()
    stats = []
    for i in range(args.steps):
        _, st = ctx.generate(prompts[i], max_new)     # returns after the generation's last synchronisation
        stats.append(st)
        progress(f"step {i + 1} of {args.steps} done")
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # ---- after it: one more generation with a HIP event pair around every launch of the dominant kernel
    # (the gate/up product of the draft and verify passes: MFMA family on bf16, VALU on fp32) ----
    ctx.profile_begin(1 if bf16 else 0, 2, shape["d_model"])
    ctx.generate(prompts[0], max_new)
    n_launch, ms_kernel = ctx.profile_end()
    progress("dominant kernel timed")

    passes, mean_k, mean_commit = summarise(stats, shape, n_prompt, max_new, bf16, si)
    passes["weight_init_s"] = t_weights
    if bf16:
        passes["prefill"] = time_prefill(ctx, torch, prompts[0], shape, si)
    if not args.headline_only and args.tree_width < 2 and args.controller == "beta":
        passes["autoregressive"] = autoregressive(ctx, torch, prompts[0], 64, args.steps * max_new / dt)
        progress("auto-regressive baseline timed")
    N, L = shape["n_draft_layers"], shape["n_layers"]
    esz = 2 if bf16 else 4
    kernel_bytes = 2 * shape["d_ff"] * shape["d_model"] * esz          # weights of one gate/up product
    avg_kernel_s = (ms_kernel / max(1, n_launch)) * 1e-3
    achieved = kernel_bytes / avg_kernel_s / 1e9 if n_launch else 0.0

    out = {
        "metric": "decoded tokens/s bs=1 (70B-shape bf16); HBM GB/s of draft+verify passes",
        "value": args.steps * max_new / dt,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"full EESD generation, {shape['name']} (L={L}, N={N}), random weights seed {wseed}, "
                               f"prompt {n_prompt} uniform ids (a different one per step), {max_new} new tokens, Beta-TS K cap {k_cap}, "
                               f"temperature {args.temperature:g}, batch 1"
                               + (f", candidate tree of width {args.tree_width}" if args.tree_width >= 2 else "")
                               + (", tile-major weight layout" if tiled else ", row-major weights")
                               + (", verify reuses the draft steps' layer-N hidden states" if args.verify_reuse else "")
                               + (", calibrated controller with a random predictor" if args.controller == "cali" else "")
                               + (f", draft correlated with the target (gamma {args.draft_correlation:g})" if args.draft_correlation is not None else ""),
                   "prefill": "included in every step (blocks of up to 512 rows, MFMA GEMM on tile-major weights)" if bf16 else "included in every step (16-row blocks)"},
        "roofline": {"bound": "hbm", "kernel": "gemm_mfma_kernel<SWIGLU> (gate/up product of the draft and verify passes)" if bf16
                     else "gemm_valu_kernel<SWIGLU>",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": stored_traffic(args.workload), "launches_timed": n_launch, "avg_kernel_us": avg_kernel_s * 1e6,
                     "bytes_per_launch": kernel_bytes,
                     "timed_in": "one extra generation after the timed steps (an event pair around every launch)",
                     "pass_frac": {"draft": (passes["draft_step_GBps"] or 0.0) / HBM_PEAK_GBS, "verify": (passes["verify_GBps"] or 0.0) / HBM_PEAK_GBS}},
        "passes": passes,
    }
    if bf16:
        out["roofline"]["prefill_frac_of_mfma_peak"] = passes["prefill"]["frac"]    # the one MFMA-bound part, against 2.5 PFLOP/s
    if args.latency_sweep and not extras:
        ks = [k for k in (0, 1, 2, 3, 5, 7, 10, 15) if k <= k_cap]
        out["latency_vs_K"] = latency_sweep(ctx, torch, sweep_tokens, ks, shape, si)
    ctx.close()
    del ctx
    if extras:
        # greedy decoding on the same weights (random weights: a greedy draft almost never matches, K collapses to 1)
        out["passes_T0"] = side_generation(pk, si, torch, w, shape, n_prompt, max_new, k_cap, 0.0, tiled, 2)
        progress("greedy generations done")
        # the verify micro-benchmark of the 70B shape: one block of 1, 2, 4, 8, 16 rows over a 2048-token cache, then the
        # accept / resample kernel on 32000-way bf16 logits with the context's seeded uniforms
        c4 = pk.EESD(w, max_seq=2048 + 64, temperature=1.0, seed=0, k_cap=15, kv_page=64, weight_layout=layout, logits_bf16=1)
        out["latency_vs_K"] = {"cache_tokens": 2048, "logits": "bf16", "by_verify_rows": latency_sweep(c4, torch, 2048, (0, 1, 3, 7, 15), shape, si, pk)}
        c4.close()
        del c4
        progress("latency sweep done")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cpu_w, shape, args.temperature, mean_k, mean_commit, si)
        progress("oracle timed on the host")
    if extras:
        # the regime the method is made for - a draft that often agrees with the target: the same shape with a synthetic
        # early-exit layer and head correlated with the target's (gamma 0.1), greedy decoding, and plain auto-regressive
        # decoding on the same weights; the acceptance is a property of that synthetic pair, not of a trained model
        del w
        torch.cuda.empty_cache()
        w = si.make_weights(shape, seed=wseed, device="cuda", correlated_draft=0.1)
        if tiled:
            w = pk.pack_weights(w)
        torch.cuda.synchronize()
        pc = side_generation(pk, si, torch, w, shape, n_prompt, max_new, k_cap, 0.0, tiled, 2, ar_tokens=64)
        pc["workload"] = f"full EESD generation, {shape['name']}, early-exit layer and head correlated with the target (gamma 0.1), greedy, prompt {n_prompt}, {max_new} new tokens, K cap {k_cap}"
        out["passes_correlated_draft_T0"] = pc
        progress("correlated-draft generations done")
        # the 13B shape: the 70B weights go first
        del w
        torch.cuda.empty_cache()
        key13, seed13, np13, new13, cap13 = WORKLOADS["13b"]
        shape13 = getattr(si, key13)
        w13 = pk.pack_weights(si.make_weights(shape13, seed=seed13, device="cuda"))
        torch.cuda.synchronize()
        # (For about 5 s after the 137 GB of 70B-shape weights have been given back, every pass on the device runs 2 % slower
        # - 13B-shape draft step 0.766 against 0.750 ms - whatever memory it uses, and then returns to its rate while
        # the work goes on; the warm-up generations cover that time.)
        p13 = side_generation(pk, si, torch, w13, shape13, np13, new13, cap13, 1.0, True, 4, ar_tokens=128, warmup_s=8.0)
        p13["workload"] = f"full EESD generation, {shape13['name']} (L={shape13['n_layers']}, N={shape13['n_draft_layers']}), prompt {np13}, {new13} new tokens, K cap {cap13}, temperature 1"
        p13["pass_frac"] = {"draft": p13["draft_step_GBps"] / HBM_PEAK_GBS, "verify": p13["verify_GBps"] / HBM_PEAK_GBS}
        out["passes_13b"] = p13
        out["roofline"]["pass_frac_13b"] = p13["pass_frac"]          # the second shape the 70 % target names
        progress("13B-shape generations done")
        out["passes_13b_T0"] = side_generation(pk, si, torch, w13, shape13, np13, new13, cap13, 0.0, True, 2)
        progress("13B-shape greedy generations done")
        # the long-context configuration of the same shape: a 3840-token prompt, the cache grows to 4096
        _, _, npl, newl, capl = WORKLOADS["13b-long"]
        pl = side_generation(pk, si, torch, w13, shape13, npl, newl, capl, 1.0, True, 2)
        pl["workload"] = f"full EESD generation, {shape13['name']}, prompt {npl}, {newl} new tokens, K cap {capl}, temperature 1"
        pl["pass_frac"] = {"draft": pl["draft_step_GBps"] / HBM_PEAK_GBS, "verify": pl["verify_GBps"] / HBM_PEAK_GBS}
        out["passes_13b_long"] = pl
        out["roofline"]["pass_frac_13b_long_context"] = pl["pass_frac"]
        progress("13B-shape long-context generations done")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
