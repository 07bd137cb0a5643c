#!/usr/bin/env python3
"""Benchmark of the PEARL hot path on one MI355X.

One step = one pass of the whole path: gamma draft forwards on the draft stream alongside one
target forward on the target stream, then the fused accept / reject and the KV rollback.
Workload (default): the 70B/7B-shape pair, bf16 random-init, 4096-token uniform prompt, temperature 1,
window size gamma = round(T_target / T_draft) measured on the box (capped at 16).

Prints ONE JSON line: decode tokens/s of PEARL over K timed steps (after W warm-up steps), the
roofline of the dominant kernel (the target's projection kernel, HIP events around every launch of
it in the timed region), the CPU oracle timed on a bounded sample, and side results (AR and fixed-gamma
SD on the same kernels, forced-acceptance runs, pass-alone bandwidths).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0      # dense bf16 matrix-core peak of the MI355X


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=96)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", default="70b_7b", help="tiny | small | 7b_1b | 33b_1b | 70b_7b")
    ap.add_argument("--gamma", type=int, default=0, help="0 = calibrate gamma = round(c) on the box")
    ap.add_argument("--depth", type=int, default=0, help="truncate the target to this many layers (experiments)")
    ap.add_argument("--draft-depth", type=int, default=0)
    ap.add_argument("--wgs", type=int, default=-1, help="projection workgroups per CU: -1 auto, 1, 2")
    ap.add_argument("--tail", type=int, default=-1,
                    help="SPEC_OPT_TARGET_TAIL_LAYERS: -1 = balanced by the library at run time, n = fixed (experiments)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: tokens/s of PEARL and SD over window sizes and acceptance rates")
    ap.add_argument("--sweep-part", default="all", help="with --sweep: all | gamma | cu (which part of the study to run)")
    ap.add_argument("--phase", default="", choices=["", "verify", "verify-graph", "draft", "step-chains"],
                    help="run only that pass alone (N = --steps forwards at the prompt's context length) and print its "
                         "figures: verify = kernel by kernel with an event pair per projection launch, verify-graph / draft = "
                         "captured graphs replayed; the commands the rocprofv3 summaries under profiles/ are made with")
    ap.add_argument("--library-generator", action="store_true",
                    help="weights of the same shapes and distributions from PyTorch's generator instead of the counter-based "
                         "one: for runs under rocprofv3 --pmc, whose counter collection crashes on PyTorch's run-time-compiled "
                         "inverse-normal kernel (kernel counters do not depend on the values)")
    ap.add_argument("--rows", type=int, default=0, help="with --phase verify / verify-graph: tokens per forward (default gamma)")
    ap.add_argument("--fuse", type=int, default=-1, help="SPEC_OPT_FUSE_SINGLE value (experiments)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-side", action="store_true", help="skip AR / SD / forced-acceptance side runs")
    return ap.parse_args()


def forward_bytes(shape, n_ctx, m):
    """Algorithmic HBM bytes of one forward over m tokens at context n_ctx: every projection weight once,
    the KV cache read once, m new KV rows written, fp32 logits written."""
    return 2 * shape.streamed_params() + n_ctx * shape.kv_bytes_per_token() + m * shape.kv_bytes_per_token() \
        + m * shape.vocab * 4


def timed(fn, sync):
    sync()
    t0 = time.perf_counter()
    out = fn()
    sync()
    return out, time.perf_counter() - t0


def cpu_baseline(cfg, gamma, device):
    """The oracle as it stands, on the host cores, on a bounded sample: a depth-truncated pair of the
    same widths (weights from the same generator), a short prompt, a few PEARL steps.  Per-layer times
    are scaled to the full depths; the result is a reported baseline, not a target."""
    import torch
    import synth
    from oracle import loops, transformer
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    lt, ld = (2, 1) if cfg.target.d_model >= 4096 else (min(4, cfg.target.n_layers), min(2, cfg.draft.n_layers))
    lt, ld = min(lt, cfg.target.n_layers), min(ld, cfg.draft.n_layers)
    small = synth.config(cfg.name, depth=lt, draft_depth=ld)
    tw, dw = synth.make_pair(small, device=device)

    def to_np(w, memo={}):
        cv = lambda t: memo.setdefault(t.data_ptr(), t.float().cpu().numpy())
        return {"tok_embed": cv(w["tok_embed"]), "lm_head": cv(w["lm_head"]), "final_norm": cv(w["final_norm"]),
                "layers": [{k: cv(v) for k, v in lay.items()} for lay in w["layers"]]}

    mk = lambda w, s: transformer.Model(to_np(w), s.n_heads, s.n_kv_heads, s.head_dim, s.rope_theta, s.rms_eps)
    tm, dm = mk(tw, small.target), mk(dw, small.draft)
    del tw, dw
    n_prompt, budget_s = 64, 5.0
    prompt = synth.prompt_tokens(n_prompt, cfg.target.vocab, cfg.seed_prompt).tolist()
    n_cache = 2048

    def forwards_for(model, seconds):
        """Single-token forwards behind the prompt for about `seconds` (at least 5, after 2 untimed ones)."""
        cm = transformer.CachedModel(model, n_cache)
        cm.feed(prompt[:-1])
        for i in range(2):
            cm.feed([prompt[i]])
        n, t0 = 0, time.perf_counter()
        while (n < 5 or time.perf_counter() - t0 < seconds) and cm.len < n_cache - 1:
            cm.feed([prompt[n % n_prompt]])
            n += 1
        return (time.perf_counter() - t0) / n, n

    def head_time(model, d_model):
        x = np.ones((1, d_model), dtype=np.float32)
        for _ in range(2):
            _ = x @ model.lm_head.T
        t0 = time.perf_counter()
        for _ in range(10):
            _ = x @ model.lm_head.T
        return (time.perf_counter() - t0) / 10

    # time the two passes of a step separately so that they can be scaled to the full depths, and split each
    # into per-layer and head parts with a second measurement on the LM head alone
    t_target, n_t = forwards_for(tm, budget_s)
    t_draft, n_d = forwards_for(dm, budget_s)
    t_head_t = head_time(tm, cfg.target.d_model)
    t_head_d = head_time(dm, cfg.draft.d_model)
    per_layer_t = max(t_target - t_head_t, 0.0) / lt
    per_layer_d = max(t_draft - t_head_d, 0.0) / ld
    full_t = per_layer_t * cfg.target.n_layers + t_head_t
    full_d = per_layer_d * cfg.draft.n_layers + t_head_d
    # a PEARL step on the CPU runs its gamma draft forwards and its target forward one after the other;
    # it commits at least one token, so 1 token/step is the floor used here (the GPU line reports its own rate)
    step = full_t + gamma * full_d
    return {"value": 1.0 / step, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": (f"oracle forward timed on a depth-truncated {cfg.name} pair ({lt} target + {ld} draft layers, "
                       f"same widths, {n_prompt}-token prompt, {n_t} target and {n_d} draft single-token forwards, "
                       f"about {budget_s:.0f} s of CPU work each after 2 untimed ones); per-layer time x full depth + LM "
                       f"head; one PEARL step = 1 target + {gamma} draft "
                       f"forwards in series, counted at its floor of 1 committed token per step"),
            "target_forward_s": full_t, "draft_forward_s": full_d}


def sweep(args, cfg, ctx, amd, synth, sync, n0, tp, tq, log):
    """Window-size and co-location study (the analogue of the paper's gamma tables on one GPU): tokens/s of
    PEARL with one or two projection workgroups per CU and of vanilla SD, for gamma in a range, with the
    pair's own acceptance decisions and with forced Bernoulli(alpha) decisions."""
    steps = max(8, args.steps // 4)
    rows = []

    def run(algo, g, wgs, alpha):
        ctx.rewind(n0)
        ctx.set_option(amd.SPEC_OPT_GEMM_WGS_PER_CU, wgs)
        u = synth.make_uniforms(steps + 3, g, cfg.seed_uniform)
        fb = None
        if alpha is not None:
            fb = (synth.uniform_array((steps + 3) * (g + 1), 5, 7).view(steps + 3, g + 1).numpy() < alpha)
        ctx.generate(algo, g, 1 << 20, u, force_bits=fb, max_steps=2)
        sync(); t0 = time.perf_counter()
        _, s = ctx.generate(algo, g, 1 << 20, u, force_bits=fb, max_steps=steps)
        sync(); dt = time.perf_counter() - t0
        return s["committed"] / dt, s["committed"] / s["steps"], dt / s["steps"] * 1e3

    ar = run(amd.ALGO_AR, 1, 2, None)
    log(f"[sweep] AR: {ar[0]:.2f} tok/s, {ar[2]:.2f} ms/step; c = {tp / tq:.2f}")
    for alpha in (None, 0.7, 0.9) if args.sweep_part in ("all", "gamma") else ():
        for g in (2, 3, 4, 6, 8, 10, 12):
            r = {"alpha": "pair" if alpha is None else alpha, "gamma": g}
            for name, algo, wgs in (("pearl_1wg", amd.ALGO_PEARL, 1), ("pearl_2wg", amd.ALGO_PEARL, 2),
                                    ("sd", amd.ALGO_SD, 2)):
                tps, tpstep, ms = run(algo, g, wgs, alpha)
                r[name] = {"tokens_per_s": round(tps, 2), "tokens_per_step": round(tpstep, 3), "step_ms": round(ms, 2)}
            rows.append(r)
            log(f"[sweep] {json.dumps(r)}")
    # CU partition between the two streams (the paper's resource-competition setting, Appendix on RC): the target
    # stream gets the first T compute units, the draft stream the rest; decisions forced to Bernoulli(0.9) so that
    # every point sees the same mix of pre- and post-verify steps
    from paper_2408_11850_amd import harness
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, cfg.seed_prompt).tolist()
    g = args.gamma or 7
    split_rows = []
    for t_cus in (None, 256, 224, 192, 160, 128, 96, None) if args.sweep_part in ("all", "cu") else ():
        c2 = harness.make_context(cfg, ctx.target, ctx.draft, 16, extra_seq=64, target_cus=t_cus)
        c2.prefill(prompt)
        r = {"target_cus": t_cus or "all (plain streams)", "draft_cus": "all" if not t_cus or t_cus >= 256 else 256 - t_cus}
        for wgs in (1, 2):
            c2.set_option(amd.SPEC_OPT_GEMM_WGS_PER_CU, wgs)
            c2.rewind(n0)
            u = synth.make_uniforms(steps + 8, g, cfg.seed_uniform)
            fb = (synth.uniform_array((steps + 8) * (g + 1), 5, 7).view(steps + 8, g + 1).numpy() < 0.9)
            c2.generate(amd.ALGO_PEARL, g, 1 << 20, u, force_bits=fb, max_steps=6)   # captures every graph variant
            sync(); t0 = time.perf_counter()
            _, s2 = c2.generate(amd.ALGO_PEARL, g, 1 << 20, u, force_bits=fb, max_steps=steps)
            sync(); dt = time.perf_counter() - t0
            r[f"pearl_{wgs}wg"] = {"tokens_per_s": round(s2["committed"] / dt, 2), "step_ms": round(dt / s2["steps"] * 1e3, 2)}
        c2.close()
        split_rows.append(r)
        log(f"[sweep] cu split {json.dumps(r)}")
    print(json.dumps({"workload": cfg.name, "n_prompt": n0, "steps_per_point": steps, "c": tp / tq,
                      "ar_tokens_per_s": ar[0], "rows": rows, "cu_split_gamma": g, "cu_split": split_rows}))


def step_chains(args, cfg, ctx, amd, sync, n0, gamma, log):
    import torch
    import synth
    N = max(4, args.steps)
    post = args.rows != 1
    ctx.set_option(amd.SPEC_OPT_GEMM_WGS_PER_CU, 1 if args.wgs < 0 else args.wgs)
    ctx.set_option(amd.SPEC_OPT_TARGET_TAIL_LAYERS, max(args.tail, 0))
    uni = synth.make_uniforms(N + 1, gamma, cfg.seed_uniform)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    mode, rows = amd.SPEC_MODE_PRE, []
    ctx.rewind(n0)
    for t in range(N):
        e0t, e0d, et, ed = ev(), ev(), ev(), [ev() for _ in range(gamma)]
        sync()
        e0t.record(ctx.stream_target); e0d.record(ctx.stream_draft)
        pre = mode == amd.SPEC_MODE_PRE
        ctx.verify(n_tokens=1 if pre else gamma)
        et.record(ctx.stream_target)
        for i in range(gamma):
            ctx.draft_step(float(uni.draft[t, i])); ed[i].record(ctx.stream_draft)
        res = ctx.accept(amd.SPEC_ACCEPT_PRE if pre else amd.SPEC_ACCEPT_POST, uni.accept[t, :gamma + 1].numpy(),
                         float(uni.resample[t]), (1 << (gamma + 1)) - 1 if post else 0)
        if res["keep_len"] >= 0:
            for w in (amd.SPEC_TARGET, amd.SPEC_DRAFT):
                if ctx.kv_len(w) > res["keep_len"]:
                    ctx.rollback_kv(w, res["keep_len"])
        sync()
        rows.append({"mode": "pre" if pre else "post", "target_chain_ms": round(e0t.elapsed_time(et), 2),
                     "draft_forwards_end_ms": [round(e0d.elapsed_time(e), 2) for e in ed]})
        mode = res["next_mode"]
    keep = rows[len(rows) // 2:]                       # the first steps capture graphs
    avg = lambda xs: round(sum(xs) / len(xs), 2)
    out = {"phase": "step-chains", "workload": cfg.name, "gamma": gamma, "n_ctx": n0 - 1,
           "projection_workgroups_per_cu": ctx.get_option(amd.SPEC_OPT_GEMM_WGS_PER_CU),
           "target_tail_layers": ctx.get_option(amd.SPEC_OPT_TARGET_TAIL_LAYERS), "steps_kept": len(keep),
           "mode": keep[-1]["mode"], "target_chain_ms": avg([r["target_chain_ms"] for r in keep]),
           "draft_chain_ms": avg([r["draft_forwards_end_ms"][-1] for r in keep]),
           "first_draft_forward_ms": avg([r["draft_forwards_end_ms"][0] for r in keep]),
           "last_step": keep[-1]}
    log(f"[bench] step-chains: {json.dumps(out)}")
    print(json.dumps(out))


def phase(args, cfg, ctx, amd, sync, n0, gamma, log):
    """One pass alone, N = --steps forwards at the prompt's context length; the commands behind the per-kernel tables
    in profiles/ (run under `rocprofv3 --kernel-trace --stats` or `--pmc ...`, with --gamma given so that no
    calibration forwards mix in).
      verify        kernel by kernel, every projection launch stamping a HIP event pair with its own start / end:
                    the dominant kernel's average launch duration as bench.py's roofline object measures it
      verify-graph  the same forwards as the library runs them (captured graphs replayed): the pass's wall time
      draft         draft forwards (with their draws), graphs replayed
      step-chains   PEARL steps driven call by call with events on both streams: when the target chain and every
                    draft forward of a step end (the tracer runs the two streams one after the other, so this is
                    the untraced view of the overlap); --tail fixes the trailing target layers that launch with
                    two workgroups per CU, decisions forced to accept (post-verify steps) unless --rows 1
                    (rejections: pre-verify steps)"""
    N = max(1, args.steps)
    if args.phase == "step-chains":
        return step_chains(args, cfg, ctx, amd, sync, n0, gamma, log)
    verify = args.phase.startswith("verify")
    shape = cfg.target if verify else cfg.draft
    out = {"phase": args.phase, "workload": cfg.name, "n_ctx": n0 - 1, "forwards": N, "gamma": gamma}

    def run_verify(m):
        toks = list(range(1, m + 1))
        for _ in range(N):
            ctx.verify(toks)
            ctx.rollback_kv(amd.SPEC_TARGET, n0 - 1)

    def run_draft(_m):
        done = 0
        while done < N:                       # at most 2 * gamma_max drafts may be pending
            k = min(N - done, 2 * ctx.gamma_max)
            for _ in range(k):
                ctx.draft_step(0.5)
            ctx.rewind(n0)
            done += k

    for m in ((args.rows or gamma,) if verify else (1,)):
        b = forward_bytes(shape, n0 - 1, m)
        if args.phase == "verify":
            ctx.set_profile(1); ctx.profile_read()
            _, t = timed(lambda: run_verify(m), sync)
            ms, n, by = ctx.profile_read()
            ctx.set_profile(0)
            out[f"m{m}"] = {"projection_kernel": {
                "launches": int(n), "avg_launch_us": ms / max(n, 1) * 1e3, "avg_bytes_per_launch": by / max(n, 1),
                "GBps": by / max(ms, 1e-9) / 1e6, "frac_of_peak": by / max(ms, 1e-9) / 1e6 / HBM_PEAK_GBS},
                "forward_ms_kernel_by_kernel": t / N * 1e3}
        else:
            run = run_verify if verify else run_draft
            run(m); sync()                        # captures the graphs of this shape
            _, t = timed(lambda: run(m), sync)
            out[f"m{m}"] = {"forward_ms": t / N * 1e3, "GBps": b / (t / N) / 1e9,
                            "frac_of_peak": b / (t / N) / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes": b}
        log(f"[bench] phase {args.phase} M={m}: {json.dumps(out[f'm{m}'])}")
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (both models and both streams share one MI355X); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    import synth
    import paper_2408_11850_amd as amd
    from paper_2408_11850_amd import harness
    amd.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda"
    sync = torch.cuda.synchronize
    cfg = synth.config(args.config, depth=args.depth or None, draft_depth=args.draft_depth or None)
    gamma_max = 16
    log = lambda *a: print(*a, file=sys.stderr, flush=True)

    (pair, t_build) = timed(lambda: harness.build_pair(cfg, dev, library_generator=args.library_generator), sync)
    target, draft = pair
    log(f"[bench] built {cfg.name}: target {target.nbytes() / 1e9:.2f} GB, draft {draft.nbytes() / 1e9:.2f} GB in {t_build:.1f}s")
    ctx = harness.make_context(cfg, target, draft, gamma_max, extra_seq=64)
    ctx.set_option(amd.SPEC_OPT_GEMM_WGS_PER_CU, args.wgs)
    ctx.set_option(amd.SPEC_OPT_TARGET_TAIL_LAYERS, args.tail)
    if args.fuse >= 0:
        ctx.set_option(amd.SPEC_OPT_FUSE_SINGLE, args.fuse)
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, cfg.seed_prompt).tolist()
    # prompt pass of each model alone (dense matrix-core path when the shapes allow it), then both for the run
    def prefill_flops(sh, c):
        per_layer = sh.d_model * (sh.n_heads + 2 * sh.n_kv_heads) * sh.head_dim + sh.n_heads * sh.head_dim * sh.d_model \
            + 3 * sh.d_model * sh.d_ffn
        return 2.0 * c * per_layer * sh.n_layers + 2.0 * sh.head_dim * sh.n_heads * c * c * sh.n_layers
    ctx.prefill(prompt[:130], which_mask=3)            # first use allocates the prompt-path buffers
    _, t_pf_t = timed(lambda: ctx.prefill(prompt, which_mask=1), sync)
    _, t_pf_d = timed(lambda: ctx.prefill(prompt, which_mask=2), sync)
    _, t_prefill = timed(lambda: ctx.prefill(prompt), sync)
    c_pf = cfg.n_prompt - 1
    prefill_stats = {"tokens": c_pf, "target_s": t_pf_t, "draft_s": t_pf_d, "both_s": t_prefill,
                     "target_TFLOPs": prefill_flops(cfg.target, c_pf) / t_pf_t / 1e12,
                     "draft_TFLOPs": prefill_flops(cfg.draft, c_pf) / t_pf_d / 1e12, "bound": "mfma",
                     "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS}
    prefill_stats["target_frac_of_peak"] = prefill_stats["target_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
    log(f"[bench] prefill of {cfg.n_prompt} tokens: {json.dumps({k: (round(v, 4) if isinstance(v, float) else v) for k, v in prefill_stats.items()})}")
    n0 = cfg.n_prompt

    # ---- window size: gamma = round(c), c = T(target forward) / T(draft forward) ---------------
    # (Section 4.4.1; the library measures it: each model with the GPU to itself, as on the paper's separate devices,
    # and with both streams busy at once, as inside a PEARL step on one GPU)
    if args.phase and args.gamma:
        phase(args, cfg, ctx, amd, sync, n0, args.gamma, log)
        ctx.close()
        return
    g_cal, tp, tq = ctx.calibrate_gamma(8, gamma_max, concurrent=False)
    g_con, tp_c, tq_c = ctx.calibrate_gamma(8, gamma_max, concurrent=True)
    gamma = args.gamma or g_cal
    log(f"[bench] alone: target fwd {tp * 1e3:.2f} ms, draft fwd {tq * 1e3:.2f} ms, c = {tp / tq:.2f} -> gamma {g_cal}; "
        f"both streams busy: {tp_c * 1e3:.2f} / {tq_c * 1e3:.2f} ms, c = {tp_c / tq_c:.2f} -> gamma {g_con}; using {gamma}")
    ctx.rewind(n0)

    if args.phase:
        phase(args, cfg, ctx, amd, sync, n0, gamma, log)
        ctx.close()
        return

    if args.sweep:
        sweep(args, cfg, ctx, amd, synth, sync, n0, tp, tq, log)
        ctx.close()
        return

    # ---- each pass alone: bytes / time ---------------------------------------------------------
    def alone(fn, n):
        fn(); sync()
        _, t = timed(lambda: [fn() for _ in range(n)], sync)
        return t / n

    t_v1 = alone(lambda: ctx.verify([1]), 6); ctx.rewind(n0)
    t_vg = alone(lambda: ctx.verify(list(range(1, gamma + 1))), 6); ctx.rewind(n0)
    # the dominant kernel with the stream to itself: HIP events around every target projection of 3 forwards
    ctx.set_profile(1); ctx.profile_read()
    for _ in range(3):
        ctx.verify(list(range(1, gamma + 1)))
    ms_a, n_a, bytes_a = ctx.profile_read()
    ctx.set_profile(0); ctx.rewind(n0)
    gemm_alone = bytes_a / max(ms_a, 1e-9) / 1e6

    def draft_chain():
        ctx.draft_step(0.5)
    t_d = alone(draft_chain, min(10, 2 * gamma_max - 2)); ctx.rewind(n0)
    bw = lambda b, t: b / t / 1e9
    alone_stats = {
        "verify_m1_ms": t_v1 * 1e3, "verify_m1_GBps": bw(forward_bytes(cfg.target, n0, 1), t_v1),
        "verify_mgamma_ms": t_vg * 1e3, "verify_mgamma_GBps": bw(forward_bytes(cfg.target, n0, gamma), t_vg),
        "draft_ms": t_d * 1e3, "draft_GBps": bw(forward_bytes(cfg.draft, n0, 1), t_d),
    }
    for k in ("verify_m1", "verify_mgamma", "draft"):
        alone_stats[k + "_frac_of_peak"] = alone_stats[k + "_GBps"] / HBM_PEAK_GBS
    log(f"[bench] alone: {json.dumps({k: round(v, 3) for k, v in alone_stats.items()})}")

    # streaming-read ceiling of this machine: plain 16-byte loads over 2 GiB (10 launches back to back between two events,
    # best of 3): what a long stream reaches; a launch of the projection kernel streams 134 - 940 MB and pays its
    # ramp and tail on every one of them
    buf = torch.empty(1 << 30, dtype=torch.bfloat16, device=dev).fill_(1.0)
    amd.read_probe(buf); sync()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    read_ceiling = 0.0
    for _ in range(3):
        e0.record()
        for _ in range(10):
            amd.read_probe(buf)
        e1.record(); sync()
        read_ceiling = max(read_ceiling, buf.numel() * 2 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del buf

    # ---- the timed region: W warm-up + K timed PEARL steps -------------------------------------
    K, W = args.steps, args.warmup
    uni = synth.make_uniforms(max(K, W) + 1, gamma, cfg.seed_uniform)
    if W > 0:
        ctx.generate(amd.ALGO_PEARL, gamma, 1 << 20, uni, max_steps=W)
    # the timed region: K PEARL steps as the library runs them (captured forwards replayed)
    sync()
    t0 = time.perf_counter()
    toks, st = ctx.generate(amd.ALGO_PEARL, gamma, 1 << 20, uni, max_steps=K)
    sync()
    elapsed = time.perf_counter() - t0
    committed = int(st["committed"])
    # The same K steps once more (same start state, same uniforms, hence the same tokens) with a HIP event pair
    # around every target projection launch.  The events need kernel-by-kernel launches and put two barrier
    # packets around each of ~320 launches per forward, which lengthens a step by about 4 %; so this pass gives
    # the kernel's in-region launch durations, the clean pass above gives the throughput.
    ctx.rewind(n0)
    if W > 0:
        ctx.generate(amd.ALGO_PEARL, gamma, 1 << 20, uni, max_steps=W)
    ctx.set_profile(1)
    ctx.profile_read()
    sync()
    t0i = time.perf_counter()
    toks_i, st_i = ctx.generate(amd.ALGO_PEARL, gamma, 1 << 20, uni, max_steps=K)
    sync()
    elapsed_i = time.perf_counter() - t0i
    ms_gemm, n_gemm, bytes_gemm = ctx.profile_read()
    ctx.set_profile(0)
    same_tokens = toks_i == toks
    if not same_tokens:
        log("[bench] WARNING: the instrumented pass committed other tokens than the timed pass")
    value = committed / elapsed
    step_bytes = forward_bytes(cfg.target, n0, gamma) + gamma * forward_bytes(cfg.draft, n0, 1)
    pearl = {"tokens_per_step": committed / st["steps"], "alpha": st["accepted"] / max(st["tested"], 1),
             "post_fraction": st["post_steps"] / st["steps"], "step_ms": elapsed / st["steps"] * 1e3,
             "step_GBps": bw(step_bytes, elapsed / st["steps"]),
             "overlap_efficiency": (gamma * t_d + (t_vg if st["post_steps"] else t_v1)) / (elapsed / st["steps"])}
    pearl["target_tail_layers"] = ctx.get_option(amd.SPEC_OPT_TARGET_TAIL_LAYERS)
    log(f"[bench] PEARL: {value:.2f} tok/s, {json.dumps({k: round(v, 3) for k, v in pearl.items()})}")

    side = {}
    if not args.no_side:
        ks = max(8, K // 3)
        def run(algo, g, force_alpha=None, steps=ks, serial_ctx=None):
            c = serial_ctx or ctx
            c.rewind(n0)
            u = synth.make_uniforms(steps + 1, g, cfg.seed_uniform)
            fb = None
            if force_alpha is not None:
                fb = (synth.uniform_array((steps + 1) * (g + 1), 5, 7).view(steps + 1, g + 1).numpy() < force_alpha)
            c.generate(algo, g, 1 << 20, u, force_bits=fb, max_steps=2)
            sync(); t0 = time.perf_counter()
            _, s = c.generate(algo, g, 1 << 20, u, force_bits=fb, max_steps=steps)
            sync(); dt = time.perf_counter() - t0
            return {"tokens_per_s": s["committed"] / dt, "tokens_per_step": s["committed"] / s["steps"],
                    "step_ms": dt / s["steps"] * 1e3, "alpha": s["accepted"] / max(s["tested"], 1)}
        side["ar"] = run(amd.ALGO_AR, 1, steps=max(ks, 16))
        side["sd"] = run(amd.ALGO_SD, gamma)
        for a in (0.5, 0.7, 0.9):
            side[f"pearl_forced_alpha_{a}"] = run(amd.ALGO_PEARL, gamma, a)
            side[f"sd_forced_alpha_{a}"] = run(amd.ALGO_SD, gamma, a)
        # the two ablations of Section 4.3 on the same kernels (analogue of the paper's ablation table)
        for a in (None, 0.9):
            tag = "" if a is None else f"_forced_alpha_{a}"
            side["pearl_without_pre_verify" + tag] = run(amd.ALGO_PEARL_NO_PRE, gamma, a)
            side["pearl_without_post_verify" + tag] = run(amd.ALGO_PEARL_NO_POST, gamma, a)
        # pre-verify over guessed continuations (closing remark of Section 4.3): on random-init text the pool hardly
        # ever guesses right, so this shows what the extra rows of the pre-verify forward cost, not what they can gain
        for a in (None, 0.9):
            tag = "" if a is None else f"_forced_alpha_{a}"
            side["pearl_guessed_pre_verify" + tag] = run(amd.ALGO_PEARL_GUESS, gamma, a)
        log(f"[bench] side runs: {json.dumps(side, default=float)}")

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(cfg.name, {}).get("gemm_target_bytes_per_launch")
        except Exception:
            traffic = None
    in_step = bytes_gemm / max(ms_gemm, 1e-9) / 1e6     # bytes/ms -> GB/s
    out = {
        "metric": "tokens/sec at 1 GPU, 70B/7B-shape pair; verify-pass HBM GB/s % of peak",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / max(st["steps"], 1) * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: PEARL decode, target {cfg.target.n_layers}L d={cfg.target.d_model} "
                               f"Hq={cfg.target.n_heads} Hkv={cfg.target.n_kv_heads} F={cfg.target.d_ffn}, draft "
                               f"{cfg.draft.n_layers}L d={cfg.draft.d_model}, V={cfg.target.vocab}, batch 1, prompt "
                               f"{cfg.n_prompt}, temperature {cfg.temperature}, gamma {gamma} (c={tp / tq:.2f})",
                   "gamma": gamma, "c": tp / tq, "gamma_both_streams_busy": g_con, "c_both_streams_busy": tp_c / tq_c,
                   "n_prompt": cfg.n_prompt, "two_streams": True},
        "roofline": {"bound": "hbm", "kernel": "gemm_partial_kernel<1, 8, 0, 4> (target projections)",
                     "achieved": gemm_alone, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gemm_alone / HBM_PEAK_GBS,
                     "traffic": traffic, "launches": int(n_a), "avg_launch_us": ms_a / max(n_a, 1) * 1e3,
                     "avg_bytes_per_launch": bytes_a / max(n_a, 1), "read_ceiling_GBps": read_ceiling,
                     "note": "achieved = weight bytes of the target's projection launches / their durations by the kernel's own "
                             "wall-clock stamps (first workgroup in to last workgroup out), "
                             "measured in this run over 3 verify forwards (M = gamma, context = the prompt) with the GPU "
                             "to itself: the figure `rocprofv3 --kernel-trace --stats -- python3 bench.py --phase verify` "
                             "reproduces (profiles/verify_alone_70b_7b_kernel_stats.md; the tracer runs the two streams of "
                             "a PEARL step one after the other, so only the stream-alone figure can be traced).  "
                             "in_step_* = the same kernel inside the timed PEARL steps, where it shares the HBM pipe and "
                             "every CU with the draft stream: the K timed steps run a second time (same state, same "
                             "uniforms, same tokens) with the stamps switched on, which needs kernel-by-kernel "
                             "launches and costs instrumented_ms_per_step - ms_per_step.  read_ceiling_GBps = plain "
                             "16-byte loads over 2 GiB, 10 launches between two events, measured in this run.  traffic is not measured in this "
                             "run: it is read from profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on the "
                             "stand-alone projection driver, bytes per launch)",
                     "in_step_achieved": in_step, "in_step_frac": in_step / HBM_PEAK_GBS,
                     "in_step_launches": int(n_gemm), "in_step_avg_launch_us": ms_gemm / max(n_gemm, 1) * 1e3,
                     "instrumented_ms_per_step": elapsed_i / max(st_i["steps"], 1) * 1e3,
                     "instrumented_pass_same_tokens": same_tokens,
                     "verify_pass_frac_of_peak": alone_stats["verify_mgamma_frac_of_peak"],
                     "draft_pass_frac_of_peak": alone_stats["draft_frac_of_peak"]},
        "pearl": pearl, "alone": alone_stats, "side": side,
        "prefill": prefill_stats,
        "setup_s": {"build": t_build, "prefill": t_prefill},
    }
    if not args.no_cpu:
        torch.cuda.synchronize()
        out["cpu_baseline"] = cpu_baseline(cfg, gamma, dev)
    else:
        out["cpu_baseline"] = None
    ctx.close()
    print(json.dumps(out, default=float))


if __name__ == "__main__":
    main()
