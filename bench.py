#!/usr/bin/env python3
"""Throughput of the SJD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one SJD iteration (window forward + verification + window slide) of a running
generation, with weights, KV cache, window and loop state resident in HBM.  Prints ONE JSON line:
`ms_per_step` over exactly K timed steps; `value` = image tokens/s over WHOLE images (mean of the
images of seeds 0..4, with its range: the tokens an iteration fixes vary, so a rate taken over a few
steps of one image swings by 20 %, and late iterations read a longer cache than early ones); forward
passes per image for SJD and for ordinary auto-regressive decoding (the same loop with window 1); the
roofline position of the dominant kernel (the weight-streaming projections) measured inside the
library with HIP events that the runtime stamps with each kernel's own begin and end; the other
workloads (child processes, summarised under config.also_measured); and the CPU oracle timed on a
bounded sample of the same workload on this host's cores.

Only one GPU is used; --gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def recorded_traffic(workload):
    """HBM bytes per projection launch as rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE counted them (scaled by what
    the same counters read for a plain 1 GiB copy) in the committed run profiles/projections_<workload>.md,
    which ends in a line `traffic_bytes_per_launch: <read + written>`.  A recorded figure, not one of this run:
    the JSON names its source.  None when there is no such file."""
    path = os.path.join(ROOT, "profiles", f"projections_{workload}.md")
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch:"):
                return int(float(ln.split(":")[1].split()[0])), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(w, blob, prompt_ids, prompt_emb, seed, budget_steps):
    """The oracle as it stands, on a bounded sample: a truncated prompt (so that the CPU prefill
    stays short; untimed) and `budget_steps` timed SJD iterations."""
    import numpy as np
    import oracle
    om = oracle.Model(w.shape, blob)
    keep_ids = prompt_ids[:8]
    keep_emb = None if prompt_emb is None or len(prompt_emb) == 0 else prompt_emb[:8 - len(keep_ids)]
    P = len(keep_ids) + (0 if keep_emb is None else len(keep_emb))
    lp = om.prefill(keep_ids, keep_emb)
    smp = oracle.Sampler(w.top_k, w.temperature)
    init = oracle.Init(w.init_mode, w.row_stride, w.eol_id)
    lo, L = w.shape.samp_lo, w.window
    q0 = oracle.dist(lp, smp.top_k, smp.temperature)
    draft, p_old = oracle.first_window(q0, L, lo, init, seed)
    out = []
    t0 = time.perf_counter()
    for c in range(1, budget_steps + 1):
        logits = om.forward_tokens(P + len(out), draft)
        a, nd, pn = oracle.verify(logits, p_old, draft, lo, smp, init, len(out), np.array(out, np.int32), seed, c)
        out += draft[:a].tolist()
        draft, p_old = nd, pn
    dt = time.perf_counter() - t0
    om.close()
    return {"value": len(out) / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"prompt cut to {P} positions (prefill untimed), {budget_steps} SJD iterations of L={L} timed "
                      f"({len(out)} tokens fixed in {dt:.2f} s)",
            "s_per_step": dt / budget_steps}


def spread(xs):
    return {"mean": sum(xs) / len(xs), "min": min(xs), "max": max(xs), "n": len(xs)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256, help="timed iterations (ms_per_step)")
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="7b_32x32")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--images", type=int, default=5,
                    help="whole images generated for `value` (seeds seed .. seed + images - 1; 0 = none: value falls back to "
                         "the tokens fixed during the timed steps)")
    ap.add_argument("--profile-steps", type=int, default=24)
    ap.add_argument("--cpu-steps", type=int, default=-1, help="oracle iterations to time (0 = skip)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--skip-images", action="store_true", help="same as --images 0 --skip-ar")
    ap.add_argument("--window", type=int, default=0, help="override the workload's window size L")
    ap.add_argument("--top-k", type=int, default=0, help="override the workload's top-K (1 = greedy = Jacobi decoding)")
    ap.add_argument("--temperature", type=float, default=0.0, help="override the workload's sampling temperature")
    ap.add_argument("--init-mode", type=int, default=-1, help="override the initialiser: 0 uniform, 1 repeat above, 2 repeat left, 3 sample left, 4 sample above")
    ap.add_argument("--no-refine", action="store_true", help="ablation: no refinement of unaccepted drafts")
    ap.add_argument("--cfg", type=float, default=None,
                    help="classifier-free guidance weight: run a second (unconditional) context in every forward")
    ap.add_argument("--batch", type=int, default=1,
                    help="images decoded together, one pass over the weights per iteration")
    ap.add_argument("--skip-ar", action="store_true", help="skip the auto-regressive (window 1) image")
    ap.add_argument("--compare-init", type=int, default=-1,
                    help="also generate the images with this initialiser (same seeds) and report both side by side")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads measured afterwards in child processes and summarised under "
                         "config.also_measured ('none' = skip; default: every other configuration when the 7B default "
                         "runs unmodified)")
    ap.add_argument("--gemm-bench", default=None, metavar="M,N,K,tn,wk,u[,iters]",
                    help="only time the bf16 projection kernel alone at one shape and tiling (sjd_gemm_bench; cold weights "
                         "when iters < 0, default -40): for counter runs on single kernels")
    ap.add_argument("--gemm-sweep", default=None, metavar="M[,M...]",
                    help="only sweep the projection kernels alone over the 7B and 775M layer shapes at these row counts "
                         "(cold weights): skinny kernel with 3- and 4-byte activation planes and its wave / prefetch "
                         "variants up to 32 rows, wide kernel with its K-slice / group variants at any row count")
    ap.add_argument("--verify-scaled", action="store_true",
                    help="only time the sampling-distribution kernel (top-K + softmax of Step 3) at a scaled shape: 4096 "
                         "logits rows in one launch, where it is a bandwidth problem rather than a launch (off-path evidence)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain device copies of 1 GiB (reference for scaling HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (independent images per GPU is how it would scale); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.skip_images:
        args.images = 0
        args.skip_ar = True

    import numpy as np
    import torch
    from paper_2410_01699_amd import binding as B
    from paper_2410_01699_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4, "copies": 5}))
        return
    if args.gemm_bench:
        v = [int(x) for x in args.gemm_bench.split(",")]
        M_, N_, K_, tn_, wk_, u_ = v[:6]
        it_ = v[6] if len(v) > 6 else -40
        us = B.sjd_gemm_bench(M_, N_, K_, tn_, wk_, u_, it_)
        by = N_ * K_ * 2
        print(json.dumps({"M": M_, "N": N_, "K": K_, "tn": tn_, "wk": wk_, "u": u_, "iters": it_, "us_per_launch": us,
                          "weight_GBps": by / us / 1e3, "frac_of_hbm_peak": by / us / 1e3 / HBM_PEAK_GBS,
                          "mfma_TFLOPs_hi_and_lo": 4.0 * M_ * N_ * K_ / us / 1e6}))
        return
    if args.gemm_sweep:
        shapes = {"7b_qkv": (12288, 4096, 3), "7b_o": (4096, 4096, 1), "7b_gate_up": (22016, 4096, 2), "7b_down": (4096, 11008, 1),
                  "7b_lm_head": (8192, 4096, 2), "775m_qkv": (4608, 1536, 2), "775m_o": (1536, 1536, 1),
                  "775m_gate_up": (8192, 1536, 2), "775m_down": (1536, 4096, 1)}
        rows_out = []
        for M_ in [int(x) for x in args.gemm_sweep.split(",")]:
            for name, (N_, K_, tn_) in shapes.items():
                res = {"model's choice": B.sjd_gemm_bench(M_, N_, K_, tn_, 0, 0, -40)}
                # plain reads of the same weight bytes: by as many workgroups as the skinny kernel launches, each a
                # contiguous share (the kernel's own pattern), and the fastest plain read found (many workgroups
                # sweeping the bytes together)
                floor_us = B.sjd_gemm_bench(M_, N_, K_, 0, max(128, N_ // 16 // tn_), 0, -40)
                sweep_wgs = 1024 if N_ * K_ * 2 >= 1024 * 16384 * 4 else 256
                floor_best_us = B.sjd_gemm_bench(M_, N_, K_, 0, sweep_wgs, 1, -40)
                if M_ <= 32:
                    for wk_ in (4, 8):
                        for u_ in (2, 4):
                            for f_, fname in ((0, "3B"), (10, "4B")):
                                try:
                                    res[f"skinny wk{wk_} u{u_} {fname}"] = B.sjd_gemm_bench(M_, N_, K_, tn_, wk_, u_ + f_, -40)
                                except B.SjdError:
                                    pass
                for g_ in ((1, 2) if tn_ < 3 else (1,)):
                    for ks_ in (1, 2, 3, 4, 6, 8):
                        try:
                            res[f"wide g{g_} ks{ks_}"] = B.sjd_gemm_bench(M_, N_, K_, tn_, 100 + ks_, g_, -40)
                        except B.SjdError:
                            pass
                best = sorted(res.items(), key=lambda kv: kv[1])
                rows_out.append({"M": M_, "shape": name, "N": N_, "K": K_, "weight_MB": N_ * K_ * 2 / 1e6, "plain_read_us": round(floor_us, 2), "plain_read_sweep_us": round(floor_best_us, 2),
                                 "us": {k: round(v, 2) for k, v in best},
                                 "best": best[0][0], "best_TBps": N_ * K_ * 2 / best[0][1] / 1e6})
                log(f"M={M_} {name}: " + "  ".join(f"{k}: {v:.1f}us" for k, v in best[:5]))
        print(json.dumps({"gemm_sweep": rows_out}))
        return
    if args.verify_scaled:
        # Step 3's distribution kernel on many independent rows at once.  Algorithmic bytes: one fp32 logits row in,
        # one fp32 probability row out.  Timed with events on the stream the launches go to (torch's current = default).
        out = {"kernel": "sjd_dist_kernel (top-K select + softmax, one workgroup per row: 256 threads for V_s <= 8192 and 512 up to 16384 at this row count)", "peak_GBps": HBM_PEAK_GBS,
               "shapes": []}
        for V, K in ((8192, 2000), (16384, 2000), (8192, 8192)):
            rows = 4096
            z = torch.from_numpy(synth.random_logits(rows, V, seed=5)).cuda()
            q = torch.empty_like(z)
            smp = B.sjd_sampler(K, 1.0)
            for _ in range(3):
                B.sjd_dist(z, rows, V, smp, None, q)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            iters = 20
            e0.record()
            for _ in range(iters):
                B.sjd_dist(z, rows, V, smp, None, q)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / iters
            by = rows * V * 8
            out["shapes"].append({"rows": rows, "V_s": V, "top_k": K, "us_per_launch": us, "algorithmic_bytes": by,
                                  "GBps": by / us / 1e3, "frac_of_hbm_peak": by / us / 1e3 / HBM_PEAK_GBS,
                                  "rows_per_s": rows / us * 1e6})
        print(json.dumps(out))
        return
    w = synth.WORKLOADS[args.workload]
    import dataclasses
    if args.window > 0:
        w = dataclasses.replace(w, window=args.window)
    if args.top_k > 0:
        w = dataclasses.replace(w, top_k=args.top_k)
    if args.init_mode >= 0:
        w = dataclasses.replace(w, init_mode=args.init_mode)
    if args.temperature > 0:
        w = dataclasses.replace(w, temperature=args.temperature)
    # (a larger window than the workload's own needs a few more cache rows)
    need = w.n_prompt_ids + w.n_prompt_embeds + w.n_image_tokens + w.window
    if need > w.shape.max_seq:
        w = dataclasses.replace(w, shape=dataclasses.replace(w.shape, max_seq=need))
    shape = w.shape
    t0 = time.perf_counter()
    blob = synth.make_weights(shape, seed=0, threads=16)
    log(f"weights: {shape.n_params() / 1e9:.2f} G params generated in {time.perf_counter() - t0:.1f} s")
    ids, emb = synth.make_prompt(w)
    t0 = time.perf_counter()
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kv = B.sjd_kv_create(m)
    nb = args.batch
    kvs = [kv] + [B.sjd_kv_create(m) for _ in range(nb - 1)]
    log(f"model on device in {time.perf_counter() - t0:.1f} s")
    if args.no_graph:
        B.sjd_kv_use_graph(kv, False)
    smp = B.sjd_sampler(w.top_k, w.temperature)
    flags = 1 if args.no_refine else 0
    init = B.sjd_init(w.init_mode, w.row_stride, w.eol_id, flags)
    N, L = w.n_image_tokens, w.window
    q_first = torch.empty(shape.v_s, dtype=torch.float32, device="cuda")
    guided = args.cfg is not None
    # the unconditional context: a short synthetic prompt of its own (a quarter of the conditional one)
    u_ids = synth.random_tokens(max(1, (len(ids) + len(emb)) // 4), 0, shape.samp_lo or shape.vocab_total, seed=77)
    rows_per_image = (1 << max(0, (L - 1).bit_length())) if nb > 1 else L
    rows_needed = rows_per_image * nb * (2 if guided else 1)
    if L > B.SJD_MAX_WINDOW or rows_needed > B.SJD_MAX_ROWS or (nb > 1 and (shape.dtype != 1 or nb * (2 if guided else 1) > 8)):
        print(f"bench.py: window {L} x batch {nb}{' x 2 contexts' if guided else ''} does not fit one forward "
              f"(at most {B.SJD_MAX_ROWS} rows and 8 contexts, windows up to {B.SJD_MAX_WINDOW}; batches need a bf16 model)",
              file=sys.stderr)
        sys.exit(2)
    # every image of a batch has its own prompt (same length, different ids)
    prompts = [ids] + [synth.random_tokens(len(ids), 0, shape.samp_lo or shape.vocab_total, seed=200 + b)
                       for b in range(1, nb)]

    image = [args.seed]

    def new_image():
        for b, h in enumerate(kvs):
            B.sjd_prefill(m, h, prompts[b] if len(ids) else ids, emb, smp, init, q_first)
            if guided:
                B.sjd_prefill_uncond(m, h, u_ids, None, args.cfg, smp, init, q_first)
            B.sjd_decode_begin(m, h, q_first, N, L, smp, init, image[0])
            image[0] += 1
        torch.cuda.synchronize()

    def safe_steps():
        """iterations every image can still run without finishing, tokens fixed so far (all images)"""
        safe, fixed_all = 1 << 30, 0
        for h in kvs:
            fixed, _, done = B.sjd_decode_status(h)
            safe = min(safe, 0 if done else (N - 2 - fixed) // L)
            fixed_all += fixed
        return safe, fixed_all

    def steps(k):
        if nb > 1:
            B.sjd_decode_steps_batch(m, kvs, k)
        else:
            B.sjd_decode_steps(m, kv, k)

    def run_steps(k, timed):
        """exactly k iterations of a live generation; returns (seconds, tokens fixed)"""
        secs, toks = 0.0, 0
        while k > 0:
            safe, fixed0 = safe_steps()
            if safe < 1:
                new_image()
                continue
            seg = min(k, safe)
            torch.cuda.synchronize()
            t = time.perf_counter()
            steps(seg)
            torch.cuda.synchronize()
            secs += time.perf_counter() - t
            _, fixed1 = safe_steps()
            toks += fixed1 - fixed0
            k -= seg
        return secs, toks

    new_image()
    run_steps(args.warmup, False)
    secs, toks = run_steps(args.steps, True)
    ms_per_step = secs / args.steps * 1e3
    log(f"{args.steps} steps: {ms_per_step:.3f} ms/step, {toks} tokens fixed, {toks / secs:.1f} tokens/s over these steps")

    # ---- roofline of the dominant kernel: HIP events around every launch, same stream ----
    prof_steps = args.profile_steps
    safe, _ = safe_steps()
    if safe < prof_steps:
        new_image()
    p = B.sjd_profile_steps_batch(m, kvs, prof_steps) if nb > 1 else B.sjd_profile_steps(m, kv, prof_steps)
    classes = {}
    for i, name in enumerate(B.PROF_KINDS):
        ms, by, n = p.ms[i], p.bytes[i], p.launches[i]
        classes[name] = {"ms_per_step": ms / prof_steps, "launches_per_step": n / prof_steps,
                         "us_per_launch": (ms * 1e3 / n) if n else None,
                         "algorithmic_GB_per_step": by / prof_steps / 1e9,
                         "GBps": (by / 1e9) / (ms / 1e3) if ms > 0 else None}
    g = classes["gemm"]
    # the projections alone, back to back (no per-launch dispatch latency inside the interval)
    g["ms_per_step_back_to_back"] = p.ms_gemm_back_to_back / prof_steps
    g["us_per_launch"] = p.ms_gemm_back_to_back * 1e3 / p.launches[0]
    g["GBps"] = (p.bytes[0] / 1e9) / (p.ms_gemm_back_to_back / 1e3)
    # Attention: the library counts the K/V bytes AS STORED for the positions actually cached during the
    # profiled iterations (device-resident lengths, read before each one).  bf16 models store every value as
    # a hi + lo bf16 pair (4 bytes), twice the 2 bytes per value that the plain algorithm's count assumes.
    at = classes["attention"]
    stored_over_alg = 2.0 if shape.dtype == 1 else 1.0
    at["stored_GB_per_step"] = at.pop("algorithmic_GB_per_step")
    at["GBps_stored"] = at.pop("GBps")
    at["algorithmic_GB_per_step"] = at["stored_GB_per_step"] / stored_over_alg
    at["GBps_algorithmic"] = None if at["GBps_stored"] is None else at["GBps_stored"] / stored_over_alg
    at["stored_over_algorithmic_bytes"] = stored_over_alg
    at["kv_bytes_per_token_stored"] = 2 * shape.n_layers * shape.d_model * (4 if shape.dtype == 1 else 4)
    at["kv_bytes_per_token_algorithmic"] = 2 * shape.n_layers * shape.d_model * (2 if shape.dtype == 1 else 4)
    plain = (nb == 1 and not guided and args.window == 0 and args.top_k == 0 and args.temperature == 0
             and args.init_mode < 0 and not args.no_refine and not args.no_graph)
    # (the counter runs were made on the default configuration of a workload only)
    traffic, traffic_src = recorded_traffic(args.workload) if plain else (None, None)
    roofline = {"bound": "hbm", "kernel": "gemm_fused_kernel (all projections + LM head)" if shape.dtype == 1
                else "gemm_f32_kernel", "achieved": g["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": g["GBps"] / HBM_PEAK_GBS, "traffic": traffic,
                "traffic_source": None if traffic is None else f"recorded rocprofv3 --pmc run, {traffic_src} (not measured by this run)",
                "bytes_per_launch": g["algorithmic_GB_per_step"] * 1e9 / g["launches_per_step"],
                "us_per_launch": g["us_per_launch"], "launches_per_step": g["launches_per_step"]}
    weight_bytes = g["algorithmic_GB_per_step"] * 1e9
    step_floor_ms = weight_bytes / (HBM_PEAK_GBS * 1e9) * 1e3
    log(f"gemm: {g['GBps']:.0f} GB/s over {g['launches_per_step']:.0f} launches/step; "
        f"whole step at {weight_bytes / 1e9 / (ms_per_step / 1e3):.0f} GB/s of weight stream")

    # ---- whole images: tokens/s (the headline), forward passes per image, SJD vs ordinary AR (window 1) ----
    extra = {}

    class _LoopStats:
        pass

    def generate_guided_batch(window, ini, seed):
        """guided batches have no one-call entry point: prefill both contexts of every image, then drive the batched
        loop in pieces (a few iterations per call, never more than the image furthest from its end can still take)"""
        for b, h in enumerate(kvs):
            B.sjd_prefill(m, h, prompts[b] if len(ids) else ids, emb, smp, ini, q_first)
            B.sjd_prefill_uncond(m, h, u_ids, None, args.cfg, smp, ini, q_first)
            B.sjd_decode_begin(m, h, q_first, N, window, smp, ini, seed * nb + b)
        torch.cuda.synchronize()
        t = time.perf_counter()
        most_left, all_done, n_steps = N - 1, False, 0
        while not all_done:
            k = max(1, min(8, (most_left + window - 1) // window))
            B.sjd_decode_steps_batch(m, kvs, k)
            all_done, most_left = True, 0
            for h in kvs:
                fixed, st_steps, done = B.sjd_decode_status(h)
                all_done &= done
                n_steps = max(n_steps, st_steps)
                if not done:
                    most_left = max(most_left, N - 1 - fixed)
        st = _LoopStats()
        st.ms_decode = (time.perf_counter() - t) * 1e3
        st.steps = n_steps
        return None, st

    def generate(window, ini, seed):
        if nb > 1 and guided:
            return generate_guided_batch(window, ini, seed)
        if nb > 1:
            t, sts = B.sjd_generate_batch(m, kvs, prompts, None if not len(emb) else [emb] * nb, N, window, smp, ini,
                                          [seed * nb + b for b in range(nb)])
            return t, sts[0]
        if guided:
            return B.sjd_generate_cfg(m, kv, ids, emb, u_ids, None, args.cfg, N, window, smp, ini, seed)
        return B.sjd_generate(m, kv, ids, emb, N, window, smp, ini, seed)

    def images(ini):
        """args.images whole generations: per-image tokens/s, forwards, tokens fixed per forward"""
        rate, fwd = [], []
        for sd in range(args.seed, args.seed + args.images):
            _, st = generate(L, ini, sd)
            rate.append(nb * N / (st.ms_decode / 1e3))
            fwd.append(st.steps)
        return {"seeds": list(range(args.seed, args.seed + args.images)),
                "image_tokens_per_s": spread(rate), "forwards_per_image": spread(fwd),
                "tokens_fixed_per_forward": spread([N / f for f in fwd]),
                "ms_per_forward_whole_image": spread([nb * N / r * 1e3 / f for r, f in zip(rate, fwd)])}

    value, value_basis = toks / secs, f"tokens fixed during the {args.steps} timed steps (no whole image was generated)"
    if args.images > 0:
        t = time.perf_counter()
        im = images(init)
        extra["whole_images"] = im
        value = im["image_tokens_per_s"]["mean"]
        value_basis = (f"whole images: N = {N} image tokens{' x ' + str(nb) + ' images' if nb > 1 else ''} / wall time of the decoding "
                       f"loop, mean over seeds {im['seeds'][0]}..{im['seeds'][-1]} (prefill excluded, as in the paper's protocol)")
        extra["sjd_forwards_per_image"] = im["forwards_per_image"]["mean"]
        log(f"{args.images} images: {value:.1f} tokens/s (min {im['image_tokens_per_s']['min']:.1f}, max "
            f"{im['image_tokens_per_s']['max']:.1f}), {im['forwards_per_image']['mean']:.0f} forwards/image "
            f"({time.perf_counter() - t:.1f} s)")
        if args.compare_init >= 0:
            other = B.sjd_init(args.compare_init, w.row_stride, w.eol_id, flags)
            extra["whole_images_init_mode_%d" % args.compare_init] = images(other)
    if not args.skip_ar:
        _, sa = generate(1, init, args.seed)
        extra["ar_forwards_per_image"] = sa.steps
        extra["ar_image_seconds"] = sa.ms_decode / 1e3
        extra["ar_image_tokens_per_s"] = nb * N / (sa.ms_decode / 1e3)
        if args.images > 0:
            extra["step_compression"] = sa.steps / extra["sjd_forwards_per_image"]
            extra["latency_speedup_vs_ar"] = value / extra["ar_image_tokens_per_s"]
        log(f"AR image: {sa.steps} forwards / {sa.ms_decode:.0f} ms")
    for h in kvs:
        B.sjd_kv_free(h)
    B.sjd_free_model(m)

    cpu_steps = args.cpu_steps
    if cpu_steps < 0:
        cpu_steps = 3 if shape.n_params() > 2e9 else (8 if shape.n_params() > 1e8 else 40)
    cpu = None
    if guided or nb > 1:
        cpu_steps = 0          # the CPU leg times the unguided single-image path only
    if cpu_steps > 0:
        log("timing the CPU oracle on a bounded sample ...")
        cpu = cpu_baseline(w, blob, ids, emb, args.seed, cpu_steps)
    del blob

    out = {
        "metric": "image_tokens_per_s", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if shape.dtype == 1 else "f32", "data": "synthetic",
        "value_basis": value_basis,
        "tokens_per_s_over_timed_steps": toks / secs,
        "config": {"workload": w.name, "window_L": L, "top_k": w.top_k, "temperature": w.temperature,
                   "init_mode": w.init_mode, "no_refine": bool(args.no_refine), "cfg_weight": args.cfg, "batch_images": nb,
                   "uncond_prompt_positions": len(u_ids) if guided else None,
                   "image_tokens_N": N, "prompt_positions": len(ids) + len(emb), "layers": shape.n_layers,
                   "d_model": shape.d_model, "sampling_vocab": shape.v_s, "hip_graph": not args.no_graph,
                   "rows_per_forward": rows_needed,
                   "tokens_fixed_per_step_timed": toks / args.steps, "step_hbm_floor_ms": step_floor_ms,
                   "step_weight_stream_GBps": weight_bytes / 1e9 / (ms_per_step / 1e3), **extra},
        "roofline": roofline, "kernel_classes": classes, "cpu_baseline": cpu,
    }
    also = args.also
    if also is None:
        also = "775m,tiny,7b_48x48" if (plain and args.workload == "7b_32x32") else "none"
    if also != "none":
        # the other configurations, same measurement without the CPU leg, each in a process of its own (this one
        # has released the GPU memory; their lines are parsed, not re-printed).  The 48 x 48 workload generates
        # its images twice: uniform initialisation and repeat-above, same seeds, side by side.
        import subprocess
        out["config"]["also_measured"] = {}
        for name in also.split(","):
            log(f"measuring workload {name} in a child process ...")
            cmd = [sys.executable, os.path.abspath(__file__), "--workload", name, "--also", "none", "--cpu-steps", "0",
                   "--steps", str(args.steps), "--warmup", str(args.warmup), "--images", str(args.images)]
            if name == "7b_48x48":
                cmd += ["--compare-init", "1"]
            r = subprocess.run(cmd, capture_output=True, text=True)
            line = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
            if r.returncode == 0 and line:
                o = json.loads(line[-1])
                c = o["config"]
                keep = {k: c[k] for k in c if k.startswith("whole_images") or k in
                        ("window_L", "init_mode", "image_tokens_N", "ar_forwards_per_image", "ar_image_tokens_per_s",
                         "step_compression", "latency_speedup_vs_ar", "tokens_fixed_per_step_timed")}
                out["config"]["also_measured"][name] = {
                    "value": o["value"], "unit": o["unit"], "ms_per_step": o["ms_per_step"], "dtype": o["dtype"], **keep,
                    "roofline": {k: o["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac")}}
            else:
                out["config"]["also_measured"][name] = {"error": (r.stderr or "no output")[-300:]}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
