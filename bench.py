#!/usr/bin/env python3
"""Benchmark of the AdaDecode hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic input: Algorithm 1 generating `gen_len` tokens
from a `prompt_len`-token random prompt on the Llama-3-8B-shaped bf16 model (32 layers, exit heads at layers
8/16/24, threshold 0.9, random-init weights), inputs and weights resident in HBM before the timed region.
value = generated tokens / wall time of the timed steps (prefill of the prompt included).

The same JSON line also carries:
  roofline      the weight-streaming kernel sampled live with stream events during the timed steps
  layer_step    the single-layer microbenchmark: 1000 ragged calls per row count m at context 4096, every call on
                freshly drawn N(0,1) rows (pre-generated on the device), rotating over the model's 32 distinct
                layers so that no cache can hold the weights
  forced        the same generation with exits forced from a seeded schedule (0.2/0.2/0.2 at layers 8/16/24)
  long          the long-generation workload: prompt 1024, 8192 generated tokens, the same kind of forced schedule,
                verification on, context growing to 9216
  cpu_baseline  the CPU oracle, as it stands, timed on bounded samples on this machine's host cores: Algorithm 1 on the
                benchmark's model, the tiny fp32 workload in full, and ten layer steps per m of the microbenchmark,
                at all cores and on one thread
  gamma_sweep   (only with --gamma-sweep) the threshold sweep of Fig. 5 and the schedule switches of Table 3, in shape
                only: early-prediction rate, rejection rate and tokens/s per threshold, thresholds placed at quantiles
                of the synthetic model's own head confidences (random-init heads are never 0.9-confident)
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


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def layer_step_bytes(shape, ctx, m):
    s = shape.elem_bytes()
    return shape.layer_weight_elems() * s + 2 * shape.d_kv * s * (ctx + m) + 2 * shape.d_kv * s * m


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="8b", choices=["8b", "13b", "8b-long", "8b-mini", "tiny"],
                    help="8b-long: the timed steps are the long-generation workload itself (forced schedule)")
    ap.add_argument("--gen-len", type=int, default=None)
    ap.add_argument("--prompt-len", type=int, default=None)
    ap.add_argument("--micro-calls", type=int, default=None, help="layer-step calls per m in the microbenchmark (default 1000)")
    ap.add_argument("--skip-long", action="store_true")
    ap.add_argument("--phase-trace", action="store_true",
                    help="fused layer mode: also report where a layer step's time goes, phase by phase (the kernel's own timestamps)")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--skip-micro", action="store_true")
    ap.add_argument("--skip-forced", action="store_true")
    ap.add_argument("--skip-decision", action="store_true", help="skip the measurement of the host's cost per exit decision")
    ap.add_argument("--gamma-sweep", action="store_true", help="also run the threshold sweep and the ablation switches")
    ap.add_argument("--layer-mode", default="kernels", choices=["fused", "kernels"],
                    help="layer step as one kernel per phase (default) or as one persistent kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no sharding, no collectives); run with --gpus 1")
        sys.exit(2)

    import torch
    from paper_2506_03700_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    shape = synth.SHAPES[args.workload]
    gen_len = args.gen_len or shape.gen_len
    prompt_len = args.prompt_len or shape.prompt_len
    cap = 7
    ctx_micro = 4096
    micro_calls = args.micro_calls or synth.MICRO_CALLS
    main_is_long = args.workload == "8b-long"
    # the long-generation leg rides along with the 8B workload (same model); it needs the deeper cache
    long_shape = synth.LLAMA8B_LONG
    with_long = (args.workload == "8b" and not args.skip_long and args.gen_len is None and args.prompt_len is None)
    max_pos = max(prompt_len + gen_len + 8, ctx_micro + 16, (long_shape.prompt_len + long_shape.gen_len + 8) if with_long else 0)

    t0 = time.time()
    w = synth.make_weights(shape, seed=0)
    log(f"[bench] weights for {shape.name} generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    g = binding.Model(shape, w, max_pos=max_pos)
    log(f"[bench] model on device in {time.time() - t0:.1f}s")
    prompt = synth.make_prompt(shape, 0, n=prompt_len)
    fused = args.layer_mode == "fused" and shape.dtype == synth.BF16
    g.ad_set_layer_mode(binding.AD_LAYER_FUSED if fused else binding.AD_LAYER_KERNELS)

    main_sched = synth.make_forced_schedule(shape, 0, max_pos) if main_is_long else None

    def run(**kw):
        if main_is_long:
            kw = dict(kw, forced_exit=main_sched)
        return g.ad_generate(prompt, gen_len, shape.gamma, cap, want_events=False, **kw)

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    g.ad_profile_start(binding.AD_PROF_LAYER if fused else binding.AD_PROF_GEMM, period=7, max_samples=16384)
    t0 = time.perf_counter()
    stats = None
    for _ in range(args.steps):
        toks, stats, _ = run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = g.ad_profile_stop()
    tokens_per_s = args.steps * gen_len / dt
    log(f"[bench] {args.steps} x {gen_len} tokens in {dt:.3f}s -> {tokens_per_s:.1f} tok/s; stats {stats}")

    # HBM traffic per launch: algorithmic bytes x the measured ratio (rocprofv3 FETCH_SIZE + WRITE_SIZE of the four
    # GEMM launches of a layer step, calibrated on a copy of known size; see the file named in traffic_source)
    traffic_ratio, traffic_src = None, os.path.join("profiles", "layer_step_8b_ctx4096_hbm_traffic.md")
    ratio_key = "traffic_ratio_layer_fused" if fused else "traffic_ratio_gemm"
    try:
        for line in open(os.path.join(ROOT, traffic_src)):
            if line.startswith(ratio_key):
                traffic_ratio = float(line.split("=")[1].split()[0])
    except OSError:
        pass
    avg_ms = prof["sampled_ms"] / max(1, prof["samples"])
    avg_bytes = prof["sampled_bytes"] / max(1, prof["samples"])
    achieved = avg_bytes / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
    kernel = ("ad::k_layer_fused (one decoder-layer step over the call's m rows as one persistent kernel: QKV, attention, "
              "Wo, gate/up, down; bytes = the layer's weights + KV rows read and written)") if fused else \
             ("ad::k_gemm (weight-streaming skinny GEMM: every projection of the layer step and the vocabulary pass)")
    roofline = {"bound": "hbm", "kernel": kernel,
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "time_base": "a pair of events on the launch stream around each sampled launch (every 7th), i.e. from the end of the "
                             "previous kernel to the end of the sampled one: the dispatch gap ahead of the kernel is inside the "
                             "figure; rocprofv3's own duration of the same kernel (profiles/) is shorter by that gap",
                "traffic": None if traffic_ratio is None else int(avg_bytes * traffic_ratio),
                "traffic_source": None if traffic_ratio is None else f"{traffic_src}: measured HBM bytes / algorithmic bytes = {traffic_ratio}",
                "avg_launch_us": round(avg_ms * 1e3, 2), "avg_bytes_per_launch": int(avg_bytes),
                "launches": prof["launches"], "sampled": prof["samples"]}
    decode_bytes = stats["bytes_algorithmic"]
    e2e = {"algorithmic_GB_per_step": round(decode_bytes / 1e9, 3),
           "achieved_GBps_whole_step": round(args.steps * decode_bytes / dt / 1e9, 1),
           "layer_steps_per_s": round(args.steps * stats["layer_steps"] / dt, 1),
           "early_preds": stats["early_preds"], "rejections": stats["rejections"], "head_evals": stats["head_evals"],
           "note": "random-init exit heads are never 0.9-confident: at the workload's threshold no exit is taken, so `value` is plain "
                   "decoding plus the head evaluations that never fire; the adaptive path (ragged steps, deferred layers, rejections) "
                   "is timed in `forced` and `long`" if stats["early_preds"] == 0 else ""}

    forced = None
    if not args.skip_forced and shape.exit_layers and not main_is_long:
        sched = synth.make_forced_schedule(shape, 0, max_pos)
        g.ad_generate(prompt, min(gen_len, 64), shape.gamma, cap, forced_exit=sched, want_events=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, fst, _ = g.ad_generate(prompt, gen_len, shape.gamma, cap, forced_exit=sched, want_events=False)
        torch.cuda.synchronize()
        fdt = time.perf_counter() - t0
        forced = {"schedule": "each token exits at an exit layer with probability 0.2 each, else full depth (seeded)",
                  "tokens_per_s": round(gen_len / fdt, 1), "layer_steps": fst["layer_steps"], "steps_by_m": fst["steps_by_m"],
                  "early_preds": fst["early_preds"], "rejections": fst["rejections"],
                  "achieved_GBps": round(fst["bytes_algorithmic"] / fdt / 1e9, 1)}
        log(f"[bench] forced schedule: {forced}")

    long = None
    if with_long:
        lp = synth.make_prompt(long_shape, 0, n=long_shape.prompt_len)
        lsched = synth.make_forced_schedule(long_shape, 0, max_pos)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, lst, _ = g.ad_generate(lp, long_shape.gen_len, long_shape.gamma, cap, forced_exit=lsched, want_events=False)
        torch.cuda.synchronize()
        ldt = time.perf_counter() - t0
        long = {"workload": f"prompt {long_shape.prompt_len}, {long_shape.gen_len} generated tokens, context to "
                            f"{long_shape.prompt_len + long_shape.gen_len}; each token exits at an exit layer with probability 0.2 each, "
                            "else full depth (seeded), verification on; one run, prefill included",
                "tokens_per_s": round(long_shape.gen_len / ldt, 1), "seconds": round(ldt, 2),
                "layer_steps_per_s": round(lst["layer_steps"] / ldt, 1), "layer_steps": lst["layer_steps"],
                "steps_by_m": lst["steps_by_m"], "early_preds": lst["early_preds"], "rejections": lst["rejections"],
                "head_evals": lst["head_evals"], "verifies": lst["verifies"],
                "algorithmic_GB": round(lst["bytes_algorithmic"] / 1e9, 1),
                "achieved_GBps": round(lst["bytes_algorithmic"] / ldt / 1e9, 1),
                "frac_of_peak": round(lst["bytes_algorithmic"] / ldt / 1e9 / HBM_PEAK_GBS, 4)}
        log(f"[bench] long generation: {long}")

    # What the host's part in an exit decision costs: a token with a head evaluation after each exit layer and the
    # verification (4 per token on the 8B shape) against a token with the verification only (cap 0: no exit head is
    # evaluated), per extra evaluation, minus what an evaluation takes when evaluations are queued back to back on
    # the stream with no host in between.  Both with and without the issue-ahead of the expected continuation.
    decision = None
    if not args.skip_decision and shape.exit_layers and not main_is_long:
        n_dc = min(gen_len, 384)

        def us_per_token(cap_, ahead):
            g.ad_generate(prompt, 32, shape.gamma, cap_, want_events=False, no_issue_ahead=not ahead)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            _, st, _ = g.ad_generate(prompt, n_dc, shape.gamma, cap_, want_events=False, no_issue_ahead=not ahead)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / n_dc * 1e6, st

        hrow = torch.from_numpy(synth.make_hidden(shape, 7, 1)).to("cuda")
        for _ in range(20):
            g.ad_exit_head(shape.exit_layers[0], hrow, sync=False)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(200):
            g.ad_exit_head(shape.exit_layers[0], hrow, sync=False)
        e1.record()
        torch.cuda.synchronize()
        head_us = e0.elapsed_time(e1) * 1e3 / 200
        decision = {"tokens": n_dc, "head_evaluation_back_to_back_us": round(head_us, 2),
                    "note": "us_per_token figures include the prompt's prefill spread over the run's tokens (the same in both runs of a "
                            "pair, so it cancels in us_per_extra_head_evaluation)"}
        for ahead in (True, False):
            t_all, st_all = us_per_token(cap, ahead)
            t_one, st_one = us_per_token(0, ahead)
            extra = (st_all["head_evals"] + st_all["verifies"] - st_one["verifies"]) / n_dc      # evaluations per token beyond the verification
            per_eval = (t_all - t_one) / extra
            decision["issue_ahead" if ahead else "no_issue_ahead"] = {
                "us_per_token": round(t_all, 1), "us_per_token_verification_only": round(t_one, 1),
                "head_evaluations_per_token": round(extra + 1, 3), "us_per_extra_head_evaluation": round(per_eval, 2),
                "host_decision_us": round(per_eval - head_us, 2),
                "share_of_token": round((extra + 1) * (per_eval - head_us) / t_all, 5)}
        log(f"[bench] host decision cost: {decision}")

    sweep = None
    if args.gamma_sweep and shape.exit_layers:
        n_sw = min(gen_len, 256)

        def timed(gamma, **kw):
            g.ad_generate(prompt, min(n_sw, 32), gamma, cap, want_events=False, **kw)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            _, st, _ = g.ad_generate(prompt, n_sw, gamma, cap, want_events=False, **kw)
            torch.cuda.synchronize()
            sdt = time.perf_counter() - t0
            return {"gamma": float(gamma), "tokens_per_s": round(n_sw / sdt, 1),
                    "early_prediction_rate": round(st["early_preds"] / max(1, st["early_preds"] + st["verifies"]), 4),
                    "rejection_rate": round(st["rejections"] / max(1, st["early_preds"]), 4),
                    "layer_steps": st["layer_steps"], "head_evals": st["head_evals"], "steps_by_m": st["steps_by_m"]}

        # the confidences the heads report when nothing exits (gamma = 1): their quantiles place the thresholds
        _, _, ev = g.ad_generate(prompt, n_sw, 1.0, cap)
        confs = np.sort(ev[ev["kind"] == binding.EV_HEAD]["conf"].astype(np.float64))
        rows = []
        for q in (1.0, 0.9, 0.75, 0.5, 0.25, 0.1, 0.0):
            gam = 1.0 if q == 1.0 else (0.0 if q == 0.0 else float(confs[int(q * (len(confs) - 1))]))
            r = timed(gam)
            r["confidence_quantile"] = q
            rows.append(r)
            log(f"[bench] gamma sweep: {r}")
        gam = float(confs[len(confs) // 2])
        abl = []
        for name, kw in [("all heads, verified", {}), ("no verification", {"no_verify": True})] + \
                        [(f"only the head at layer {l}", {"head_mask": 1 << i}) for i, l in enumerate(shape.exit_layers)]:
            r = timed(gam, **kw)
            r["variant"] = name
            abl.append(r)
            log(f"[bench] ablation: {r}")
        sweep = {"tokens": n_sw, "note": "thresholds at quantiles of the head confidences of this random-init model; "
                 "early_prediction_rate = early predictions / (early predictions + tokens produced by the last layer)",
                 "rows": rows, "ablations_at_median_confidence": abl}

    micro = None
    if not args.skip_micro:
        micro = {}
        K, V = g.kv_views()
        gen = torch.Generator(device="cuda").manual_seed(0)
        K[:, :, :ctx_micro, :] = torch.randn(K[:, :, :ctx_micro, :].shape, generator=gen, device="cuda").to(K.dtype)
        V[:, :, :, :ctx_micro] = torch.randn(V[:, :, :, :ctx_micro].shape, generator=gen, device="cuda").to(V.dtype)
        L = shape.n_layers
        dgen = torch.Generator(device="cuda")

        def rows_for(m, n, first_from_synth=0):
            """[n, m, d] N(0,1) rows, one slice per call: the first calls' rows are the ones the parity test checks
            against the oracle (synth.micro_call_seed), the rest are drawn on the device from the next seed."""
            dgen.manual_seed(synth.micro_call_seed(m, first_from_synth))
            buf = torch.randn((n, m, shape.d_model), generator=dgen, device="cuda", dtype=torch.float32)
            for c in range(min(first_from_synth, n)):
                buf[c] = torch.from_numpy(synth.make_hidden(shape, synth.micro_call_seed(m, c), m)).to("cuda")
            return buf

        def timed_batches(fn, n_calls, n_batches=10):
            """Mean over all calls and median over the batch means (events on the launch stream)."""
            per = max(1, n_calls // n_batches)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_batches + 1)]
            ev[0].record()
            for b in range(n_batches):
                for i in range(per):
                    fn(b * per + i)
                ev[b + 1].record()
            torch.cuda.synchronize()
            t = [ev[b].elapsed_time(ev[b + 1]) * 1e3 / per for b in range(n_batches)]
            return float(np.mean(t)), float(np.median(t))

        for m in synth.MICRO_M:
            pos = np.arange(ctx_micro, ctx_micro + m)
            calls = micro_calls
            n_warm = 64
            H = rows_for(m, calls, first_from_synth=10)
            Hw = torch.randn((n_warm, m, shape.d_model), generator=dgen, device="cuda")     # warm-up rows

            def one(i, buf=H):
                layer = i % L + 1
                g.kv_set_len(layer, ctx_micro)
                g.ad_layer_step(layer, buf[i], pos)

            for i in range(n_warm):
                one(i, Hw)
            torch.cuda.synchronize()
            us, us_med = timed_batches(one, calls)
            gbs = layer_step_bytes(shape, ctx_micro, m) / (us * 1e-6) / 1e9
            micro[str(m)] = {"us": round(us, 2), "us_median_of_10_batches": round(us_med, 2), "GBps": round(gbs, 1),
                             "frac": round(gbs / HBM_PEAK_GBS, 4)}
            if m == 1:
                # the same call on ONE layer's weights over and over: the 256 MB memory-side cache may serve part of them
                H1 = torch.randn((calls, m, shape.d_model), generator=dgen, device="cuda")

                def same(i):
                    g.kv_set_len(1, ctx_micro)
                    g.ad_layer_step(1, H1[i], pos)
                for i in range(16):
                    one(i, Hw)
                torch.cuda.synchronize()
                us1, _ = timed_batches(same, calls)
                micro[str(m)]["us_single_weight_copy_cache_assisted"] = round(us1, 2)
            if L % 8 == 0:
                # the same layers as stretches of 8 per call (what ad_generate issues between two exit heads)
                n8 = max(10, calls // 8)
                H8 = torch.randn((n8, m, shape.d_model), generator=dgen, device="cuda")

                def stretch(i, buf=H8):
                    first = (i * 8) % L + 1
                    for layer in range(first, first + 8):
                        g.kv_set_len(layer, ctx_micro)
                    g.ad_layer_steps(first, 8, buf[i], pos)
                for i in range(8):
                    stretch(i, Hw)
                torch.cuda.synchronize()
                us8, _ = timed_batches(stretch, n8)
                gbs8 = layer_step_bytes(shape, ctx_micro, m) / (us8 / 8 * 1e-6) / 1e9
                micro[str(m)]["us_per_layer_in_stretches_of_8"] = round(us8 / 8, 2)
                micro[str(m)]["frac_in_stretches_of_8"] = round(gbs8 / HBM_PEAK_GBS, 4)
            if fused and args.phase_trace and L % 8 == 0:
                # the fused kernel's own clock: per workgroup, ticks before and after each grid barrier of the last layer
                # of a launch (a steady-state layer when the launch covers 8); a phase ends when its last workgroup is done
                tr = g.ad_layer_trace(True)
                acc = []
                for i in range(16):
                    stretch(i % n8)
                    torch.cuda.synchronize()
                    if i >= 4:
                        acc.append(tr.cpu().numpy().copy())
                g.ad_layer_trace(False)
                a = np.stack(acc).astype(np.float64) * 0.01                       # us, [launch, workgroup, stamp]
                a -= a[:, :, 0].max(axis=1)[:, None, None]                        # 0 = the last workgroup entering the layer
                names = ["QKV", "barrier", "attention", "barrier", "fold", "barrier", "Wo", "barrier", "gate/up", "barrier", "down"]
                ends = a.max(axis=1).mean(axis=0)
                micro[str(m)]["fused_phase_end_us"] = {f"{j:02d} {nm}": round(float(ends[j + 1]), 2) for j, nm in enumerate(names)}
                micro[str(m)]["fused_phase_mean_us_per_workgroup"] = {f"{j:02d} {nm}": round(float((a[:, :, j + 1] - a[:, :, j]).mean()), 2)
                                                                      for j, nm in enumerate(names)}
                log(f"[bench] fused layer step m={m}: phase ends (us after the layer's start) {micro[str(m)]['fused_phase_end_us']}")
            log(f"[bench] layer step m={m}: {us:.2f} us (median of batches {us_med:.2f}), {gbs:.1f} GB/s ({gbs / HBM_PEAK_GBS:.1%} of peak)"
                + (f"; {micro[str(m)]['us_per_layer_in_stretches_of_8']:.2f} us per layer in stretches of 8" if L % 8 == 0 else ""))
            del H, Hw
        # what the machine gives kernels that only read a layer step's bytes: as one launch, and as one launch per phase
        probe = {}
        for nm, mode in (("one_kernel", binding.AD_PROBE_ONE_KERNEL), ("one_kernel_per_phase", binding.AD_PROBE_PER_PHASE)):
            def pr(i, mode=mode):
                g.ad_probe_stream(i % L + 1, ctx_micro, mode)
            for i in range(64):
                pr(i)
            torch.cuda.synchronize()
            pus, _ = timed_batches(pr, micro_calls)
            probe[nm + "_us"] = round(pus, 2)
            probe[nm + "_frac"] = round(layer_step_bytes(shape, ctx_micro, 0) / (pus * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        probe["note"] = ("kernels that read a layer's packed weights and its cached K/V rows and drop them (ad_probe_stream), rotating over "
                         "the layers like the calls above: the bytes alone, and the bytes with a kernel boundary between the five "
                         "phases that read memory; no arithmetic, no activations, no dependence through data")
        log(f"[bench] stream probe: {probe}")
        micro = {"ctx": ctx_micro, "calls_per_m": micro_calls, "distinct_weight_copies": L, "stream_probe": probe,
                 "rows": "N(0,1), drawn afresh for every call from a pre-generated device buffer (the first 10 calls of each m are the "
                         "rows of the parity test)",
                 "algorithmic_bytes_m1": layer_step_bytes(shape, ctx_micro, 1), "by_m": micro}
        roofline["layer_step_frac_by_m"] = {k: v["frac"] for k, v in micro["by_m"].items()}

    cpu = None
    if not args.skip_cpu:
        from oracle import oracle as orc
        cores = orc.num_threads()

        def at_threads(n, fn):
            orc.set_num_threads(n)
            t0 = time.perf_counter()
            r = fn()
            dt_ = time.perf_counter() - t0
            orc.set_num_threads(cores)
            return dt_, r

        # (a) Algorithm 1 on the benchmark's own model and weights: about 10 s of oracle time on the 8B shape
        n_prompt, n_new = 17, 64
        o = orc.Oracle(shape, w, max_pos=n_prompt + n_new + 8)
        cdt, (ot, ost, _) = at_threads(cores, lambda: o.generate_ada(prompt[:n_prompt], n_new, shape.gamma, cap))
        cpu = {"value": round(n_new / cdt, 4), "unit": "tokens/s", "cores": cores, "kind": "oracle",
               "sample": f"Algorithm 1 on the same model and weights, prompt {n_prompt} tokens, {n_new} generated tokens, "
                         f"gamma {shape.gamma}; {cdt:.1f}s wall, prefill included",
               "layer_steps_per_s": round((ost["layer_steps"] + (n_prompt - 1)) / cdt, 3)}
        n_one = 2
        cdt1, _ = at_threads(1, lambda: o.generate_ada(prompt[:2], n_one, shape.gamma, cap))
        cpu["one_thread"] = {"value": round(n_one / cdt1, 4), "unit": "tokens/s",
                             "sample": f"prompt of 2 tokens, {n_one} generated tokens; {cdt1:.1f}s wall, prefill included"}
        o.close()
        # (b) the tiny fp32 workload in full (prompt 32, 64 generated tokens, threshold 0.9)
        ts = synth.TINY
        tw = synth.make_weights(ts, seed=0)
        tp = synth.make_prompt(ts, 0)
        ot_ = orc.Oracle(ts, tw, max_pos=ts.prompt_len + ts.gen_len + 8)
        tall, (_, tst, _) = at_threads(cores, lambda: ot_.generate_ada(tp, ts.gen_len, ts.gamma, cap))
        tone, _ = at_threads(1, lambda: ot_.generate_ada(tp, ts.gen_len, ts.gamma, cap))
        ot_.close()
        cpu["tiny_workload"] = {"sample": f"tiny fp32 model, prompt {ts.prompt_len}, {ts.gen_len} generated tokens, in full",
                                "tokens_per_s": round(ts.gen_len / tall, 1), "tokens_per_s_one_thread": round(ts.gen_len / tone, 1),
                                "layer_steps_per_s": round(tst["layer_steps"] / tall, 1)}
        # (c) the layer-step microbenchmark: ten calls per m on one layer of the benchmark's shape at context 4096
        if shape.d_model == synth.LLAMA8B.d_model and shape.dtype == synth.BF16 and not args.skip_micro:
            ls = synth.LLAMA8B_LAYER
            lw = {k: v for k, v in w.items() if k.startswith("layers.0.") or k in ("final_norm",)}
            lw["embed"] = w["embed"][:ls.vocab]
            lw["lm_head"] = w["lm_head"][:ls.vocab]
            ol = orc.Oracle(ls, lw, max_pos=ctx_micro + 8)
            kk, vv = synth.make_kv_prefill(ls, 0, 0, ctx_micro)
            ol.kv_write(1, 0, kk.reshape(ctx_micro, -1), vv.reshape(ctx_micro, -1))
            by_m = {}

            def ten(m):
                for c in range(10):
                    ol.kv_set_len(1, ctx_micro)
                    ol.layer_step(1, synth.make_hidden(ls, synth.micro_call_seed(m, c), m), np.arange(ctx_micro, ctx_micro + m))

            for m in synth.MICRO_M:
                d_all, _ = at_threads(cores, lambda: ten(m))
                by_m[str(m)] = {"ms_per_call": round(d_all * 100, 2),
                                "GBps": round(layer_step_bytes(ls, ctx_micro, m) / (d_all / 10) / 1e9, 2)}
            for m in (1, 8):
                d_one, _ = at_threads(1, lambda: ten(m))
                by_m[str(m)]["ms_per_call_one_thread"] = round(d_one * 100, 2)
            ol.close()
            cpu["layer_step"] = {"sample": "ten oracle layer steps per m on one layer of the 8B shape, cache of 4096 positions, the "
                                           "rows of the microbenchmark's first ten calls; one thread for m = 1 and 8 only",
                                 "by_m": by_m}
        log(f"[bench] cpu oracle: {cpu}")

    out = {"metric": "decoded tokens/sec @batch1 (8B-shape bf16); layer-step HBM GB/s vs peak",
           "value": round(tokens_per_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(dt / args.steps * 1e3, 2), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": {synth.F32: "f32", synth.BF16: "bf16", synth.F16: "f16"}[shape.dtype], "data": "synthetic",
           "config": {"workload": f"{shape.name}: {shape.n_layers} layers d={shape.d_model} heads {shape.n_q_heads}/{shape.n_kv_heads}x{shape.head_dim} "
                                  f"ffn {shape.d_ffn} vocab {shape.vocab}, exit heads at {list(shape.exit_layers)}, gamma {shape.gamma}, "
                                  f"cap {cap}, prompt {prompt_len}, generate {gen_len}, batch 1, random-init N(0,0.02)"
                                  + (", exits forced from a seeded 0.2/0.2/0.2 schedule, verification on" if main_is_long else ""),
                      "global_batch": 1, "seq_len": prompt_len + gen_len},
           "roofline": roofline, "end_to_end": e2e, "forced": forced, "long": long, "decision": decision, "layer_step": micro,
           "cpu_baseline": cpu}
    if sweep is not None:
        out["gamma_sweep"] = sweep
    print(json.dumps(out), flush=True)
    g.close()


if __name__ == "__main__":
    main()
