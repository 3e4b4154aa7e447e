#!/usr/bin/env python3
"""Benchmark of the HTTM global-attention layer on one MI355X.

A "step" is one httm_layer_forward call (reorder + match/merge + attention + unmerge + inverse
reorder) on one batch of seeded synthetic VGGT-shaped Q/K/V that already sits in HBM.
Prints ONE JSON line on stdout; progress goes to stderr.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--no-extras] [--no-cpu]
                  [--no-other-configs]

metric  : global-attention-layer tokens/s = N / t_layer on the headline workload (--config, default 5):
          K steps bracketed by device synchronisation, wall clock.
configs : the same measurement for every workload 1-5 (the headline one included): per-step times
          from events on the launch stream (median and min over the K steps), per-stage times
          (median and min), achieved GB/s of the HBM-bound kernels and TFLOP/s of the attention,
          each as a fraction of the chip's peak.
roofline: for the dominant kernel of the headline workload (the MFMA attention): algorithmic flop
          4*H*M_q*M_k*64 per launch over its launch time, measured with events on the launch stream.
extras  : the same inputs without merging (r = 0), with the head-uniform variant, with first-frame
          anchoring, with the outlier filter and in the paper's own block configuration.
clock   : the shader clock the driver (or rocm-smi) reports before, between and after the timed regions (unpinned).
cpu_baseline: the CPU oracle timed on a bounded sample (a few heads) of the headline workload.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def event_times_ms(fn, iters, warmup=1):
    """Milliseconds of every one of `iters` calls of fn(), from events on the current stream (the
    stream the binding launches on)."""
    import torch
    for _ in range(warmup):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(iters):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    return [ev[i].elapsed_time(ev[i + 1]) for i in range(iters)]


def summary(ts):
    return {"ms": statistics.median(ts), "ms_min": min(ts), "ms_mean": sum(ts) / len(ts), "n": len(ts)}


def gpu_time_ms(fn, iters, warmup=1):
    """Median milliseconds per call of fn()."""
    return statistics.median(event_times_ms(fn, iters, warmup))


def shader_clock_mhz():
    """Current shader clock of GPU 0 in MHz (None if it cannot be read): the starred level of the
    driver's pp_dpm_sclk file, else what rocm-smi reports.  Under a profiler that is preloaded into
    every child process no other program is started, so there only the file is tried."""
    import glob
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        try:
            for line in open(path):
                m = re.match(r"\s*\d+:\s*(\d+)\s*Mhz\s*\*", line, re.IGNORECASE)
                if m:
                    return int(m.group(1))
        except OSError:
            pass
    if "rocprof" in os.environ.get("LD_PRELOAD", "") or any(k.startswith("ROCPROF") for k in os.environ):
        return None
    try:
        r = subprocess.run(["rocm-smi", "-d", "0", "--showclocks"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL,
                           text=True, timeout=20)
        m = re.search(r"sclk clock level:?\s*\d*:?\s*\(?(\d+)\s*Mhz", r.stdout, re.IGNORECASE)
        return int(m.group(1)) if m else None
    except Exception:
        return None


def mfma_sustained_tflops():
    """What the chip sustains on the attention kernel's MFMA instruction alone: a register-only loop of
    v_mfma_f32_32x32x16_bf16 with pseudo-random operands (paper_2511_21317_amd/csrc/mfma_probe.hip, its
    own small library), two workgroups of four waves per compute unit, about 25 ms per launch so that
    the clock has settled under the power limit.  Median of 5 launches; None if the probe is not built."""
    import ctypes
    import torch
    path = os.path.join(ROOT, "paper_2511_21317_amd", "libhttm_probe.so")
    if not os.path.exists(path):
        return None
    lib = ctypes.CDLL(path)
    lib.httm_probe_mfma_bf16.restype = ctypes.c_double
    lib.httm_probe_mfma_bf16.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    out = torch.zeros(1, dtype=torch.float32, device="cuda")
    flop = [0.0]

    def run():
        flop[0] = lib.httm_probe_mfma_bf16(out.data_ptr(), 40000, 2, torch.cuda.current_stream().cuda_stream)
    ts = event_times_ms(run, 5, warmup=2)
    if flop[0] <= 0.0:
        return None
    ms = statistics.median(ts)
    return {"TFLOP/s": flop[0] / (ms * 1e-3) / 1e12, "ms": ms, "flop": flop[0],
            "what": "register-only loop of v_mfma_f32_32x32x16_bf16, pseudo-random operands, 512 workgroups of 4 waves"}


def pmc_traffic_bytes(kernel: str, workload_index: int):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE + WRITE_SIZE, already scaled by the copy-kernel calibration), and the file, or None."""
    import glob
    for path in glob.glob(os.path.join(ROOT, "profiles", f"hbm_traffic_pmc_cfg{workload_index}_S*_N*.txt")):
        for line in open(path):
            if line.startswith(kernel) and "|" in line:
                cols = [c.split() for c in line.split("|")]
                return (float(cols[1][0]) + float(cols[1][1])) * 1e6, os.path.relpath(path, ROOT)
    return None, None


def cpu_oracle_baseline(w, q, k, v, budget_s=20.0):
    """Time the oracle (as it stands) on the first heads of the workload until ~budget_s is used."""
    from oracle import httm_oracle as orc
    from synth.vggt_tokens import bf16_to_f32_numpy
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    g = orc.Geometry(w.S, w.Hp, w.Wp, w.b, w.T, n_special=w.n_special)
    done, t0 = 0, time.perf_counter()
    while done < w.H:
        qh, kh, vh = (bf16_to_f32_numpy(t[done:done + 1]) for t in (q, k, v))
        orc.layer_forward(qh, kh, vh, g, w.rho, w.rho)
        done += 1
        el = time.perf_counter() - t0
        if el > budget_s or el / done * (done + 1) > 1.5 * budget_s:
            break
    el = time.perf_counter() - t0
    tokens_per_s = w.N / (el / done * w.H)
    return {"value": tokens_per_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{done} of {w.H} heads of {w.name}, full merged path per head "
                      f"({el:.1f} s measured, scaled to {w.H} heads)"}


def measure_workload(httm, w, q, k, v, plan, steps, warmup, stage_iters, wall_clock):
    """Layer and stage timings of one plan on resident inputs.  Returns (record, ms_per_step_wall)."""
    import torch
    H, N, Mq, Mk = plan.H, plan.N, plan.M_q, plan.M_k
    LK = plan.log2_keys
    out = torch.empty((N, H * 64), dtype=torch.bfloat16, device="cuda")
    ws = httm.alloc_workspace(plan)
    views = httm.workspace_views(plan, ws)
    step = lambda: httm.layer_forward(plan, q, k, v, out, ws)   # noqa: E731
    ms_wall = None
    if wall_clock:
        # the timed region of the headline number: K steps between two device synchronisations
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms_wall = (time.perf_counter() - t0) * 1e3 / steps
    layer = summary(event_times_ms(step, steps, warmup=0 if wall_clock else warmup))

    it = stage_iters
    row = 128
    q_off = [h * Mq for h in range(H + 1)]
    k_off = [h * Mk for h in range(H + 1)]
    qr = torch.empty_like(q)
    t_reorder = summary(event_times_ms(lambda: httm.reorder(plan, q, qr, 0), it))
    t_fused = summary(event_times_ms(lambda: httm.reorder_match_merge(
        plan, q, k, v, views["q_m"], views["k_m"], views["v_m"], views["assign_q"], views["assign_k"]), it))
    kr, vr = torch.empty_like(k), torch.empty_like(v)
    httm.reorder(plan, k, kr, 0)
    httm.reorder(plan, v, vr, 0)
    t_merge = summary(event_times_ms(lambda: httm.match_merge(
        plan, qr, kr, vr, views["q_m"], views["k_m"], views["v_m"], views["assign_q"], views["assign_k"]), it))
    del kr, vr, qr
    if LK:   # with the workspace's scratch region, as httm_layer_forward runs it
        attn = lambda: httm.attention_log2(views["q_m"], views["k_m"], views["v_m"], views["o_m"],   # noqa: E731
                                           q_off, k_off, scratch=views["attn_split"])
    else:
        attn = lambda: httm.attention(views["q_m"], views["k_m"], views["v_m"], views["o_m"],         # noqa: E731
                                      q_off, k_off, 0.125, scratch=views["attn_split"])
    t_attn = summary(event_times_ms(attn, it))
    t_unmerge = summary(event_times_ms(lambda: httm.unmerge(plan, views["o_m"], views["assign_q"], out, True), it))

    b_reorder = 2 * H * N * row                                   # one tensor, read + write
    b_merge = 3 * H * N * row + H * (Mq + 2 * Mk) * row + 2 * H * N * 4
    b_unmerge = N * H * row + H * Mq * row + H * N * 4
    f_attn = 4.0 * H * Mq * Mk * 64

    def hbm(t, nbytes):
        gbs = nbytes / (t["ms"] * 1e-3) / 1e9
        return {**t, "GB/s": gbs, "frac_hbm": gbs / PEAK_HBM_GBS, "algorithmic_bytes": nbytes}

    tf = f_attn / (t_attn["ms"] * 1e-3) / 1e12
    stages = {
        "reorder_one_tensor": hbm(t_reorder, b_reorder),
        "match_merge_on_reordered": hbm(t_merge, b_merge),
        "reorder_match_merge_fused": hbm(t_fused, b_merge),
        "attention": {**t_attn, "TFLOP/s": tf, "frac_mfma": tf / PEAK_BF16_TFLOPS, "algorithmic_flop": f_attn},
        "unmerge_inverse_reorder_fused": hbm(t_unmerge, b_unmerge),
    }
    rec = {"workload": w.name, "N": N, "M_q": Mq, "M_k": Mk, "log2_keys": LK,
           "layer": {**layer, "tokens/s": N / (layer["ms"] * 1e-3)}, "stages": stages}
    log(f"[bench] {w.name}: layer {layer['ms']:.4f} ms (min {layer['ms_min']:.4f}) -> {rec['layer']['tokens/s']:.4g} tokens/s; "
        f"fused match/merge {t_fused['ms']:.4f} ms ({stages['reorder_match_merge_fused']['frac_hbm']:.3f} of HBM), "
        f"attention {t_attn['ms']:.4f} ms ({stages['attention']['frac_mfma']:.3f} of bf16 MFMA), "
        f"unmerge {t_unmerge['ms']:.4f} ms ({stages['unmerge_inverse_reorder_fused']['frac_hbm']:.3f}), "
        f"reorder {t_reorder['ms']:.4f} ms ({stages['reorder_one_tensor']['frac_hbm']:.3f})")
    del ws, views, out
    torch.cuda.empty_cache()
    return rec, ms_wall


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-extras", action="store_true", help="skip the r=0, head-uniform, anchored, filtered and paper-block runs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-other-configs", action="store_true", help="measure the headline workload only")
    ap.add_argument("--stage-iters", type=int, default=20)
    ap.add_argument("--paper-blocks", action="store_true",
                    help="time the layer with the paper's own block geometry and ratios (Sec. 4.1: runs of "
                         "128 tokens x 30 frames, 90 %% of the queries and 70 %% of the keys / values merged) "
                         "on the workload's tokens instead of the benchmark's configuration")
    ap.add_argument("--outlier-frac", type=float, default=0.0,
                    help="time the layer WITH the adaptive outlier filtering of the queries (Sec. 3.4) at "
                         "this share of all query tokens; 0 (default) is the benchmark's configuration")
    ap.add_argument("--plain-keys", action="store_true",
                    help="merged keys without the logit scale and the general stage-3 kernel (the default is "
                         "HTTM_FLAG_LOG2_KEYS: stage 2 folds log2(e)/sqrt(d) into the merged keys, stage 3 skips "
                         "the multiplication per score)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build targets ONE GPU (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_21317_amd as httm
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    httm.lib()   # fails loudly if libhttm.so is missing
    clocks = {"tool": "pp_dpm_sclk of the driver, else rocm-smi -d 0 --showclocks (sclk, MHz; clocks are not pinned)", "before": shader_clock_mhz()}
    LK = not args.plain_keys
    special = args.paper_blocks or args.outlier_frac > 0.0

    def mk_geom(*a, **kw):
        return httm.make_geom(*a, log2_keys=LK, **kw)

    w = synth.workload(args.config)
    log(f"[bench] workload {w.name}: N={w.N} H={w.H} block {w.b}x{w.b}x{w.T} rho={w.rho}")
    q, k, v = synth.make_qkv(w, device="cuda")
    torch.cuda.synchronize()

    if special:
        headline, ms_per_step, plan_desc = measure_special(httm, args, w, q, k, v, mk_geom)
    else:
        plan = httm.Plan(mk_geom(w.S, w.Hp, w.Wp, w.b, w.T, w.rho, H=w.H, n_special=w.n_special))
        headline, ms_per_step = measure_workload(httm, w, q, k, v, plan, args.steps, args.warmup, args.stage_iters, True)
        plan_desc = {"M_q": plan.M_q, "M_k": plan.M_k}
        plan.close()
    H, N = w.H, w.N
    tokens_per_s = N / (ms_per_step * 1e-3)
    log(f"[bench] layer: {ms_per_step:.3f} ms/step -> {tokens_per_s:.4g} tokens/s")
    clocks["after_headline"] = shader_clock_mhz()

    a = headline["stages"]["attention"]
    traffic, traffic_file = pmc_traffic_bytes("attention_kernel<2, 4, false>" if LK else "attention_kernel<2, 4, true>", w.index)
    roofline = {"kernel": "attention_kernel", "bound": "mfma", "achieved": a["TFLOP/s"],
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": a["TFLOP/s"] / PEAK_BF16_TFLOPS,
                "traffic": None if special else traffic,
                "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated; not measured in this "
                                "run but read from the committed summary named in traffic_source)",
                "traffic_source": None if special else traffic_file,
                "flop_per_launch": a["algorithmic_flop"], "ms_per_launch": a["ms"], "ms_per_launch_min": a["ms_min"]}
    # context for that fraction (the peak above stays the published one): the rate the same MFMA
    # instruction reaches alone on this chip, under its power limit
    if not args.no_extras:
        sus = mfma_sustained_tflops()
        if sus:
            roofline["mfma_sustained_on_this_chip"] = sus
            roofline["frac_of_sustained"] = a["TFLOP/s"] / sus["TFLOP/s"]
            log(f"[bench] MFMA instruction alone: {sus['TFLOP/s']:.0f} TFLOP/s sustained ({sus['TFLOP/s'] / PEAK_BF16_TFLOPS:.3f} "
                f"of the published peak); attention = {roofline['frac_of_sustained']:.3f} of that")

    # ---- extras: variants on the headline workload's inputs -------------------------------------
    extras = {}
    if not args.no_extras and not special:
        extras = measure_extras(httm, w, q, k, v, mk_geom, max(4, args.stage_iters // 2), ms_per_step,
                                headline["stages"]["reorder_match_merge_fused"]["ms"])
    clocks["after_extras"] = shader_clock_mhz()

    cpu = None
    if not args.no_cpu and not special:   # the CPU leg times the benchmark's own configuration
        log("[bench] timing the CPU oracle on a bounded sample ...")
        cpu = cpu_oracle_baseline(w, q.cpu(), k.cpu(), v.cpu())
        log(f"[bench] cpu oracle: {cpu['value']:.4g} tokens/s on {cpu['cores']} threads ({cpu['sample']})")
    del q, k, v
    torch.cuda.empty_cache()

    # ---- every workload, same protocol (events on the launch stream; median and min) -----------------
    configs = []
    if not special:
        for idx in (1, 2, 3, 4, 5):
            if idx == args.config:
                configs.append(headline)
                continue
            if args.no_other_configs:
                continue
            wi = synth.workload(idx)
            qi, ki, vi = synth.make_qkv(wi, device="cuda")
            torch.cuda.synchronize()
            plan_i = httm.Plan(mk_geom(wi.S, wi.Hp, wi.Wp, wi.b, wi.T, wi.rho, H=wi.H, n_special=wi.n_special))
            rec, _ = measure_workload(httm, wi, qi, ki, vi, plan_i, args.steps, args.warmup, args.stage_iters, False)
            plan_i.close()
            configs.append(rec)
            del qi, ki, vi
            torch.cuda.empty_cache()
    clocks["after_all_configs"] = shader_clock_mhz()
    log(f"[bench] shader clock (MHz): {clocks}")

    result = {
        "metric": "global-attn layer tokens/s (merge+attn+unmerge)",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_median_events": headline["layer"]["ms"],
        "ms_per_step_min_events": headline["layer"]["ms_min"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "S": w.S, "grid": [w.Hp, w.Wp], "N": N, "H": H, "d_head": 64,
                   "block": [w.b, w.b, w.T], "rho": w.rho, **plan_desc,
                   "outlier_frac": args.outlier_frac, "log2_keys": LK,
                   "paper_blocks_ns128_nt30_rq0.9_rkv0.7": bool(args.paper_blocks)},
        "roofline": roofline,
        "stages": headline["stages"],
        "configs": configs,
        "extras": extras,
        "clock_mhz": clocks,
        "cpu_baseline": cpu,
        # context only (another machine, another scope: never the target and never in vs_baseline)
        "paper_context": {
            "hardware": "one Nvidia A100, bf16, third-party FlashAttention kernel, whole VGGT* model on real datasets",
            "end_to_end_speedup_over_unmerged_vggt_1000_frames": "7x (724.6 s -> 102.8 s, Table 2)",
            "merging_cost_vs_fastvggt_global_attention_layers": "4.58x lower (matching + aggregation 0.53 s vs 2.42 s, Table 3)",
            "layer_tokens_per_s": None,
        },
    }
    print(json.dumps(result), flush=True)


def measure_special(httm, args, w, q, k, v, mk_geom):
    """--paper-blocks / --outlier-frac: the layer in that configuration (no per-stage HBM fractions:
    the stage-2 entry point with the filter has other traffic)."""
    import torch
    filtered = args.outlier_frac > 0.0
    if args.paper_blocks:
        plan = httm.Plan(mk_geom(w.S, w.Hp, w.Wp, 128, 30, 0.9, 0.7, H=w.H, n_special=w.n_special,
                                 chunked_blocks=True, outlier_frac=args.outlier_frac))
    else:
        plan = httm.Plan(mk_geom(w.S, w.Hp, w.Wp, w.b, w.T, w.rho, H=w.H, n_special=w.n_special,
                                 outlier_frac=args.outlier_frac))
    H, N, Mq, Mk = plan.H, plan.N, plan.M_q, plan.M_k
    out = torch.empty((N, H * 64), dtype=torch.bfloat16, device="cuda")
    ws = httm.alloc_workspace(plan)
    views = httm.workspace_views(plan, ws)
    step = lambda: httm.layer_forward(plan, q, k, v, out, ws)   # noqa: E731
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_wall = (time.perf_counter() - t0) * 1e3 / args.steps
    layer = summary(event_times_ms(step, args.steps, warmup=0))
    it = args.stage_iters
    q_off = [h * Mq for h in range(H + 1)]
    k_off = [h * Mk for h in range(H + 1)]
    if filtered:
        t_s2 = summary(event_times_ms(lambda: httm.reorder_match_merge_filtered(
            plan, q, k, v, views["q_m"], views["k_m"], views["v_m"], views["assign_q"], views["assign_k"],
            views["eps_q"], views["q_out"]), it))
    else:
        t_s2 = summary(event_times_ms(lambda: httm.reorder_match_merge(
            plan, q, k, v, views["q_m"], views["k_m"], views["v_m"], views["assign_q"], views["assign_k"]), it))
    if plan.log2_keys:
        attn = lambda: httm.attention_log2(views["q_m"], views["k_m"], views["v_m"], views["o_m"],   # noqa: E731
                                           q_off, k_off, scratch=views["attn_split"])
    else:
        attn = lambda: httm.attention(views["q_m"], views["k_m"], views["v_m"], views["o_m"],         # noqa: E731
                                      q_off, k_off, 0.125, scratch=views["attn_split"])
    t_attn = summary(event_times_ms(attn, it))
    f_attn = 4.0 * H * Mq * Mk * 64
    tf = f_attn / (t_attn["ms"] * 1e-3) / 1e12
    stages = {"stage2": {**t_s2, "with_outlier_filter": filtered},
              "attention": {**t_attn, "TFLOP/s": tf, "frac_mfma": tf / PEAK_BF16_TFLOPS, "algorithmic_flop": f_attn}}
    if filtered:
        t_a2 = summary(event_times_ms(lambda: httm.attention_outliers(plan, views["q_out"], views["k_m"],
                                                                       views["v_m"], views["o_out"]), it))
        t_un = summary(event_times_ms(lambda: httm.unmerge_filtered(plan, views["o_m"], views["o_out"],
                                                                     views["assign_q"], out), it))
        tau, counts = httm.outlier_stats(plan)
        f2 = 4.0 * sum(counts) * Mk * 64
        stages["outlier_attention"] = {**t_a2, "TFLOP/s": f2 / (t_a2["ms"] * 1e-3) / 1e12, "outliers": sum(counts), "tau": tau}
        stages["unmerge_inverse_reorder_fused"] = {**t_un, "with_outlier_rows": True}
    else:
        stages["unmerge_inverse_reorder_fused"] = summary(event_times_ms(
            lambda: httm.unmerge(plan, views["o_m"], views["assign_q"], out, True), it))
    for name, s in stages.items():
        log(f"[bench] {name}: " + ", ".join(f"{k_}={v_:.4g}" if isinstance(v_, float) else f"{k_}={v_}" for k_, v_ in s.items()))
    rec = {"workload": w.name, "N": N, "M_q": Mq, "M_k": Mk, "log2_keys": plan.log2_keys,
           "layer": {**layer, "tokens/s": N / (layer["ms"] * 1e-3)}, "stages": stages}
    desc = {"M_q": Mq, "M_k": Mk}
    plan.close()
    return rec, ms_wall, desc


def measure_extras(httm, w, q, k, v, mk_geom, it, ms_per_step, t_fused_merge):
    import torch
    H, N = w.H, w.N
    extras = {}
    out_u = torch.empty((N, H * 64), dtype=torch.bfloat16, device="cuda")
    plan_u = httm.Plan(mk_geom(w.S, w.Hp, w.Wp, w.b, w.T, w.rho, H=w.H, n_special=w.n_special, variant="uniform"))
    ws_u = httm.alloc_workspace(plan_u)
    t_uni = gpu_time_ms(lambda: httm.layer_forward(plan_u, q, k, v, out_u, ws_u), it)
    extras["head_uniform_layer"] = {"ms": t_uni, "tokens/s": N / (t_uni * 1e-3)}
    log(f"[bench] head-uniform layer: {t_uni:.3f} ms")
    plan_u.close()
    del ws_u
    torch.cuda.empty_cache()
    plan_a = httm.Plan(mk_geom(w.S, w.Hp, w.Wp, w.b, w.T, w.rho, H=w.H, n_special=w.n_special, anchor_first_frame=True))
    ws_a = httm.alloc_workspace(plan_a)
    t_anc = gpu_time_ms(lambda: httm.layer_forward(plan_a, q, k, v, out_u, ws_a), it)
    extras["first_frame_anchored_layer"] = {"ms": t_anc, "tokens/s": N / (t_anc * 1e-3), "M_q": plan_a.M_q}
    log(f"[bench] first-frame-anchored layer: {t_anc:.3f} ms (M = {plan_a.M_q})")
    plan_a.close()
    del ws_a
    torch.cuda.empty_cache()
    # adaptive outlier filtering of the queries at the paper's setting (Sec. 4.1: 10 % of all
    # query tokens are taken out of the merging again and attend on their own)
    plan_f = httm.Plan(mk_geom(w.S, w.Hp, w.Wp, w.b, w.T, w.rho, H=w.H, n_special=w.n_special, outlier_frac=0.1))
    ws_f = httm.alloc_workspace(plan_f)
    t_fil = gpu_time_ms(lambda: httm.layer_forward(plan_f, q, k, v, out_u, ws_f), it)
    vf = httm.workspace_views(plan_f, ws_f)
    t_s2 = gpu_time_ms(lambda: httm.reorder_match_merge_filtered(
        plan_f, q, k, v, vf["q_m"], vf["k_m"], vf["v_m"], vf["assign_q"], vf["assign_k"], vf["eps_q"], vf["q_out"]), it)
    t_a2 = gpu_time_ms(lambda: httm.attention_outliers(plan_f, vf["q_out"], vf["k_m"], vf["v_m"], vf["o_out"]), it)
    tau, counts = httm.outlier_stats(plan_f)
    f_a2 = 4.0 * sum(counts) * plan_f.M_k * 64
    extras["outlier_filtered_layer_d0.1"] = {
        "ms": t_fil, "tokens/s": N / (t_fil * 1e-3), "outliers": sum(counts),
        "outliers_per_head_min_max": [min(counts), max(counts)], "tau": tau,
        "stage2_with_filter_ms": t_s2, "outlier_attention_ms": t_a2,
        "outlier_attention_TFLOP/s": f_a2 / (t_a2 * 1e-3) / 1e12}
    log(f"[bench] outlier-filtered layer (d = 0.1): {t_fil:.3f} ms; stage 2 {t_s2:.3f} ms, "
        f"second attention {t_a2:.3f} ms ({sum(counts)} outlier queries)")
    plan_f.close()
    del ws_f, vf
    torch.cuda.empty_cache()
    # the paper's own configuration on the same tokens (Sec. 4.1): runs of 128 tokens x 30 frames =
    # blocks of 3840, 90 % of the queries and 70 % of the keys / values merged, 10 % of all query
    # tokens filtered out again as outliers
    for frac_p, tag in ((0.0, "paper_blocks_ns128_nt30_rq0.9_rkv0.7_layer"),
                        (0.1, "paper_configuration_ns128_nt30_rq0.9_rkv0.7_d0.1_layer")):
        plan_p = httm.Plan(mk_geom(w.S, w.Hp, w.Wp, 128, 30, 0.9, 0.7, H=w.H, n_special=w.n_special,
                                   chunked_blocks=True, outlier_frac=frac_p))
        ws_p = httm.alloc_workspace(plan_p)
        vp = httm.workspace_views(plan_p, ws_p)
        t_pap = gpu_time_ms(lambda: httm.layer_forward(plan_p, q, k, v, out_u, ws_p), it)
        if frac_p:
            t_pmm = gpu_time_ms(lambda: httm.reorder_match_merge_filtered(
                plan_p, q, k, v, vp["q_m"], vp["k_m"], vp["v_m"], vp["assign_q"], vp["assign_k"],
                vp["eps_q"], vp["q_out"]), it)
            n_out = sum(httm.outlier_stats(plan_p)[1])
        else:
            t_pmm = gpu_time_ms(lambda: httm.reorder_match_merge(
                plan_p, q, k, v, vp["q_m"], vp["k_m"], vp["v_m"], vp["assign_q"], vp["assign_k"]), it)
            n_out = 0
        f_p = 4.0 * (H * plan_p.M_q + n_out) * plan_p.M_k * 64
        b_p = 3 * H * N * 128 + H * (plan_p.M_q + 2 * plan_p.M_k) * 128 + 2 * H * N * 4
        extras[tag] = {"ms": t_pap, "tokens/s": N / (t_pap * 1e-3), "M_q": plan_p.M_q, "M_k": plan_p.M_k,
                       "outlier_queries": n_out, "stage2_ms": t_pmm, "attention_flop": f_p,
                       "stage2_frac_hbm_plain_traffic": b_p / (t_pmm * 1e-3) / 1e9 / PEAK_HBM_GBS}
        log(f"[bench] paper blocks (3840 tokens, 90 % / 70 %, d = {frac_p}): layer {t_pap:.3f} ms, stage 2 "
            f"{t_pmm:.3f} ms (M_q = {plan_p.M_q}, M_k = {plan_p.M_k}, {n_out} outlier queries)")
        plan_p.close()
        del ws_p, vp
        torch.cuda.empty_cache()
    # the cost the merging blocks remove (Sec. 3.3, Table 3 "Matching"): un-blocked matching of
    # the queries with 25 % dst tokens, against the block-local stage 2 (Q, K and V, with merging)
    best = torch.empty((H, N), dtype=torch.int32, device="cuda")
    t_glob = gpu_time_ms(lambda: httm.global_match(q, 0.25, best), 1, warmup=1)
    kd_g = int(0.25 * N)
    extras["global_matching_q_dst0.25"] = {
        "ms": t_glob, "TFLOP/s": 2.0 * H * N * kd_g * 64 / (t_glob * 1e-3) / 1e12,
        "x_block_local_stage2": t_glob / t_fused_merge}
    log(f"[bench] un-blocked matching of Q (25 % dst): {t_glob:.2f} ms = {t_glob / t_fused_merge:.0f}x the "
        f"block-local matching + merging of Q, K and V")
    del best
    plan_0 = httm.Plan(mk_geom(w.S, w.Hp, w.Wp, w.b, w.T, 0.0, H=w.H, n_special=w.n_special, variant="none"))
    ws_0 = httm.alloc_workspace(plan_0)
    big = N > 100000
    t_un = gpu_time_ms(lambda: httm.layer_forward(plan_0, q, k, v, out_u, ws_0), 1 if big else it, warmup=0 if big else 1)
    f_un = 4.0 * H * N * N * 64
    extras["unmerged_layer_r0"] = {"ms": t_un, "tokens/s": N / (t_un * 1e-3),
                                   "attention_TFLOP/s_lower_bound": f_un / (t_un * 1e-3) / 1e12,
                                   "speedup_of_merging": t_un / ms_per_step}
    log(f"[bench] unmerged (r=0) layer: {t_un:.2f} ms  ({t_un / ms_per_step:.1f}x the merged layer)")
    plan_0.close()
    del ws_0, out_u
    torch.cuda.empty_cache()
    return extras


if __name__ == "__main__":
    main()
