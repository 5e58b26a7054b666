#!/usr/bin/env python3
"""Throughput of the OIM + SPU hot path on one MI355X.

A step = luvc_oim_merge (every call of the workload's schedule) + luvc_spu_score + luvc_spu_prune
over one batch of seeded synthetic input that is already resident in HBM.  Prints ONE JSON line:
tokens/s (visual tokens entering OIM per second) of the four target workloads (`configs`, headline =
the largest), the roofline of the headline's dominant kernel measured with HIP events on the launch
stream, and the CPU oracle timed on the same chain on this host's cores (all cores and one thread),
which also checks the GPU's chained OIM -> projection -> SPU run.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=None,
                    help="time one workload 0..4 of BASELINE.json only (default: 1..4, headline on the largest, cfg2)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg (timing and the check of the chained run)")
    ap.add_argument("--no-pipelined", dest="pipelined", action="store_false", help="skip the two-stream leg")
    ap.add_argument("--oim-wide", action="store_true",
                    help="also time luvc_oim_merge_wide on the workload's grid in the paper's setting (whole-line matching, merge number 2, three operations)")
    ap.add_argument("--next-rows", action="store_true",
                    help="also time the calls beyond the hot path: keyed merge, value enhancement, a cascade, ragged batches")
    ap.add_argument("--rotate-mb", type=float, default=600.0, help="distinct input bytes cycled through (defeats cache reuse)")
    ap.add_argument("--preheat-ms", type=float, default=100.0, help="untimed steps run for this long before the warm-up steps, to bring the clocks up (0: none)")
    return ap.parse_args()


HEADLINE = 2            # the largest of the four target workloads (46 080 tokens per step)
TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic.json")


def run_config(cfg, args, lv, wl, torch, np):
    """Times the step of one workload.  Returns (json-ready result, context for the optional legs)."""
    dev = torch.device("cuda:0")
    w = wl.workload(cfg)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    es = 2 if w.dtype == "bf16" else 4
    code = lv.LUVC_BF16 if w.dtype == "bf16" else lv.LUVC_F32

    def upload(a):
        if w.dtype == "bf16":
            return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(a).to(dev)

    def download(t):
        if t.dtype == torch.bfloat16:
            return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()

    t0 = time.time()
    x_oim_host = wl.oim_input(w)
    x_oim0 = upload(x_oim_host)

    # ---- preallocate every output and workspace: nothing is allocated inside the timed region
    calls = []
    H, W = w.H, w.W
    ws_bytes = 256
    for passes in w.oim_calls:
        Ho, Wo = lv.out_grid(H, W, passes)
        out = dict(x=torch.empty((w.grids, Ho, Wo, w.D), dtype=tdt, device=dev),
                   sizes=torch.empty((w.grids, Ho, Wo), dtype=torch.int32, device=dev),
                   merged_map=torch.empty((w.grids, H * W), dtype=torch.int32, device=dev),
                   kept_map=torch.empty((w.grids, Ho * Wo), dtype=torch.int32, device=dev))
        ws_bytes = max(ws_bytes, lv.luvc_oim_workspace_bytes(w.grids, H, W, w.D, code, passes))
        calls.append((passes, out))
        H, W = Ho, Wo
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    # the SPU calls get a workspace of their own, so that they may run beside the OIM call of another step
    workspace_spu = torch.empty(max(256, lv.luvc_spu_workspace_bytes(w.spu_B, w.spu_N, w.spu_D, code, w.sigma)), dtype=torch.uint8, device=dev)
    scores = torch.empty((w.spu_B, w.spu_N), dtype=torch.float32, device=dev)
    pr_out = dict(kept_idx=torch.empty((w.spu_B, w.n_keep), dtype=torch.int32, device=dev),
                  x=torch.empty((w.spu_B, w.n_keep, w.spu_D), dtype=tdt, device=dev))
    stream = torch.cuda.current_stream()

    def oim(x, st):
        sizes = None
        for passes, out in calls:
            lv.luvc_oim_merge(x, passes, sizes=sizes, workspace=workspace, stream=st, out=out)
            x, sizes = out["x"], out["sizes"]

    # ---- the chain the configurations describe, once, untimed: OIM on the GPU, the merged tokens projected to the LLM
    # width on the host (input generation, workloads.spu_input_from_merged), SPU on the result.  The SPU calls of the
    # timed steps read this tensor.
    oim(x_oim0, stream)
    torch.cuda.synchronize()
    oim_out_host = [{k: download(v) for k, v in out.items()} for _, out in calls]
    merged_vals = wl.bf16_bits_to_f32(oim_out_host[-1]["x"]) if w.dtype == "bf16" else oim_out_host[-1]["x"]
    x_spu_host = wl.spu_input_from_merged(w, merged_vals)
    x_spu0 = upload(x_spu_host)
    lv.luvc_spu_score(x_spu0, w.sigma, True, workspace=workspace_spu, stream=stream, out=scores)
    lv.luvc_spu_prune(x_spu0, scores, w.n_keep, stream=stream, out=pr_out)
    torch.cuda.synchronize()
    chain_gpu = dict(oim=oim_out_host, scores=scores.cpu().numpy().copy(), kept_idx=pr_out["kept_idx"].cpu().numpy().copy(),
                     x_keep=download(pr_out["x"]).copy())

    set_bytes = x_oim0.numel() * es + x_spu0.numel() * es
    n_rot = max(2, int(np.ceil(args.rotate_mb * 1e6 / set_bytes)))
    xs_oim = [x_oim0] + [x_oim0.clone() for _ in range(n_rot - 1)]
    xs_spu = [x_spu0] + [x_spu0.clone() for _ in range(n_rot - 1)]
    gen_s = time.time() - t0

    def step(i, ev=None):
        if ev: ev[0].record(stream)
        oim(xs_oim[i % n_rot], stream)
        if ev: ev[1].record(stream)
        xs = xs_spu[i % n_rot]
        lv.luvc_spu_score(xs, w.sigma, True, workspace=workspace_spu, stream=stream, out=scores)
        if ev: ev[2].record(stream)
        lv.luvc_spu_prune(xs, scores, w.n_keep, stream=stream, out=pr_out)
        if ev: ev[3].record(stream)

    # Before the W warm-up steps the GPU is brought to its working clocks: a short run starts on a chip that has been
    # idle through input generation and ramps up over the first tens of milliseconds (cfg2, 20 timed steps: 126 us per
    # step after 5 warm-up steps alone, 120 us with this, 116 us in a long run).  Untimed, and reported as `preheat_steps`.
    preheat, t_heat = 0, time.perf_counter()
    while time.perf_counter() - t_heat < args.preheat_ms * 1e-3:
        for i in range(25):
            step(preheat + i)
        torch.cuda.synchronize()
        preheat += 25
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # the timed region holds the K steps and nothing else: no event records between the launches
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # per-call durations (oim, score, prune) from stream events, in a pass of their own
    n_seg = min(args.steps, 50)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n_seg)]
    for i in range(n_seg):
        step(i, events[i])
    torch.cuda.synchronize()

    seg = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in events])      # ms: oim, score, prune
    seg_mean = seg.mean(axis=0)
    ms_per_step = wall * 1e3 / args.steps
    tokens_per_s = w.tokens_in / (wall / args.steps)

    # ---- the same K steps once more as a two-stream pipeline: the OIM call of a step and its SPU calls work on
    # independent tensors (in a model, SPU sees an image long after OIM did), so a serving loop can run the
    # memory-bound merge beside the arithmetic-bound transform.  Reported beside `value`, never as `value`.
    pipelined = None
    if args.pipelined:
        s_oim, s_spu = torch.cuda.Stream(), torch.cuda.Stream()

        def step2(i):
            oim(xs_oim[i % n_rot], s_oim)
            xs = xs_spu[i % n_rot]
            lv.luvc_spu_score(xs, w.sigma, True, workspace=workspace_spu, stream=s_spu, out=scores)
            lv.luvc_spu_prune(xs, scores, w.n_keep, stream=s_spu, out=pr_out)

        for rep in range(2):                       # the first pass over new streams is a warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                step2(i)
            torch.cuda.synchronize()
            wall2 = time.perf_counter() - t0
        pipelined = {"ms_per_step": round(wall2 * 1e3 / args.steps, 5), "value": round(w.tokens_in / (wall2 / args.steps), 1),
                     "unit": "tokens/s", "streams": 2,
                     "what": "luvc_oim_merge on one stream, luvc_spu_score + luvc_spu_prune on another, same K steps"}

    # ---- second pass over the same steps with two HIP events around every kernel launch, recorded by the
    # library on the launch stream (luvc_profile_start): per-kernel durations for the roofline
    n_prof = min(args.steps, 50)
    launches_per_step = 16
    prof = lv.LaunchProfile(n_prof * launches_per_step)
    prof.start()
    for i in range(n_prof):
        step(i)
    prof.stop()
    torch.cuda.synchronize()
    per_kernel = {}
    for name, ms in prof.results():
        per_kernel.setdefault(name, []).append(ms)
    prof.close()

    # ---- algorithmic work per launch: every input element read once, every output element written once
    oim_bytes = 0
    H, W = w.H, w.W
    for passes, out in calls:
        Ho, Wo = lv.out_grid(H, W, passes)
        oim_bytes += w.grids * (H * W + Ho * Wo) * w.D * es
        H, W = Ho, Wo
    score_bytes = w.spu_B * w.spu_N * w.spu_D * es
    prune_bytes = 2 * w.spu_B * w.n_keep * w.spu_D * es
    alg = dict(oim=oim_bytes, spu_score=score_bytes, spu_prune=prune_bytes)
    # per kernel: (algorithmic bytes per step, flops per step or None, roofline that bounds it)
    L = 2 * w.sigma + 1
    fft_flops = None
    n1 = next((16 * q for q in (16, 15, 9) if w.spu_N % (16 * q) == 0 and L <= 16 * q), None)
    if n1 and w.spu_N <= 4096:
        n2 = w.spu_N // n1
        # per packed channel pair: N2 forward + N2 inverse N1-point transforms (5 P log2 P each), the
        # pass-band accumulation and expansion (8 flops per bin and subsequence, both ways), the energy.
        # This is the work of Eq. 4-8 as the transform decomposition states it; a kernel that reaches the same
        # scores with fewer operations is credited with these, not with its own count.
        fft_flops = w.spu_B * (w.spu_D / 2) * (2 * n2 * 5 * n1 * np.log2(n1) + 2 * 8 * n2 * L + 4 * w.spu_N)
    work = {
        "oim_halve_pair": (oim_bytes, None, "hbm"), "oim_halve": (oim_bytes, None, "hbm"),
        "spu_fft16q": (score_bytes, fft_flops, "alu"),
        "spu_fwd_dense": (score_bytes, None, "hbm"), "spu_dense_fused": (score_bytes, None, "hbm"),
        "spu_gather": (prune_bytes, None, "hbm"), "spu_prune_fused": (prune_bytes, None, "hbm"),
    }
    try:
        with open(os.path.join(ROOT, TRAFFIC_FILE)) as f:
            measured_traffic = json.load(f).get(w.name, {})
    except (OSError, ValueError):
        measured_traffic = {}
    kernels = []
    for name, v in per_kernel.items():
        per_step = len(v) / n_prof
        avg_ms = float(np.mean(v))
        k = {"kernel": name, "launches_per_step": round(per_step, 2), "avg_us": round(avg_ms * 1e3, 2),
             "us_per_step": round(avg_ms * 1e3 * per_step, 2)}
        if name in work:
            by, fl, bound = work[name]
            k["bound"] = bound
            k["algorithmic_bytes_per_launch"] = int(by / per_step)
            k["hbm_GBps"] = round(by / per_step / (avg_ms * 1e-3) / 1e9, 1)
            k["hbm_frac"] = round(k["hbm_GBps"] / HBM_PEAK_GBS, 4)
            if fl:
                k["algorithmic_flops_per_launch"] = int(fl / per_step)
                k["TFLOPs"] = round(fl / per_step / (avg_ms * 1e-3) / 1e12, 2)
        t = measured_traffic.get(name)
        if t:
            k["traffic_bytes_per_launch"] = int(t["read_bytes"] + t["write_bytes"])
        kernels.append(k)
    kernels.sort(key=lambda k: -k["us_per_step"])
    dom = kernels[0]
    if dom.get("bound") == "alu":
        # fp32 vector peak of MI355X: 256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2 flops x 2.4 GHz
        roofline = {"bound": "alu", "kernel": dom["kernel"], "achieved": dom["TFLOPs"], "peak": 157.3, "unit": "TFLOP/s",
                    "frac": round(dom["TFLOPs"] / 157.3, 4), "traffic": dom.get("traffic_bytes_per_launch"),
                    "avg_us": dom["avg_us"], "algorithmic_flops": dom["algorithmic_flops_per_launch"],
                    "hbm_view": {"achieved": dom["hbm_GBps"], "peak": HBM_PEAK_GBS, "frac": dom["hbm_frac"],
                                 "algorithmic_bytes": dom["algorithmic_bytes_per_launch"]}}
    else:
        roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom.get("hbm_GBps"), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": dom.get("hbm_frac"), "traffic": dom.get("traffic_bytes_per_launch"), "avg_us": dom["avg_us"],
                    "algorithmic_bytes": dom.get("algorithmic_bytes_per_launch")}
    # the traffic figures are NOT measured by this run: hardware counters need a profiler run of their own
    roofline["traffic_source"] = (f"{TRAFFIC_FILE} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this script, "
                                  "calibrated on copy kernels; see the summaries beside it)") if roofline.get("traffic") else None
    roofline["timing"] = f"start/stop HIP events attached by the library to every dispatch on the launch stream, {n_prof} steps after the timed region"
    roofline["kernels"] = kernels
    roofline["whole_step"] = {"algorithmic_bytes": sum(alg.values()),
                              "achieved": round(sum(alg.values()) / (ms_per_step * 1e-3) / 1e9, 1),
                              "frac": round(sum(alg.values()) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    roofline["calls_ms"] = {n: round(float(v), 5) for n, v in zip(["oim", "spu_score", "spu_prune"], seg_mean)}

    result = {
        "value": round(tokens_per_s, 1), "ms_per_step": round(ms_per_step, 5), "dtype": w.dtype,
        "config": {"workload": w.name, "tokens_per_step": w.tokens_in, "oim": f"{w.grids}x{w.H}x{w.W}x{w.D}",
                   "spu": f"{w.spu_B}x{w.spu_N}x{w.spu_D}", "n_keep": w.n_keep, "sigma": w.sigma,
                   "spu_input": "the GPU's own OIM output, projected on the host to the SPU width",
                   "rotating_input_sets": n_rot, "input_gen_s": round(gen_s, 1), "preheat_steps": preheat},
        "roofline": roofline,
        "pct_of_peak_hbm": round(100.0 * roofline["whole_step"]["frac"], 2),      # algorithmic bytes of the whole step / step time / 8 TB/s
    }
    if pipelined:
        result["pipelined"] = pipelined
    ctx = dict(w=w, xs_oim=xs_oim, xs_spu=xs_spu, n_rot=n_rot, tdt=tdt, code=code, es=es, stream=stream,
               x_oim_host=x_oim_host, x_spu_host=x_spu_host, chain_gpu=chain_gpu)
    return result, ctx


def brief(r):
    """One workload's line of the `configs` table."""
    ro = r["roofline"]
    return {"workload": r["config"]["workload"], "tokens_per_step": r["config"]["tokens_per_step"], "ms_per_step": r["ms_per_step"],
            "value": r["value"], "unit": "tokens/s", "pct_of_peak_hbm": r["pct_of_peak_hbm"],
            "pipelined_ms_per_step": r.get("pipelined", {}).get("ms_per_step"),
            "roofline": {k: ro.get(k) for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "avg_us", "traffic", "traffic_source")},
            "kernels_us_per_step": {k["kernel"]: k["us_per_step"] for k in ro["kernels"]}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (the path shards over the batch with no exchange); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2512_09010_amd import binding as lv
    from paper_2512_09010_amd import workloads as wl

    lv.lib()                                       # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    cfgs = [args.config] if args.config is not None else [1, 2, 3, 4]
    head = args.config if args.config is not None else HEADLINE
    table, head_result, ctx = [], None, None
    for c in cfgs:
        r, cx = run_config(c, args, lv, wl, torch, np)
        table.append(brief(r))
        if c == head:
            head_result, ctx = r, cx
        else:
            del cx
            torch.cuda.empty_cache()
    w = ctx["w"]
    result = {"metric": "visual tokens compressed/sec (OIM+SPU) on 1 MI355X; % of peak HBM GB/s", "value": head_result["value"],
              "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head_result["ms_per_step"],
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head_result["dtype"], "data": "synthetic",
              "config": head_result["config"], "roofline": head_result["roofline"], "pct_of_peak_hbm": head_result["pct_of_peak_hbm"],
              "configs": table}
    if "pipelined" in head_result:
        result["pipelined"] = head_result["pipelined"]
    if args.oim_wide:
        result["oim_wide"] = oim_wide_leg(lv, torch, w, ctx["xs_oim"], ctx["n_rot"], ctx["tdt"], ctx["code"], ctx["es"], ctx["stream"], args.steps)
    if args.next_rows:
        result["next_rows"] = next_rows_leg(lv, torch, w, ctx["xs_oim"], ctx["xs_spu"], ctx["n_rot"], ctx["tdt"], ctx["code"], ctx["es"],
                                            ctx["stream"], min(args.steps, 50))
    if not args.no_cpu_baseline:
        result["cpu_baseline"], result["chained"] = cpu_baseline(w, ctx["x_oim_host"], ctx["chain_gpu"])
    print(json.dumps(result))


def oim_wide_leg(lv, torch, w, xs_oim, n_rot, tdt, code, es, stream, steps):
    """luvc_oim_merge_wide in the paper's appendix setting on the workload's encoder grid: every source of a line is
    compared with every destination of the line, merge number 2, three OIM operations (W then H, three times)."""
    import numpy as np
    dev = xs_oim[0].device
    passes = [(1, 2), (0, 2)] * 3
    Ho, Wo = lv.out_grid(w.H, w.W, passes)
    out = dict(x=torch.empty((w.grids, Ho, Wo, w.D), dtype=tdt, device=dev), sizes=torch.empty((w.grids, Ho, Wo), dtype=torch.int32, device=dev),
               merged_map=torch.empty((w.grids, w.H * w.W), dtype=torch.int32, device=dev),
               kept_map=torch.empty((w.grids, Ho * Wo), dtype=torch.int32, device=dev))
    ws = torch.empty(lv.luvc_oim_wide_workspace_bytes(w.grids, w.H, w.W, w.D, code, passes, 0), dtype=torch.uint8, device=dev)

    def call(i):
        lv.luvc_oim_merge_wide(xs_oim[i % n_rot], passes, 0, workspace=ws, stream=stream, out=out)

    for i in range(5):
        call(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        call(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    n_prof = min(steps, 20)
    prof = lv.LaunchProfile(n_prof * 32)
    prof.start()
    for i in range(n_prof):
        call(i)
    prof.stop()
    torch.cuda.synchronize()
    per = {}
    for name, t in prof.results():
        per.setdefault(name, []).append(t)
    prof.close()
    # algorithmic bytes of a pass that runs as one launch (oim_wide_line): every token of its grid read once (the merged
    # rows it writes and the index grids are a few percent); the contraction it screens with runs in the storage
    # precision on the matrix cores and is far from their limit.  Lines beyond that kernel's limit run oim_line_gram
    # (fp64 contraction) instead, which is reported against the fp64 matrix peak as before.
    flops, nbytes, H, W = 0.0, 0.0, w.H, w.W
    for axis, m in passes:
        ln, nl = (W, H) if axis else (H, W)
        flops += 2.0 * w.grids * nl * ((ln + 1) // 2) * (ln // 2) * w.D
        nbytes += float(w.grids) * H * W * w.D * es
        H, W = (H, W - m) if axis else (H - m, W)
    kernels = {k: {"launches_per_call": len(v) / n_prof, "avg_us": round(float(np.mean(v)) * 1e3, 2)} for k, v in per.items()}
    if "oim_wide_line" in per:
        g = float(np.sum(per["oim_wide_line"])) / n_prof
        roof = {"kernel": "oim_wide_line", "bound": "hbm", "achieved": round(nbytes / (g * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                "frac": round(nbytes / (g * 1e-3) / 1e9 / 8000.0, 4), "algorithmic_bytes_per_call": int(nbytes)}
    else:
        g = float(np.sum(per.get("oim_line_gram", [0.0]))) / n_prof
        roof = {"kernel": "oim_line_gram", "bound": "mfma", "dtype": "f64", "achieved": round(flops / (g * 1e-3) / 1e12, 2) if g else None,
                "peak": 78.6, "unit": "TFLOP/s", "frac": round(flops / (g * 1e-3) / 1e12 / 78.6, 4) if g else None,
                "algorithmic_flops_per_call": int(flops)}
    return {"what": "whole-line matching (radius 0), m = 2, passes (W,2),(H,2) x 3", "ms_per_call": round(ms, 5),
            "tokens_per_s": round(w.tokens_in / (ms * 1e-3), 1), "kernels": kernels, "roofline": roof}


def _time_call(torch, lv, call, steps):
    """ms per call (wall clock over `steps` calls on one stream) and the per-kernel averages of 10 more calls."""
    import numpy as np
    for i in range(3):
        call(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        call(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    n_prof = 10
    prof = lv.LaunchProfile(n_prof * 64)
    prof.start()
    for i in range(n_prof):
        call(i)
    prof.stop()
    torch.cuda.synchronize()
    per = {}
    for name, t in prof.results():
        per.setdefault(name, []).append(t)
    prof.close()
    kernels = {k: {"launches_per_call": len(v) / n_prof, "avg_us": round(float(np.mean(v)) * 1e3, 2)} for k, v in per.items()}
    return ms, kernels


def next_rows_leg(lv, torch, w, xs_oim, xs_spu, n_rot, tdt, code, es, stream, steps):
    """Timings of the entry points beyond the hot path, on tensors of the workload's shapes: decisions on a key tensor,
    value enhancement, a three-stage cascade, ragged batches.  Same rotation over input copies as the main step."""
    dev = xs_oim[0].device
    res = {}
    passes = w.oim_calls[0]
    B, H, W, D = xs_oim[0].shape
    Ho, Wo = lv.out_grid(H, W, passes)

    # ---- decisions on a key tensor of 128 channels (one attention head's keys), merge applied to tokens and keys
    Dm = 128
    keys = [x[..., :Dm].contiguous() for x in xs_oim[:2]]
    ws = torch.empty(lv.luvc_oim_keyed_workspace_bytes(B, H, W, D, Dm, code, passes, 1), dtype=torch.uint8, device=dev)
    out = dict(x=torch.empty((B, Ho, Wo, D), dtype=tdt, device=dev), metric=torch.empty((B, Ho, Wo, Dm), dtype=tdt, device=dev),
               sizes=torch.empty((B, Ho, Wo), dtype=torch.int32, device=dev), merged_map=torch.empty((B, H * W), dtype=torch.int32, device=dev),
               kept_map=torch.empty((B, Ho * Wo), dtype=torch.int32, device=dev))
    ms, kern = _time_call(torch, lv, lambda i: lv.luvc_oim_merge_keyed(xs_oim[i % n_rot], keys[i % 2], passes, 1, workspace=ws, stream=stream, out=out), steps)
    res["oim_keyed"] = {"what": f"luvc_oim_merge_keyed, keys {B}x{H}x{W}x{Dm}, same schedule as the step", "ms_per_call": round(ms, 5), "kernels": kern}

    # ---- the same keys with the paper's appendix setting: every destination of the line a candidate, merge number 2, three operations
    wpasses = [(1, 2), (0, 2)] * 3
    Hw, Ww = lv.out_grid(H, W, wpasses)
    ws2 = torch.empty(lv.luvc_oim_keyed_workspace_bytes(B, H, W, D, Dm, code, wpasses, 0), dtype=torch.uint8, device=dev)
    out2 = dict(x=torch.empty((B, Hw, Ww, D), dtype=tdt, device=dev), metric=torch.empty((B, Hw, Ww, Dm), dtype=tdt, device=dev),
                sizes=torch.empty((B, Hw, Ww), dtype=torch.int32, device=dev), merged_map=torch.empty((B, H * W), dtype=torch.int32, device=dev),
                kept_map=torch.empty((B, Hw * Ww), dtype=torch.int32, device=dev))
    ms, kern = _time_call(torch, lv, lambda i: lv.luvc_oim_merge_keyed(xs_oim[i % n_rot], keys[i % 2], wpasses, 0, workspace=ws2, stream=stream, out=out2), steps)
    res["oim_keyed_wide"] = {"what": f"luvc_oim_merge_keyed, keys {B}x{H}x{W}x{Dm}, whole-line matching, m = 2, passes (W,2),(H,2) x 3",
                             "ms_per_call": round(ms, 5), "kernels": kern}
    del ws2, out2

    # ---- V + log s on a tensor of the encoder grid's size
    sizes = torch.randint(1, 5, (B, H, W), dtype=torch.int32, device=dev)
    vout = torch.empty_like(xs_oim[0])
    ms, kern = _time_call(torch, lv, lambda i: lv.luvc_value_enhance(xs_oim[i % n_rot], sizes, stream=stream, out=vout), steps)
    k_us = kern.get("value_enhance", {}).get("avg_us")
    by = 2 * xs_oim[0].numel() * es
    res["value_enhance"] = {"what": f"luvc_value_enhance on {B * H * W} rows x {D}", "ms_per_call": round(ms, 5), "kernels": kern,
                            "roofline": {"bound": "hbm", "algorithmic_bytes": by, "achieved": round(by / (k_us * 1e-6) / 1e9, 1) if k_us else None,
                                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(by / (k_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if k_us else None}}

    # ---- a cascade of three stages without the layers between them: every stage reads the rows the previous one kept
    Bs, N, Ds = xs_spu[0].shape
    keeps = lv.luvc_spu_cascade_keeps(N, w.keep_ratio, 3, eliminate=False)
    alive = [N] + keeps[:-1]
    sigmas = [max(1, int(w.keep_ratio * n / 2)) if n > 1 else 0 for n in alive]
    wss = torch.empty(max(lv.luvc_spu_workspace_bytes(Bs, n, Ds, code, sg) for n, sg in zip(alive, sigmas)), dtype=torch.uint8, device=dev)
    outs = [dict(scores=torch.empty((Bs, n), dtype=torch.float32, device=dev), kept_idx=torch.empty((Bs, k), dtype=torch.int32, device=dev),
                 origin=torch.empty((Bs, k), dtype=torch.int32, device=dev), x=torch.empty((Bs, k, Ds), dtype=tdt, device=dev))
            for n, k in zip(alive, keeps)]

    def cascade(i):
        x, org = xs_spu[i % n_rot], None
        for st in range(3):
            o = lv.luvc_spu_stage(x, sigmas[st], keeps[st], True, origin=org, workspace=wss, stream=stream, out=outs[st])
            x, org = o["x"], o["origin"]
    ms, kern = _time_call(torch, lv, cascade, steps)
    res["spu_cascade"] = {"what": f"three luvc_spu_stage calls, tokens {alive} -> keeps {keeps}, sigma {sigmas}", "ms_per_call": round(ms, 5), "kernels": kern}

    # ---- ragged batches: the workload's tokens as grids of three aspect ratios / samples of two lengths
    shapes = [(H, W)] * max(1, B // 2) + [(H // 2, W * 2)] * max(1, B // 4) + [(H * 2, W // 2)] * max(1, B // 4)
    schedules = [lv.luvc_oim_plan_anyres(h, ww, Ho * Wo) for h, ww in shapes]
    T = sum(h * ww for h, ww in shapes)
    xr = [x.reshape(-1, D)[:T].contiguous() if x.numel() // D >= T else None for x in xs_oim[:2]]
    if all(a is not None for a in xr):
        ms, kern = _time_call(torch, lv, lambda i: lv.luvc_oim_merge_ragged(xr[i % 2], shapes, schedules, stream=stream), steps)
        res["oim_ragged"] = {"what": f"luvc_oim_merge_ragged, {len(shapes)} grids of shapes {sorted(set(shapes))}, any-res plan to {Ho * Wo} tokens each "
                                     "(the binding allocates the outputs on every call)", "ms_per_call": round(ms, 5), "kernels": kern}
    lengths = [N] * max(1, Bs // 2) + [N // 2] * (Bs - max(1, Bs // 2)) * 2
    if sum(lengths) <= Bs * N:
        xp = [x.reshape(-1, Ds)[:sum(lengths)] for x in xs_spu[:2]]
        sg = [max(1, int(w.keep_ratio * n / 2)) for n in lengths]
        kp = [lv.luvc_keep_count(n, w.keep_ratio) for n in lengths]
        ms, kern = _time_call(torch, lv, lambda i: lv.luvc_spu_stage_ragged(xp[i % 2], lengths, sg, kp, stream=stream), steps)
        res["spu_ragged"] = {"what": f"luvc_spu_stage_ragged, lengths {lengths} (the binding allocates the outputs on every call)",
                             "ms_per_call": round(ms, 5), "kernels": kern}
    return res


def _omp_threads(n):
    """Sets the thread count of the OpenMP runtime the oracle is linked against; returns the count now in force."""
    import ctypes
    try:
        g = ctypes.CDLL("libgomp.so.1")
        if n:
            g.omp_set_num_threads(int(n))
        return int(g.omp_get_max_threads())
    except OSError:
        return None


def cpu_baseline(w, x_oim_host, chain_gpu):
    """The oracle as it stands on the same chain the GPU ran once before the timed steps (OIM, the merged tokens
    projected to the SPU width, SPU score, keep): timed on all of this host's cores over the whole batch and on one
    thread over one SPU sample's share of it, and compared with what the GPU produced.  Returns (cpu_baseline, chained)."""
    import numpy as np
    import oracle
    from paper_2512_09010_amd import workloads as wl

    OIM_MARGIN, SPU_MARGIN = 1e-10, 2e-6          # as in tests/gpu_util.py
    rm = oracle.ROUND_BF16 if w.dtype == "bf16" else oracle.ROUND_F32
    oracle.lib()
    omp = _omp_threads(0) or int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))

    def chain(x_io, n_samples):
        """oracle OIM calls -> projection -> oracle score + keep on the first n_samples samples' share of the batch."""
        g = n_samples * (w.grids // w.spu_B)
        t0 = time.perf_counter()
        cur, sizes, outs = wl.widen(x_io[:g], w.dtype), None, []
        for passes in w.oim_calls:
            r = oracle.oim_merge(cur, passes, sizes=sizes, round_mode=rm)
            outs.append(r)
            cur, sizes = r["x"], r["sizes"]
        t1 = time.perf_counter()
        sub = wl.Workload(**{**w.__dict__, "grids": g, "spu_B": n_samples})
        xs = wl.spu_input_from_merged(sub, cur)            # input generation, not timed
        xs64 = wl.widen(xs, w.dtype)
        t2 = time.perf_counter()
        sc = oracle.spu_score(xs64, w.sigma, True)
        pr = oracle.spu_prune(sc, w.n_keep, xs64)
        t3 = time.perf_counter()
        return dict(oim=outs, xs=xs, scores=sc, prune=pr, t_oim=t1 - t0, t_spu=t3 - t2, tokens=g * w.H * w.W)

    full = chain(x_oim_host, w.spu_B)
    _omp_threads(1)
    one = chain(x_oim_host, 1)
    _omp_threads(omp)
    base = {"value": round(full["tokens"] / (full["t_oim"] + full["t_spu"]), 1), "unit": "tokens/s", "cores": omp, "kind": "oracle",
            "threads_used": {"oim": int(min(omp, w.grids)), "spu": int(min(omp, w.spu_B))},
            "sample": f"all {w.grids} OIM grids + all {w.spu_B} SPU samples of {w.name} (the chained run)",
            "seconds": {"oim": round(full["t_oim"], 3), "spu": round(full["t_spu"], 3)},
            "one_thread": {"value": round(one["tokens"] / (one["t_oim"] + one["t_spu"]), 1), "unit": "tokens/s", "cores": 1,
                           "sample": f"{w.grids // w.spu_B} OIM grid(s) + 1 SPU sample of {w.name}",
                           "seconds": {"oim": round(one["t_oim"], 3), "spu": round(one["t_spu"], 3)}}}

    # ---- the GPU's chained run against the oracle's
    maps_equal, bits_equal, margin = True, True, float("inf")
    for ref, got in zip(full["oim"], chain_gpu["oim"]):
        margin = min(margin, float(ref["margin"]))
        maps_equal &= bool(np.array_equal(got["merged_map"], ref["merged_map"]) and np.array_equal(got["kept_map"], ref["kept_map"])
                           and np.array_equal(got["sizes"].astype(np.int64), ref["sizes"]))
        gx = wl.widen(got["x"], w.dtype)
        bits_equal &= bool(np.array_equal(gx, ref["x"])) if w.dtype == "bf16" else bool(np.allclose(gx, ref["x"], rtol=1e-5, atol=0))
    gpu_xs = wl.spu_input_from_merged(w, wl.bf16_bits_to_f32(chain_gpu["oim"][-1]["x"]) if w.dtype == "bf16" else chain_gpu["oim"][-1]["x"])
    same_input = bool(np.array_equal(gpu_xs, full["xs"]))
    ref_sc, ref_pr = full["scores"], full["prune"]
    if not same_input:                              # the oracle then judges the SPU calls on the tensor the GPU read
        xs64 = wl.widen(gpu_xs, w.dtype)
        ref_sc = oracle.spu_score(xs64, w.sigma, True)
        ref_pr = oracle.spu_prune(ref_sc, w.n_keep, xs64)
    got_sc = chain_gpu["scores"].astype(np.float64)
    rel = float(np.max(np.abs(got_sc - ref_sc) / np.maximum(np.abs(ref_sc), 1e-300)))
    own = oracle.spu_prune(got_sc, w.n_keep)["kept_idx"]
    chained = {"what": "luvc_oim_merge -> host projection -> luvc_spu_score -> luvc_spu_prune on the GPU's own bits, once, untimed, "
                       "against the oracle run on the same chain",
               "oim_maps_and_sizes_equal": maps_equal, "oim_features_equal": bits_equal, "oim_decision_margin": margin,
               "oim_margin_threshold": OIM_MARGIN, "spu_input_equal": same_input, "score_max_rel_err": rel, "score_tolerance": 1e-5,
               "kept_idx_equal_to_selection_on_own_scores": bool(np.array_equal(chain_gpu["kept_idx"], own)),
               "kept_idx_equal_to_oracle": bool(np.array_equal(chain_gpu["kept_idx"], ref_pr["kept_idx"])),
               "keep_boundary_margin": float(ref_pr["margin"]), "keep_margin_threshold": SPU_MARGIN,
               "kept_rows_equal": bool(np.array_equal(wl.widen(chain_gpu["x_keep"], w.dtype), ref_pr["x"]))
               if np.array_equal(chain_gpu["kept_idx"], ref_pr["kept_idx"]) else None}
    chained["ok"] = bool((maps_equal and bits_equal or margin <= OIM_MARGIN) and rel <= 1e-5
                         and chained["kept_idx_equal_to_selection_on_own_scores"]
                         and (chained["kept_idx_equal_to_oracle"] or ref_pr["margin"] <= SPU_MARGIN))
    return base, chained


if __name__ == "__main__":
    main()
