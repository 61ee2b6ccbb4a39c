#!/usr/bin/env python3
"""Benchmark of the token-recall hot path on one MI355X.

One step = one ilre_recall call (row statistics, column scores, pooling, budgeted top-k) over the
1M-token Llama-3.1-8B-shaped synthetic key cache (workload cfg5_1m), inputs resident in HBM.
Prints ONE JSON line: whole-job context tokens/s, the roofline of the dominant kernel (timed with
HIP events on the launch stream) and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_MFMA_TFLOPS = 157.3  # fp32 matrix path (cfg 1 only)
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "score_kernel_cfg5_1m_hbm_traffic.md")


def recorded_traffic() -> dict:
    """HBM bytes per launch as recorded by the rocprofv3 --pmc runs (FETCH_SIZE + WRITE_SIZE scaled by the
    256 MiB copy): the machine-readable line `traffic_bytes_per_launch: name=value ...` of the summary under
    profiles/.  A counter figure from that profiled run, not something this script measures."""
    out = {}
    try:
        with open(TRAFFIC_PROFILE) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    for item in line.split(":", 1)[1].split():
                        name, value = item.split("=")
                        out[name] = float(value)
    except OSError:
        pass
    return out


def mfma_ceiling(il, torch, launches: int = 5, iters: int = 2000) -> dict:
    """Register-only loops (ilre_probe_mfma_ceiling) on random and on constant bf16 operands: TFLOP/s from HIP events,
    the shader clock from the cycle and 100 MHz counters each workgroup reads at its start and end."""
    out = torch.empty(il.ILRE_PROBE_OUT_BYTES, dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    operand_sets = {"random": torch.randn(il.ILRE_PROBE_OPERAND_BYTES // 2, device="cuda", generator=g).to(torch.bfloat16),
                    "constant": torch.ones(il.ILRE_PROBE_OPERAND_BYTES // 2, device="cuda", dtype=torch.bfloat16)}
    rows = []
    variant = 0
    while il.ilre_probe_describe(variant) is not None:
        for name, ops in operand_sets.items():
            if name == "constant" and variant > 1:
                continue
            for _ in range(2):
                flops = il.ilre_probe_mfma_ceiling(variant, iters, ops, out)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(launches):
                il.ilre_probe_mfma_ceiling(variant, iters, ops, out)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / launches
            clk = out[1 << 20:(1 << 20) + 4096].view(torch.int64).view(256, 2).double().cpu()
            per_wg = clk[:, 0] / clk[:, 1] * 0.1                       # cycles per 10 ns tick
            ghz = float(per_wg.mean())
            # workgroup b runs on XCD b mod 8: the dies do not hold the same clock under load
            by_xcd = [round(float(per_wg[x::8].mean()), 3) for x in range(8)]
            tf = flops / (ms * 1e-3) / 1e12
            rows.append({"variant": variant, "what": il.ilre_probe_describe(variant), "operands": name,
                         "ms": round(ms, 4), "tflops": round(tf, 1), "frac_of_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                         "clock_ghz": round(ghz, 3), "clock_ghz_by_xcd": by_xcd,
                         # the MFMA pipe's share of the cycles at the measured clock; for the loops without MFMAs,
                         # the same ratio for the MFMAs that were left out (above 1: the vector work alone is faster)
                         "mfma_busy": round(tf / (PEAK_BF16_TFLOPS * ghz / 2.4), 4) if ghz > 0 else None})
        variant += 1
    def pick(v, o):
        return next(r["tflops"] for r in rows if r["variant"] == v and r["operands"] == o)
    mix = max(r["tflops"] for r in rows if r["operands"] == "random" and r["variant"] in (1, 3, 6))
    return {"what": "register-only loops: 8 bf16 MFMAs 32x32x16 per 32x32 block, per logit fma + exp2 + add on the block "
                    "before (the scoring kernels' mix); no LDS, no loads, no barriers; one workgroup per CU",
            "iters": iters, "launches": launches,
            "mix_random_tflops": mix, "mix_random_frac_of_peak": round(mix / PEAK_BF16_TFLOPS, 4),
            "mfma_only_random_tflops": pick(0, "random"), "mfma_only_constant_tflops": pick(0, "constant"),
            "rows": rows}


def run_workload(il, torch, np, inputs, cfg: int, steps: int, warmup: int, calib_copy: bool = False, warm_ms: float = 0.0):
    """Times `steps` ilre_recall calls on workload cfg (inputs resident in HBM), then the same steps through the
    staged entry points with HIP events between the stages.  Returns (summary dict, state for the other legs)."""
    wl = inputs.CONFIGS[cfg]
    t0 = time.time()
    inp = inputs.generate(wl)
    gen_s = time.time() - t0
    q, k = il.to_device(inp.q), il.to_device(inp.k)
    kernels, budget = wl.pool_kernels, wl.budget
    dt = il.ILRE_BF16 if wl.dtype == "bf16" else il.ILRE_F32
    ws = il.alloc_workspace(wl.L, wl.Lq, wl.Hq, wl.Hkv, wl.d, len(kernels), dt)
    out_idx = torch.empty(min(budget, wl.L), dtype=torch.int32, device="cuda")
    out_scores = torch.empty(wl.L, dtype=torch.float32, device="cuda")

    def step():
        il.ilre_recall(q, k, budget, kernels, workspace=ws, out_idx=out_idx, out_scores=out_scores)

    if calib_copy:
        cal_src = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda")
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()
        del cal_src, cal_dst

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # the short workloads follow seconds of host-side input generation with the GPU idle: keep stepping (untimed)
    # until the chip has been busy for warm_ms, so that the timed steps do not include its clock ramp
    t_w = time.perf_counter()
    while (time.perf_counter() - t_w) * 1e3 < warm_ms:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    tokens_per_s = wl.L * steps / wall

    # Per-stage device time over the same number of steps: the three staged entry points launch
    # exactly the kernels ilre_recall launches; HIP events on the launch stream bracket each stage.
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for i in range(steps):
        ev[i][0].record()
        rmax, rsum = il.ilre_row_stats(q, k, workspace=ws)
        ev[i][1].record()
        sc = il.ilre_col_scores(q, k, rmax, rsum, workspace=ws)
        ev[i][2].record()
        il.ilre_select(sc, budget, kernels, workspace=ws, out_idx=out_idx)
        ev[i][3].record()
    torch.cuda.synchronize()
    stage_ms = [float(np.mean([ev[i][s].elapsed_time(ev[i][s + 1]) for i in range(steps)])) for s in range(3)]
    # Device time of the whole step, HIP events around the same K calls, and of the two scoring entry points run
    # back to back with no event between them.  The difference is what the selection adds to a step (the staged
    # col_scores call ends with the sum of the partial score vectors, which the whole path does inside the
    # selection's first pass, so the difference is net of that sum).  The `select` stage above is the selection
    # alone, first kernel to last, behind an event; it also pays for starting on scores no cache holds yet.
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    r0.record()
    for _ in range(steps):
        step()
    r1.record()
    torch.cuda.synchronize()
    recall_ms = r0.elapsed_time(r1) / steps
    r0.record()
    for _ in range(steps):
        rmax, rsum = il.ilre_row_stats(q, k, workspace=ws)
        sc = il.ilre_col_scores(q, k, rmax, rsum, workspace=ws)
    r1.record()
    torch.cuda.synchronize()
    scoring_ms = r0.elapsed_time(r1) / steps

    flops_per_pass = 2.0 * wl.Hq * wl.Lq * wl.L * wl.d
    dom = 0 if stage_ms[0] >= stage_ms[1] else 1
    dom_name = ("row_stats (score_kernel MODE 0)", "col_scores (score_kernel MODE 1)")[dom]
    achieved = flops_per_pass / (stage_ms[dom] * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_F32_MFMA_TFLOPS
    roofline = {"bound": "mfma", "kernel": dom_name, "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), "traffic": None,
                "flops_per_launch": flops_per_pass, "launch_ms": round(stage_ms[dom], 4)}
    # Arithmetic intensity of a scoring pass is G*Lq flop per byte of K; below the ridge (peak flops / peak
    # bytes, about 312 for bf16) the pass is priced against HBM instead: algorithmic bytes = the key cache once.
    es = 2 if wl.dtype == "bf16" else 4
    if wl.dtype == "bf16" and (wl.Hq // wl.Hkv) * wl.Lq < PEAK_BF16_TFLOPS * 1e12 / 8e12:
        k_bytes = float(wl.Hkv) * wl.L * wl.d * es + (4.0 * wl.L if dom == 1 else 0.0)
        gbs = k_bytes / (stage_ms[dom] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": dom_name, "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s",
                    "frac": round(gbs / 8000.0, 4), "traffic": None, "bytes_per_launch": k_bytes,
                    "launch_ms": round(stage_ms[dom], 4),
                    "mfma_frac_of_peak": round(achieved / peak, 4)}
    summary = {
        "value": round(tokens_per_s, 1), "ms_per_step": round(ms_per_step, 4), "dtype": wl.dtype,
        "config": {"workload": wl.name, "L": wl.L, "Lq": wl.Lq, "Hq": wl.Hq, "Hkv": wl.Hkv, "d": wl.d,
                   "pool_kernels": list(kernels), "budget": budget, "needle_spans": wl.n_spans,
                   "input_gen_s": round(gen_s, 1)},
        "stage_ms": {"row_stats": round(stage_ms[0], 4), "col_scores": round(stage_ms[1], 4),
                     "select": round(stage_ms[2], 4), "recall_device": round(recall_ms, 4),
                     "scoring_device": round(scoring_ms, 4), "selection_in_recall": round(recall_ms - scoring_ms, 4)},
        "stage_tflops": {"row_stats": round(flops_per_pass / stage_ms[0] / 1e9, 1),
                         "col_scores": round(flops_per_pass / stage_ms[1] / 1e9, 1)},
        "roofline": roofline,
        # the definition computes Q K^T once; the second pass is a recompute forced by memory
        "useful": {"flops_counted_once": flops_per_pass, "tflops": round(flops_per_pass / (ms_per_step * 1e-3) / 1e12, 1),
                   "frac_of_peak": round(flops_per_pass / (ms_per_step * 1e-3) / 1e12 / peak, 4)},
    }
    state = {"wl": wl, "inp": inp, "q": q, "k": k, "ws": ws, "out_idx": out_idx, "out_scores": out_scores, "dom": dom,
             "dt": dt}
    return summary, state


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=25)
    ap.add_argument("--config", type=int, default=5, help="workload number (1-5); the metric is quoted on 5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-row-divisor", type=int, default=2,
                    help="the cpu_baseline leg runs the oracle on all context tokens and 1/divisor of the query tokens")
    ap.add_argument("--no-configs", action="store_true", help="skip the lines for the other workloads (cfg 2-4)")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel from rocprofv3 --pmc; default: the figure "
                         "recorded under profiles/ for this workload, if any")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy, the known-size kernel that scales "
                         "FETCH_SIZE / WRITE_SIZE in rocprofv3 --pmc runs of this script")
    ap.add_argument("--no-select-scaled", action="store_true",
                    help="skip the scaled selection leg (ilre_select on 2^27 synthetic scores, HBM roofline)")
    ap.add_argument("--no-rerope", action="store_true", help="skip the leg that times the DCA re-RoPE of the key cache")
    ap.add_argument("--no-paper-allocation", action="store_true",
                    help="skip the leg that times the whole step with Algorithm 1 as printed (48 max/average combinations)")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the leg that measures what register-only MFMA loops with the scoring kernels' "
                         "instruction mix reach on this GPU (the ceiling the roofline fraction is to be read against)")
    ap.add_argument("--mfma-ceiling-only", action="store_true", help="run only that leg (for rocprofv3 --pmc runs)")
    ap.add_argument("--gemm-context", action="store_true",
                    help="also time a library bf16 GEMM (8192^3, random operands) as context for the MFMA roofline")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on exactly one GPU (got --gpus {args.gpus}); "
              "the path has no multi-GPU code. Re-run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import inputs
    import paper_2508_17892_amd as il
    to_device = il.to_device

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    il.load()  # fails loudly if the HIP library is not built
    if args.mfma_ceiling_only:
        print(json.dumps({"mfma_ceiling": mfma_ceiling(il, torch)}))
        return 0

    summary, st = run_workload(il, torch, np, inputs, args.config, args.steps, args.warmup, args.calib_copy)
    wl, inp, q, k, ws, out_idx, out_scores = (st[x] for x in ("wl", "inp", "q", "k", "ws", "out_idx", "out_scores"))
    kernels, budget, dt, dom = wl.pool_kernels, wl.budget, st["dt"], st["dom"]
    del st
    rec = recorded_traffic() if args.config == 5 else {}
    traffic = args.traffic_bytes
    if traffic is None:
        traffic = rec.get("score_mode1" if dom == 1 else "score_mode0")
    summary["roofline"]["traffic"] = traffic
    if traffic is not None and args.traffic_bytes is None:
        summary["roofline"]["traffic_source"] = "counter figure recorded in profiles/" + os.path.basename(TRAFFIC_PROFILE)
    result = {
        "metric": "context tokens/sec recalled at L=1M (single GPU)" if args.config == 5
                  else f"context tokens/sec recalled at L={wl.L} (single GPU)",
        "value": summary["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": summary["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": summary["config"], "stage_ms": summary["stage_ms"], "stage_tflops": summary["stage_tflops"],
        "roofline": summary["roofline"], "useful": summary["useful"],
    }

    if not args.no_paper_allocation:
        # The same step with Algorithm 1 as printed (strided max pooling x average pooling, the paper's
        # default 3 x 16 combinations, K_m cap, sink 4) in place of the window-max form.
        mk, ak, sink = (2, 4, 8), tuple(range(1, 17)), 4
        ws_p = il.alloc_workspace_max_avg(wl.L, wl.Lq, wl.Hq, wl.Hkv, wl.d, sink, mk, len(ak), dt)
        p_idx = torch.empty(sink + min(budget, wl.L - sink), dtype=torch.int32, device="cuda")
        p_cnt = torch.empty(1, dtype=torch.int32, device="cuda")

        def paper_step():
            il.ilre_recall_max_avg(q, k, budget, mk, ak, sink, workspace=ws_p, out_idx=p_idx, out_count=p_cnt,
                                   out_scores=out_scores)

        for _ in range(args.warmup):
            paper_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            paper_step()
        torch.cuda.synchronize()
        p_wall = time.perf_counter() - t0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            il.ilre_select_max_avg(out_scores, budget, mk, ak, sink, workspace=ws_p, out_idx=p_idx, out_count=p_cnt)
        e1.record()
        torch.cuda.synchronize()
        result["paper_allocation"] = {"max_kernels": list(mk), "avg_kernels": list(ak), "sink": sink,
                                      "ms_per_step": round(p_wall * 1e3 / args.steps, 4),
                                      "tokens_per_s": round(wl.L * args.steps / p_wall, 1),
                                      "select_ms": round(e0.elapsed_time(e1) / args.steps, 4),
                                      "kept": int(p_cnt.item())}
        del ws_p

    if not args.no_rerope:
        # DCA on: the key cache is re-RoPE'd once before the recall step (second DCA equation), one
        # streaming pass; prefill chunks of 1024 tokens, the first with the 4 sink tokens, Llama-3.1 base.
        k_rot = torch.empty_like(k)
        il.ilre_rerope_keys(k, 1024, 4, rope_base=500000.0, out=k_rot)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            il.ilre_rerope_keys(k, 1024, 4, rope_base=500000.0, out=k_rot)
        e1.record()
        torch.cuda.synchronize()
        r_ms = e0.elapsed_time(e1) / args.steps
        r_bytes = 2.0 * k.numel() * k.element_size()
        result["rerope"] = {"chunk_tokens": 1024, "first_extra": 4, "rope_base": 500000.0, "ms": round(r_ms, 4),
                            "algorithmic_bytes": r_bytes, "bound": "hbm", "achieved": round(r_bytes / (r_ms * 1e-3) / 1e9, 1),
                            "peak": 8000.0, "unit": "GB/s", "frac": round(r_bytes / (r_ms * 1e-3) / 1e9 / 8000.0, 4),
                            "note": "ilre_rerope_keys on the same key cache, out of place: every key read once, written once"}
        del k_rot

    if not args.no_select_scaled:
        # At the listed workloads the score vector (<= 4 MiB) is cache resident and the selection
        # kernels are latency-bound; their HBM roofline is shown on a scaled instance instead:
        # 2^27 synthetic scores (512 MiB, dense background plus 64 needle spans), same kernels and budget.
        ws = None

        def scaled_scores(Ls):
            g = torch.Generator(device="cuda")
            g.manual_seed(1)
            big = torch.randn(Ls, device="cuda", generator=g)
            big.mul_(0.3).add_(1.0).mul_(0.0078).clamp_min_(1e-4)
            for start in torch.randint(0, Ls - 300, (64,), generator=torch.Generator().manual_seed(2)).tolist():
                big[start:start + 160] = torch.rand(160, device="cuda", generator=g) * 8
            return big

        def time_scaled(Ls):
            big = scaled_scores(Ls)
            ws_s = il.alloc_workspace(Ls, 1, 1, 1, 128, len(kernels), il.ILRE_F32)
            il.ilre_select(big, budget, kernels, workspace=ws_s, out_idx=out_idx)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                il.ilre_select(big, budget, kernels, workspace=ws_s, out_idx=out_idx)
            e1.record()
            torch.cuda.synchronize()
            del big, ws_s
            return e0.elapsed_time(e1) / args.steps

        Ls = 1 << 27
        sel_ms = time_scaled(Ls)
        alg = len(kernels) * 4.0 * Ls + 4.0 * budget
        result["select_scaled"] = {"L": Ls, "ms": round(sel_ms, 4), "algorithmic_bytes": alg, "bound": "hbm",
                                   "achieved": round(alg / (sel_ms * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                                   "frac": round(alg / (sel_ms * 1e-3) / 1e9 / 8000.0, 4),
                                   "note": "ilre_select alone on 2^27 synthetic scores; algorithmic bytes = n*4L + 4B "
                                           "(what a pass per kernel size over the scores would move)"}
        # what the kernels of this leg really move: the scores are streamed once (the pruning pre-pass), the
        # passes after it visit a few thousand fine chunks
        moved = rec.get("select_scaled")
        if moved is not None:
            result["select_scaled"].update({
                "traffic": moved, "traffic_source": "counter figure recorded in profiles/" + os.path.basename(TRAFFIC_PROFILE),
                "traffic_rate": round(moved / (sel_ms * 1e-3) / 1e9, 1),
                "traffic_frac": round(moved / (sel_ms * 1e-3) / 1e9 / 8000.0, 4)})
        # The dozen launches after the streaming pass cost the same 0.11 ms whatever the length; on 2^30 scores
        # (4 GiB, near the longest vector the library takes) the whole call is priced against the scores read once.
        Lx = 1 << 30
        big_ms = time_scaled(Lx)
        result["select_scaled"]["larger"] = {
            "L": Lx, "ms": round(big_ms, 4), "scores_once_bytes": 4.0 * Lx,
            "scores_once_rate": round(4.0 * Lx / (big_ms * 1e-3) / 1e9, 1),
            "scores_once_frac": round(4.0 * Lx / (big_ms * 1e-3) / 1e9 / 8000.0, 4),
            "note": "same call on 2^30 scores; rate = 4 L bytes (this design's one reading of the scores) over the whole call"}

    if not args.no_mfma_ceiling:
        result["mfma_ceiling"] = mfma_ceiling(il, torch)
        if result["roofline"]["bound"] == "mfma":
            result["roofline"]["frac_of_measured_ceiling"] = round(result["roofline"]["achieved"] /
                                                                   result["mfma_ceiling"]["mix_random_tflops"], 4)

    if args.gemm_context:
        n = 8192
        ga = torch.randn(n, n, device="cuda").to(torch.bfloat16)
        gb = torch.randn(n, n, device="cuda").to(torch.bfloat16)
        torch.matmul(ga, gb)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            torch.matmul(ga, gb)
        e1.record()
        torch.cuda.synchronize()
        result["context"] = {"library_bf16_gemm_8192_tflops": round(2.0 * n ** 3 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)}
        del ga, gb

    if not args.no_configs and args.config == 5:
        # The other bf16 workloads of the target (32K, 128K, 512K tokens), same measurement; the parity tests
        # cover them, these lines only say how fast they run.
        q = k = ws = None
        torch.cuda.empty_cache()
        result["configs"] = {}
        for cfg in (2, 3, 4):
            other, ost = run_workload(il, torch, np, inputs, cfg, args.steps, args.warmup, warm_ms=100.0)
            del ost
            torch.cuda.empty_cache()
            result["configs"][other["config"]["workload"]] = {
                "tokens_per_s": other["value"], "ms_per_step": other["ms_per_step"], "stage_ms": other["stage_ms"],
                "stage_tflops": other["stage_tflops"], "roofline": other["roofline"]}

    if not args.no_cpu_baseline:
        import oracle
        # All L context tokens (so that a row's logit vector is as long as in the full job: 8 MB at 1M tokens,
        # beyond the host's L2) and a sample of the query rows: the first Lq/div query tokens of every head.
        # The oracle's time is linear in the number of rows, so tokens/s of the whole job = L / (t * div).
        div = max(1, args.cpu_row_divisor)
        lq_s = max(1, wl.Lq // div)
        q_s = np.ascontiguousarray(inp.q[:, :lq_s, :])
        t0 = time.perf_counter()
        oracle.recall(q_s, inp.k, kernels, budget)
        cpu_s = time.perf_counter() - t0
        scale = wl.Lq / lq_s
        result["cpu_baseline"] = {"value": round(wl.L / (cpu_s * scale), 1), "unit": "tokens/s", "cores": oracle.num_threads(),
                                  "kind": "oracle", "seconds": round(cpu_s, 2),
                                  "sample": f"whole path on all {wl.L} context tokens of {wl.name} with {wl.Hq * lq_s} of the "
                                            f"{wl.Hq * wl.Lq} query rows (the first {lq_s} of {wl.Lq} query tokens of every "
                                            f"head), same kernels and budget; value = L / (seconds * {scale:g})"}
        digest = os.path.join(ROOT, "tests", "golden", f"fullsize_cfg{args.config}.json")
        if os.path.exists(digest):
            with open(digest) as f:
                g = json.load(f)
            result["cpu_baseline"]["full_job_elsewhere"] = {
                "seconds": g["oracle_seconds"], "cores": g["oracle_threads"],
                "tokens_per_s": round(wl.L / g["oracle_seconds"], 1),
                "note": "the oracle on every row of this workload, timed on the machine that wrote tests/golden/ "
                        "(scoring part only; not this box)"}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
