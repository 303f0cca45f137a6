#!/usr/bin/env python3
"""Benchmark of the PWLQ hot path on one MI355X.

A step is one pass of the whole path over the ResNet-50-shaped weight set
(54 tensors, 27 560 channels, 25.5 M binary32 weights, already resident in
HBM): pwlq_search_list (absmax, partition, candidate evaluation, refine,
argmin) followed by pwlq_quantize_list (codes, flags, dequantized weights),
per channel, b = 4, 1000 candidate breakpoints.

Prints one JSON line.  `value` is candidate-element evaluations per second of
the whole step; `roofline` describes the dominant kernel (the candidate
evaluation kernel) against the chip's binary32 vector issue rate;
`cpu_baseline` is the CPU oracle timed on this machine's host cores on a
stated sample of the same workload.
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

# Algorithmic work of one (element, candidate) evaluation in its plain
# branch-free form: compare, three selects, subtract, multiply, round,
# fused multiply-add (error), fused multiply-add (accumulate).
LANE_OPS_PER_EVAL = 9
# 157.3 TFLOP/s binary32 vector peak = 256 CUs x 128 lanes x 2 flop (FMA) x 2.4 GHz,
# i.e. 78.6e12 lane-instructions per second (one VALU instruction on one lane)
PEAK_LANE_OPS = 256 * 128 * 2.4e9


# One evaluation as this build's search kernel does it once the tile is partitioned by
# candidate block: multiply (or fused multiply-add in the tail), round, subtract,
# fused multiply-accumulate.
LANE_OPS_PER_EVAL_PARTITIONED = 4
PEAK_FLOPS_FP32 = 157.3e12          # the spec-sheet figure: packed fused multiply-adds


def sources_sha16() -> str:
    """Fingerprint of the kernel sources a counter summary under profiles/ belongs to."""
    import hashlib
    d = os.path.join(ROOT, "paper_2002_00104_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip")):
            with open(os.path.join(d, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read() + b"\0")
    return h.hexdigest()[:16]


def _profile_record(name: str):
    """The machine-readable line ('#json {...}') of a committed rocprofv3 summary
    under profiles/, or None."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("#json "):
                    return json.loads(line[6:])
    except (OSError, ValueError):
        pass
    return None


def _static_counters(tag: str, kernel: str):
    """Counters of `kernel` from the committed counter runs of the workload `tag`
    ('workload2', 'workload3_only_k9', ...): (valu wave-instructions per launch,
    HBM bytes per launch, dict describing where they come from)."""
    valu = traffic = None
    src = {}
    rec = _profile_record(f"valu_lds_counters_{tag}.txt")
    if rec and kernel in rec.get("kernels", {}):
        valu = float(rec["kernels"][kernel]["SQ_INSTS_VALU"])
        src["executed"] = {"file": f"profiles/valu_lds_counters_{tag}.txt", "static": True,
                           "counter": "SQ_INSTS_VALU per launch",
                           "kernel_sources_sha16": rec.get("kernel_sources_sha16"),
                           "matches_this_build": rec.get("kernel_sources_sha16") == sources_sha16()}
    rec = _profile_record(f"hbm_traffic_{tag}.txt")
    if rec and kernel in rec.get("kernels", {}):
        k = rec["kernels"][kernel]
        traffic = float(k["read_bytes"]) + float(k["written_bytes"])
        if "read_bytes_by_request_size" in k:
            # the L2's read requests priced at their own size (32, 64, 128 bytes) + the writes
            src["traffic_by_request_size"] = float(k["read_bytes_by_request_size"]) + float(k["written_bytes"])
        src["traffic"] = {"file": f"profiles/hbm_traffic_{tag}.txt", "static": True,
                          "counter": "FETCH_SIZE + WRITE_SIZE per launch, scaled by a plain copy",
                          "kernel_sources_sha16": rec.get("kernel_sources_sha16"),
                          "matches_this_build": rec.get("kernel_sources_sha16") == sources_sha16()}
    return valu, traffic, src


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--spinup-seconds", type=float, default=0.25,
                    help="untimed steps run for this long before the warm-up steps, so that the "
                         "chip is at its sustained clock when the timed region starts (0: none)")
    ap.add_argument("--workload", type=int, default=2, help="1..5 (default 2: ResNet-50 shapes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-linear", action="store_true",
                    help="skip the timing of the integer inner-product kernel")
    ap.add_argument("--hot-path-only", action="store_true",
                    help="time only the step (search_list + quantize_list), eager and replayed "
                         "from a HIP graph: no packed output, fast search, analytic selectors "
                         "or inner product")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the replay of the step from a HIP graph")
    ap.add_argument("--only-k", type=int, default=0,
                    help="keep only the tensors whose rows have this many elements "
                         "(e.g. 9: the depthwise channels of workload 3)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy three times (scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path "
              "(groups are independent, so it would shard by giving every GPU a "
              "block of whole channels or tensors, with no exchange). "
              "Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2002_00104_amd import pwlq, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.copy_calibration:
        a = torch.ones(64 << 20, dtype=torch.float32, device="cuda")       # 256 MiB
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_each_way": a.numel() * 4, "launches": 3}))
        return 0
    wl = synth.workload(args.workload)
    host = list(wl.tensors())
    if args.only_k:
        host = [t for t in host if t.shape[1] == args.only_k]
        if not host:
            print(f"workload {wl.index} has no tensor with K={args.only_k}", file=sys.stderr)
            return 2
    dev = [torch.from_numpy(t).cuda() for t in host]
    tl = pwlq.TensorList(dev, wl.mode)
    ws_search = torch.empty(pwlq.search_list_workspace_bytes(tl, wl.bits, wl.n_cand),
                            dtype=torch.uint8, device="cuda")
    ws_quant = torch.empty(max(256, pwlq.quantize_list_workspace_bytes(tl, wl.bits)),
                           dtype=torch.uint8, device="cuda")
    out = pwlq.alloc_search_outputs(tl.n_groups, "cuda")
    qout = pwlq.alloc_quantize_outputs(tl.n_elements, "cuda")

    def step():
        pwlq.search_list(tl, wl.bits, wl.n_cand, workspace=ws_search, out=out)
        pwlq.quantize_list(tl, wl.bits, out["p_star"], out["m"], workspace=ws_quant, out=qout)

    # Device spin-up, untimed, before the W warm-up steps and not one of them: after
    # idling the chip needs some tens of milliseconds under load to reach the clock it
    # then sustains (the evaluation kernel runs about 3 % slower during the first 30
    # steps), which a handful of 2 ms warm-up steps does not give it.  Reported in the
    # JSON line as config.spinup_steps.
    spinup_steps = 0
    s0 = time.perf_counter()
    while time.perf_counter() - s0 < args.spinup_seconds:
        for _ in range(5):
            step()
        torch.cuda.synchronize()
        spinup_steps += 5

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly K steps back to back, one synchronize on each side.
    # Inside it the library records HIP events on the launch stream around its
    # dominant kernel only (a ring of the last 64 launches, read after the closing
    # synchronize).  The split of a step into its two calls and the quantize
    # kernel's own duration come from a second, instrumented run of K steps that
    # does not count for `value`.
    pwlq.profile_enable(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        pwlq.search_list(tl, wl.bits, wl.n_cand, workspace=ws_search, out=out)
        pwlq.quantize_list(tl, wl.bits, out["p_star"], out["m"], workspace=ws_quant, out=qout)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    pwlq.profile_enable(0)
    recorded = min(args.steps, 64)
    k_search_ms = [pwlq.profile_ms(0, i) for i in range(recorded)]

    pwlq.profile_enable(2)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(args.steps):
        ev[i][0].record()
        pwlq.search_list(tl, wl.bits, wl.n_cand, workspace=ws_search, out=out)
        ev[i][1].record()
        pwlq.quantize_list(tl, wl.bits, out["p_star"], out["m"], workspace=ws_quant, out=qout)
        ev[i][2].record()
    torch.cuda.synchronize()
    pwlq.profile_enable(0)
    k_emit_ms = [pwlq.profile_ms(1, i) for i in range(recorded)]
    search_ms = [e[0].elapsed_time(e[1]) for e in ev]
    quant_ms = [e[1].elapsed_time(e[2]) for e in ev]
    e0, e1, e2 = ev[0]

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    n_elements = sum(t.size for t in host)
    evals = n_elements * wl.n_cand
    value = evals / (ms_per_step * 1e-3)
    keep_search = {k: v.clone() for k, v in out.items()}      # compared with the oracle below
    ks = float(np.mean(k_search_ms))
    emit_ms = float(np.mean(k_emit_ms))
    tag = f"workload{wl.index}" + (f"_only_k{args.only_k}" if args.only_k else "")
    search_kernel = pwlq.last_search_kernel()       # k_search; k_small for a call that is one fused launch
    valu, traffic, static_src = _static_counters(tag, search_kernel)
    fresh = valu is not None and static_src["executed"]["matches_this_build"]
    # Lane-instructions of the dominant kernel per launch.  Executed: SQ_INSTS_VALU x 64 of the
    # committed counter run of this workload, used only while the kernel sources are the
    # ones that run was made with.  Otherwise the algorithmic count of the partitioned
    # evaluation (4 per pair), which the executed count can only exceed.
    lane_ops = valu * 64 if fresh else float(LANE_OPS_PER_EVAL_PARTITIONED) * evals
    achieved = lane_ops / (ks * 1e-3)
    # what the search kernel must move: the partitioned tile and its offsets in, one
    # binary32 sum per (tile, candidate) out
    shape = pwlq.last_search_shape()
    algorithmic_bytes = 4.0 * n_elements + 4.0 * shape["tiles"] * (wl.n_cand + (wl.n_cand + 63) // 64 + 1)
    result = {
        "metric": "breakpoint-search candidate-elem evals/s; ResNet-50-shape per-channel PWLQ ms",
        "value": value,
        "unit": "candidate-element evaluations/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"configs[{wl.index - 1}] {wl.name}: {len(host)} tensors, "
                        f"{tl.n_groups} groups, {n_elements} fp32 weights"
                        f"{' (only K=%d)' % args.only_k if args.only_k else ''}, "
                        f"{'per-channel' if wl.mode == 0 else 'per-tensor'}, b={wl.bits}, "
                        f"{wl.n_cand} candidates",
            "evals_per_step": evals,
            "spinup_steps": spinup_steps,
            "search_ms": float(np.mean(search_ms)),
            "quantize_ms": float(np.mean(quant_ms)),
            "search_evals_per_s": evals / (float(np.mean(search_ms)) * 1e-3),
        },
        "roofline": {
            "kernel": search_kernel,
            "bound": "alu",
            "achieved": achieved / 1e12,
            "peak": PEAK_LANE_OPS / 1e12,
            "unit": "Tlane-op/s (fp32 VALU instructions x active lanes; peak = 256 CUs x 128 "
                    "lanes x 2.4 GHz, i.e. 157.3 TFLOP/s at 2 flop per lane-instruction)",
            "frac": achieved / PEAK_LANE_OPS,
            "lane_ops_counted": ("executed (static SQ_INSTS_VALU of the committed counter run, "
                                 "live kernel time)" if fresh else
                                 "algorithmic, 4 per evaluation (no counter run of this workload "
                                 "for these kernel sources)"),
            "lane_ops_per_eval": lane_ops / evals,
            "algorithmic_frac": LANE_OPS_PER_EVAL_PARTITIONED * evals / (ks * 1e-3) / PEAK_LANE_OPS,
            "canonical_equivalent": LANE_OPS_PER_EVAL * evals / (ks * 1e-3) / PEAK_LANE_OPS,
            "canonical_equivalent_note": "9 lane-instructions per evaluation (the branch-free form "
                                         "without the partition) over the same time and peak: a "
                                         "speed-up over that form, not a utilisation; may exceed 1",
            "flop_frac_of_157.3_TFLOPs": (lane_ops + evals) / (ks * 1e-3) / PEAK_FLOPS_FP32,
            "flop_frac_note": "flops = lane-instructions + one per evaluation (the accumulate is a "
                              "fused multiply-add); the 157.3 TFLOP/s figure needs packed fused "
                              "multiply-adds, which this build does not use",
            "traffic": traffic,
            "traffic_by_request_size": static_src.pop("traffic_by_request_size", None),
            "traffic_note": "traffic: FETCH_SIZE and WRITE_SIZE, each scaled by what it reads for a plain "
                            "copy.  FETCH_SIZE prices a 128-byte read request at 64 bytes (the copy's "
                            "factor 2.0) and a 64-byte one at 64, so the scaling doubles the reads of this "
                            "kernel, whose elements arrive as 64-byte scalar-cache fills; "
                            "traffic_by_request_size prices every read request of the L2 at its size "
                            "(TCC_EA0_RDREQ_32B/_64B/_128B) and adds the same writes",
            "algorithmic_bytes": algorithmic_bytes,
            "static_sources": static_src,
            "kernel_sources_sha16": sources_sha16(),
            "kernel_ms": ks,
            "kernel_evals_per_s": evals / (ks * 1e-3),
        },
        "quantize_roofline": {
            "kernel": pwlq.kernel_name(1),
            "bound": "hbm",
            "achieved": 10.0 * n_elements / (emit_ms * 1e-3) / 1e9,
            "peak": 8000.0,
            "unit": "GB/s",
            "frac": 10.0 * n_elements / (emit_ms * 1e-3) / 8e12,
            "kernel_ms": emit_ms,
        },
    }

    # What a plain device-to-device copy reaches on this chip (read + write bytes
    # per second), as the practical ceiling beside the 8 TB/s peak.
    ca = torch.empty(64 << 20, dtype=torch.float32, device="cuda")       # 256 MiB
    cb = torch.empty_like(ca)
    cb.copy_(ca)
    torch.cuda.synchronize()
    c0 = torch.cuda.Event(enable_timing=True)
    c1 = torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        cb.copy_(ca)
    c1.record()
    c1.synchronize()
    copy_gbps = 5 * 2.0 * ca.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    result["quantize_roofline"]["device_copy_GBps"] = copy_gbps
    result["quantize_roofline"]["frac_of_device_copy"] = result["quantize_roofline"]["achieved"] / copy_gbps
    del ca, cb

    # Beyond the step above, each timed on its own (skipped by --hot-path-only, so that a
    # profiler summary of that run averages each kernel over the timed steps alone).
    def extras():
        # Bit-packed quantizer output (b-bit code stream + 1-bit flag stream, no
        # dequantized copy): not part of the step above, timed on its own.
        layout = pwlq.PackedLayout(tl, wl.bits)
        pout = (torch.empty(max(layout.code_bytes, 4), dtype=torch.uint8, device="cuda"),
                torch.empty(max(layout.flag_bytes, 4), dtype=torch.uint8, device="cuda"), None)
        for _ in range(2):
            pwlq.quantize_packed_list(tl, wl.bits, out["p_star"], out["m"], layout=layout,
                                      workspace=ws_quant, out=pout)
        torch.cuda.synchronize()
        reps = max(3, min(args.steps, 10))
        e0.record()
        for _ in range(reps):
            pwlq.quantize_packed_list(tl, wl.bits, out["p_star"], out["m"], layout=layout,
                                      workspace=ws_quant, out=pout)
        e1.record()
        e1.synchronize()
        packed_ms = e0.elapsed_time(e1) / reps
        packed_bytes = n_elements * (4.0 + wl.bits / 8.0 + 1.0 / 8.0)
        result["quantize_packed"] = {
            "ms": packed_ms,
            "bytes_per_element": 4.0 + wl.bits / 8.0 + 1.0 / 8.0,
            "achieved": packed_bytes / (packed_ms * 1e-3) / 1e9,
            "peak": 8000.0,
            "unit": "GB/s",
            "note": "call time (table upload + kernel), w_hat not requested",
        }

        # The same search through the prefix-sum evaluator (pwlq_search_fast_list):
        # identical outputs, far fewer operations, so its rate is quoted in
        # evaluations *replaced* per second, not performed.
        for _ in range(2):
            pwlq.search_list(tl, wl.bits, wl.n_cand, workspace=ws_search, out=out, fast=True)
        torch.cuda.synchronize()
        pwlq.profile_enable(0xF)
        fast_ms, k_fast_ms = [], []
        for _ in range(reps):
            e0.record()
            pwlq.search_list(tl, wl.bits, wl.n_cand, workspace=ws_search, out=out, fast=True)
            e1.record()
            k_fast_ms.append(pwlq.profile_last_ms(2))
            e1.synchronize()
            fast_ms.append(e0.elapsed_time(e1))
        pwlq.profile_enable(0)
        result["search_fast"] = {
            "ms": float(np.mean(fast_ms)),
            "kernel": pwlq.last_search_kernel(),      # k_fast, or k_small for a call small enough for one fused launch
            "kernel_ms": float(np.mean(k_fast_ms)),
            "equivalent_evals_per_s": evals / (float(np.mean(fast_ms)) * 1e-3),
            "speedup_over_exhaustive_search": float(np.mean(search_ms)) / float(np.mean(fast_ms)),
        }

        # The paper's analytic breakpoint selectors on the same weights: time of one
        # model-level call and the error they reach relative to the exhaustive
        # optimum of the step above (both errors evaluated by pwlq_mse_list).
        ws_sel = torch.empty(max(256, pwlq.select_list_workspace_bytes(tl)), dtype=torch.uint8,
                             device="cuda")
        ws_mse = torch.empty(max(256, pwlq.mse_list_workspace_bytes(tl)), dtype=torch.uint8,
                             device="cuda")
        sel_out = (torch.empty(tl.n_groups, dtype=torch.float32, device="cuda"),
                   torch.empty(tl.n_groups, dtype=torch.float32, device="cuda"))
        mse_out = torch.empty(tl.n_groups, dtype=torch.float64, device="cuda")
        best = pwlq.mse_list(tl, wl.bits, out["p_star"], out["m"], workspace=ws_mse).clone()
        result["analytic_selectors"] = {}
        for name, sel in (("gauss_fit", pwlq.GAUSS_FIT), ("gauss_solve", pwlq.GAUSS_SOLVE),
                          ("laplace_solve", pwlq.LAPLACE_SOLVE)):
            for _ in range(2):
                pwlq.select_analytic_list(tl, sel, workspace=ws_sel, out=sel_out)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                pwlq.select_analytic_list(tl, sel, workspace=ws_sel, out=sel_out)
            e1.record()
            for _ in range(reps):
                pwlq.mse_list(tl, wl.bits, sel_out[0], sel_out[1], workspace=ws_mse, out=mse_out)
            e2.record()
            e2.synchronize()
            ok = (best > 0) & torch.isfinite(best) & torch.isfinite(mse_out)
            ratio = (mse_out[ok] / best[ok])
            result["analytic_selectors"][name] = {
                "select_ms": e0.elapsed_time(e1) / reps,
                "mse_ms": e1.elapsed_time(e2) / reps,
                "mse_over_grid_optimum_geomean": float(torch.exp(torch.log(ratio).mean())),
                "mse_over_grid_optimum_max": float(ratio.max()),
                "total_sse_over_grid_optimum": float(
                    (mse_out[ok] * tl.group_counts(ok)).sum() / (best[ok] * tl.group_counts(ok)).sum()),
            }

        # Consumer of the packed format (Section 4): int8 activations [4096, 4096]
        # times a PWLQ-quantized [4096, 4096] linear weight (b = 4, Laplacian values of
        # workload 5's kind) on the int8 matrix cores.  Timed in both forms: y alone
        # (two operand planes: the offset term rides in the first product) and y with
        # the three integer sums of Section 4 (three planes).  `achieved` counts the
        # multiply-adds the matrix cores execute (planes x M x N x K); `algorithmic`
        # counts one multiply-add per (row, channel, k).
        if not args.no_linear:
            Ml, Kl, Nl, bl = 4096, 4096, 4096, 4
            gen = torch.Generator(device="cuda").manual_seed(7)
            u01 = (torch.rand((Nl, Kl), generator=gen, device="cuda") - 0.5).clamp_(-0.4999999, 0.4999999)
            wlin = (-0.02 * torch.sign(u01) * torch.log1p(-2.0 * u01.abs())).contiguous()   # Laplace(0, 0.02)
            sl = pwlq.search(wlin, bl, 100, fast=True)
            pc, pf, _ = pwlq.quantize_packed(wlin, bl, sl["p_star"], sl["m"], want_w_hat=False)
            xq = torch.randint(-128, 128, (Ml, Kl), generator=gen, device="cuda", dtype=torch.int8)
            ws_lin = torch.empty(max(256, pwlq.lib.pwlq_linear_workspace_bytes(Nl)), dtype=torch.uint8,
                                 device="cuda")
            y_lin = torch.empty((Ml, Nl), dtype=torch.float32, device="cuda")
            sums_lin = torch.empty((3, Ml, Nl), dtype=torch.int32, device="cuda")
            ops = 2.0 * Ml * Nl * Kl

            def time_linear(lout, planes):
                for _ in range(2):
                    pwlq.linear_i8(xq, 0.02, -0.5, pc, pf, Nl, bl, sl["p_star"], sl["m"],
                                   workspace=ws_lin, out=lout)
                torch.cuda.synchronize()
                pwlq.profile_enable(0xF)
                lin_ms = []
                for _ in range(reps):
                    pwlq.linear_i8(xq, 0.02, -0.5, pc, pf, Nl, bl, sl["p_star"], sl["m"],
                                   workspace=ws_lin, out=lout)
                    lin_ms.append(pwlq.profile_last_ms(3))
                pwlq.profile_enable(0)
                lm = float(np.mean(lin_ms))
                return {
                    "planes": planes,
                    "kernel_ms": lm,
                    "achieved": planes * ops / (lm * 1e-3) / 1e12,
                    "algorithmic": ops / (lm * 1e-3) / 1e12,
                    "frac": planes * ops / (lm * 1e-3) / 5e15,
                    "algorithmic_frac": ops / (lm * 1e-3) / 5e15,
                }

            folded = time_linear((y_lin, None), 2)
            y_folded = y_lin.clone()
            apart = time_linear((y_lin, sums_lin), 3)
            result["linear_i8"] = {
                "kernel": pwlq.kernel_name(3),
                "shape": f"xq [{Ml},{Kl}] int8 x packed PWLQ weight [{Nl},{Kl}], b={bl}",
                "bound": "mfma",
                "peak": 5000.0,
                "unit": "TOP/s int8 (dense MFMA)",
                **folded,
                "with_the_three_sums": apart,
                "max_abs_difference_of_y_between_the_forms": float((y_folded - y_lin).abs().max()),
                "note": "frac counts the matrix products executed per weight (2: centre codes "
                        "with the offset term, tail codes; 3 when the sums are wanted apart: "
                        "centre codes, tail codes, tail signs); algorithmic_frac counts one "
                        "multiply-add per (row, channel, k)",
                "weight_bytes_per_element": (bl + 1) / 8.0,
            }

    def graph_leg():
        # The same step recorded once into a HIP graph and replayed (the calls only
        # launch kernels): what is left of the launch overhead, which is most of the
        # time of the one-tensor workload.
        keep = {k: v.clone() for k, v in out.items()}
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        nrep = max(20, min(200, int(200.0 / max(ms_per_step, 1e-3))))
        g0 = time.perf_counter()
        for _ in range(nrep):
            graph.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        result["graph_replay"] = {
            "ms_per_step": (g1 - g0) * 1e3 / nrep,
            "eager_ms_per_step": ms_per_step,
            "replays": nrep,
            "same_outputs_as_eager": bool(all(torch.equal(keep[k], out[k], ) or
                                              bool(torch.equal(torch.nan_to_num(keep[k].double()),
                                                               torch.nan_to_num(out[k].double())))
                                              for k in keep)),
        }


    if not args.no_graph:
        graph_leg()
    if not args.hot_path_only:
        extras()

    if not args.no_cpu_baseline:
        from oracle import pwlq_ref
        pwlq_ref.search(host[0][:2], wl.bits, 8, wl.mode)            # load the library
        if wl.mode == synth.PER_CHANNEL:
            # about 2.5e10 evaluations: a few seconds on the host cores of the GPU machine
            stride = max(1, int(round(evals / 2.6e10)))
            sample = [t[::stride] for t in host]
            what = (f"one channel in every {stride} of every tensor" if stride > 1
                    else "the whole workload")
        else:
            order = np.argsort([t.size for t in host])
            sample = [host[i] for i in order[: len(order) // 2]]
            what = "the smaller half of the tensors"
        c0 = time.perf_counter()
        n_eval_cpu = 0
        ref_k, ref_mse = [], []
        for t in sample:
            t = np.ascontiguousarray(t)
            r = pwlq_ref.search(t, wl.bits, wl.n_cand, wl.mode)
            ref_k.append(r["k_star"])
            ref_mse.append(r["mse"])
            n_eval_cpu += t.size * wl.n_cand
        c1 = time.perf_counter()
        # the same groups from the timed GPU steps, side by side with the oracle's (the
        # parity tests hold the tolerances; this only reports what the two runs gave)
        gk, gm = keep_search["k_star"].cpu().numpy(), keep_search["mse"].cpu().numpy()
        if wl.mode == synth.PER_CHANNEL:
            pick = np.concatenate([tl.group_offsets[i] + np.arange(0, host[i].shape[0], stride)
                                   for i in range(len(host))])
        else:
            pick = np.array([tl.group_offsets[int(i)] for i in order[: len(order) // 2]])
        rk, rm = np.concatenate(ref_k), np.concatenate(ref_mse)
        fin = rk > 0
        result["cpu_baseline"] = {
            "value": n_eval_cpu / (c1 - c0),
            "unit": "candidate-element evaluations/s",
            "cores": pwlq_ref.num_threads(),
            "kind": "oracle",
            "sample": f"search only, {what} ({n_eval_cpu:.3e} evaluations, {c1 - c0:.1f} s)",
            "agreement_with_gpu": {
                "groups": int(rk.size),
                "k_star_equal": int((gk[pick] == rk).sum()),
                "max_mse_rel_diff": float(np.max(np.abs(gm[pick][fin] - rm[fin]) /
                                                 np.where(rm[fin] > 0, rm[fin], 1.0), initial=0.0)),
            },
        }
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
