#!/usr/bin/env python3
"""Benchmark of the stage + activation-offload hot path on one MI355X.

A step is one po_run_schedule over all microbatches of the workload (every
forward, offload, reload and backward of the rank-local 1F1B schedule).  Inputs,
parameters and outputs are resident in HBM before the timed region; slab and
pinned-buffer pools are warm.  Prints ONE JSON line.

  value            stage tokens/s at offload ratio 1 (full offload), m*s / step time
  ratios           tokens/s, ms/step, peak activation GB, overlap (exposed-copy and trace-based), host-link GB/s at ratios 0, 0.5, 1 and at
                   "auto" = min(1, 1/k) with k from the measured transfer and compute times (Section 2)
  roofline         bf16 MFMA GEMM launches of the timed steps (HIP events on the compute stream,
                   recorded by the library around every k-th GEMM launch, k = --profile-every) against 2.5 PFLOP/s
  cpu_baseline     the numpy oracle timed on a bounded sample of the same workload
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0
PEAK_F32_VECTOR_TFLOPS = 157.3
# HBM bytes per GEMM launch (average over all bf16 GEMM launches of a step) from the rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE passes summarised in profiles/hbm_traffic_c2.md, scaled by the copy-kernel calibration given there.
# Counters cannot be read inside this script, so the figure is carried here per workload; None = not collected.
MEASURED_GEMM_TRAFFIC_BYTES = {"C2": 210026173}


def model_flops_per_run(shape):
    """72 h^2 + 6 s h per token and layer (GEMMs forward + backward, causal attention), Eq. 1's T_c with the
    causal half of its attention term."""
    h, s = shape.hidden, shape.seq
    # QKV projection is h x (h + 2 hkv): 6 (1 + 2 hkv / h) h^2 instead of 18 h^2 of the 72 h^2
    qkv = 6.0 * h * (h + 2.0 * shape.kv_width)
    per_token_layer = 54.0 * h * h + qkv + 6.0 * s * h
    return per_token_layer * s * shape.n_layers * shape.n_microbatches


def cpu_baseline(shape):
    """Times the oracle (float32 instantiation, as it stands) on one microbatch of the workload: as many of its
    layers as fit about 25 s at the 0.3 TFLOP/s the numpy oracle reaches on 16 cores (all 4 at C2, 1 at C3)."""
    import numpy as np

    from oracle import stage_oracle as so
    from paper_2503_01328_amd import inputs as syn

    flops_per_layer = model_flops_per_run(shape) / (shape.n_layers * shape.n_microbatches)
    n = max(1, min(shape.n_layers, int(25.0 * 0.3e12 / flops_per_layer)))
    part = dataclasses.replace(shape, n_layers=n, n_chunks=1, vocab=0)
    params = syn.stage_params(part, 1234)
    x = {(0, 0): syn.unit_input(part, 0, 0)}
    dy = {(0, 0): syn.unit_upstream_grad(part, 0, 0)}
    t0 = time.perf_counter()
    so.run_stage(params, n, 1, part.n_heads, x, dy, dtype=np.float32)
    dt = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp and omp.isdigit():
        cores = min(cores, int(omp))
    tokens_per_s = shape.seq / (dt * shape.n_layers / n)
    return {"value": tokens_per_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"1 microbatch x {n} of {shape.n_layers} layers (fp32 numpy oracle, forward+backward, "
                      f"{dt:.2f} s), scaled by the layer count"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C2", help="workload: C1..C5 (default C2, the configuration the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-auto-ratio", action="store_true",
                    help="skip the extra measurement at the ratio min(1, 1/k) derived from the measured transfer times")
    ap.add_argument("--copy-streams", type=int, default=2)
    ap.add_argument("--prefetch", type=int, default=2)
    ap.add_argument("--staged", type=int, default=0)
    ap.add_argument("--schedule", default="auto", choices=["auto", "1f1b", "1f1b-interleaved", "gis", "po"],
                    help="auto: 1F1B, or interleaved 1F1B for a workload with several chunks; gis: generalized "
                         "interleaved schedule with split backward (Sections 3.1, 3.2); po: the uniformly repeated "
                         "schedule (Section 2, Table 1), which selects whole chunks by lifespan")
    ap.add_argument("--profile-every", type=int, default=5,
                    help="bracket every k-th GEMM / attention launch of the timed steps with HIP events (1 = all; an "
                         "event pair idles the stream for a few microseconds, which costs about 7 %% at C2 with k = 1)")
    ap.add_argument("--weight-stream", type=int, default=0, help="1: weight-gradient work on its own stream")
    ap.add_argument("--kv-heads", type=int, default=0,
                    help="grouped-query attention with this many key/value heads (Table 2 uses 8); 0 = multi-head")
    ap.add_argument("--dropout", type=float, default=0.0, help="hidden dropout probability (masks regenerated in backward)")
    ap.add_argument("--slot-k", type=float, default=0.0,
                    help="with --schedule po: place the copies into the slots of Section 4.2 for this k (a unit's "
                         "round trip over its F + B + W time) instead of the prefetch rule; 0 = prefetch rule")
    ap.add_argument("--only-ratio-0", action="store_true",
                    help="measure ratio 0 only (for a kernel profile of the compute path without copy kernels beside "
                         "it); value is then the tokens/s at ratio 0 and the workload string says so")
    ap.add_argument("--group", type=int, default=0,
                    help="group size g of --schedule gis (0 = pipeline degree) or po (0 = half the pipeline degree)")
    ap.add_argument("--select", default="auto", choices=["auto", "alternate-mb", "longest-lifespan"],
                    help="how a ratio picks units: every other microbatch, or the longest-lived chunks of every "
                         "microbatch (auto: the latter for --schedule po)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline rank on one GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2503_01328_amd import binding as po
    from paper_2503_01328_amd import inputs as syn
    from paper_2503_01328_amd.harness import StageRunner

    shape = syn.CONFIGS[args.config]
    if args.kv_heads:
        shape = dataclasses.replace(shape, n_kv_heads=args.kv_heads)
    sched_name = args.schedule
    if sched_name == "auto":
        sched_name = "1f1b-interleaved" if shape.n_chunks > 1 else "1f1b"
    sched = {"1f1b": po.PO_SCHED_1F1B, "1f1b-interleaved": po.PO_SCHED_1F1B_INTERLEAVED,
             "gis": po.PO_SCHED_GIS, "po": po.PO_SCHED_PO}[sched_name]
    select = args.select if args.select != "auto" else ("longest-lifespan" if sched_name == "po" else "alternate-mb")
    policy = {"alternate-mb": po.PO_SEL_ALTERNATE_MB, "longest-lifespan": po.PO_SEL_LONGEST_LIFESPAN}[select]
    tokens = shape.n_microbatches * shape.seq
    ratios = {}
    headline = None
    with StageRunner(shape, device_params=True, copy_streams=args.copy_streams, prefetch_passes=args.prefetch,
                     staged_copies=args.staged, profile_kernels=args.profile_every, group=args.group,
                     weight_stream=args.weight_stream, dropout_p=args.dropout, dropout_seed=20250301,
                     select_policy=policy, slot_k=args.slot_k) as r:
        r.make_inputs_on_device()
        def measure(ratio):
            for _ in range(args.warmup):
                r.run(sched, ratio)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            per = []
            for _ in range(args.steps):
                per.append(r.run(sched, ratio))
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / args.steps
            agg = {k: sum(p[k] for p in per) / len(per) for k in
                   ("compute_busy_s", "d2h_busy_s", "h2d_busy_s", "gemm_busy_s", "gemm_flops", "attn_busy_s",
                    "attn_flops", "pack_busy_s", "copy_hidden_s")}
            last = per[-1]
            return dict(
                tokens_per_s=tokens / dt, ms_per_step=dt * 1e3,
                peak_activation_gb=last["peak_slab_bytes"] / 1e9,
                peak_resident_units=last["peak_resident_units"], peak_in_flight_units=last["peak_in_flight_units"],
                d2h_gb_per_s=(last["bytes_d2h"] / agg["d2h_busy_s"] / 1e9) if agg["d2h_busy_s"] else None,
                h2d_gb_per_s=(last["bytes_h2d"] / agg["h2d_busy_s"] / 1e9) if agg["h2d_busy_s"] else None,
                copy_busy_ms=(agg["d2h_busy_s"] + agg["h2d_busy_s"]) * 1e3,
                d2h_busy_ms=agg["d2h_busy_s"] * 1e3, h2d_busy_ms=agg["h2d_busy_s"] * 1e3,
                compute_busy_ms=agg["compute_busy_s"] * 1e3,
                # trace-based overlap: share of the copy-busy time during which a compute pass was running too
                overlap_trace=(agg["copy_hidden_s"] / (agg["d2h_busy_s"] + agg["h2d_busy_s"]))
                if (agg["d2h_busy_s"] + agg["h2d_busy_s"]) > 0 else None,
                gemm_tflops=agg["gemm_flops"] / agg["gemm_busy_s"] / 1e12 if agg["gemm_busy_s"] else None,
                gemm_busy_ms=agg["gemm_busy_s"] * 1e3 * args.profile_every,  # timed sample scaled to all launches
                n_gemm_launches_timed=last["n_gemm_launches"],
                attn_tflops=agg["attn_flops"] / agg["attn_busy_s"] / 1e12 if agg["attn_busy_s"] else None,
                attn_busy_ms=agg["attn_busy_s"] * 1e3 * args.profile_every,
                mfu=model_flops_per_run(shape) / dt / (PEAK_BF16_TFLOPS * 1e12),
            )
        for ratio in ((0.0,) if args.only_ratio_0 else (0.0, 0.5, 1.0)):
            ratios[ratio] = measure(ratio)
        top = max(ratios)  # 1.0 unless --only-ratio-0
        # Largest ratio whose transfers should still hide: k measured as the busier copy direction at ratio 1 over
        # the step time at ratio 0 (both directions run at once on this machine), ratio = min(1, 1 / k).
        one = ratios[top]
        busy = [b for b in ((one["d2h_busy_ms"], one["h2d_busy_ms"])) if b]
        k_transfer = (max(busy) / ratios[0.0]["ms_per_step"]) if busy else None
        if k_transfer and not args.no_auto_ratio:
            auto = po.po_offload_ratio_for_k(k_transfer)
            ratios["auto"] = dict(ratios[top]) if auto >= 1.0 else measure(auto)
            ratios["auto"]["ratio"] = auto
            ratios["auto"]["k_transfer_measured"] = k_transfer
        base = ratios[0.0]["ms_per_step"]
        for ratio, d in ratios.items():
            if ratio != 0.0 and d["copy_busy_ms"] > 0:
                d["overlap"] = max(0.0, min(1.0, 1.0 - (d["ms_per_step"] - base) / d["copy_busy_ms"]))
            else:
                d["overlap"] = None
            d["throughput_vs_no_offload"] = base / d["ms_per_step"]
        headline = ratios[top]
        # Eq. 1 with measured rates: compute rate = model flops / compute time at ratio 0, link rate = measured D2H
        bc = model_flops_per_run(shape) / (ratios[0.0]["ms_per_step"] * 1e-3)
        bo = (headline["d2h_gb_per_s"] or 0) * 1e9
        k_meas = po.po_offload_k(shape.hidden, shape.seq, bc, bo) if bo else None
        gemm = ratios[0.0]
        dtype = "bf16" if shape.dtype == "bf16" else "f32"
        peak_tflops = PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_F32_VECTOR_TFLOPS

    out = {
        "metric": "stage tokens/sec at offload ratio 0/0.5/1; peak activation HBM GB; overlap %",
        "value": headline["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": headline["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{args.config}: GPT stage, {shape.n_layers} layers, hidden {shape.hidden}, "
                               f"{shape.n_heads} heads{' (%d key/value heads)' % shape.n_kv_heads if shape.n_kv_heads else ''}, FFN {shape.ffn}, seq {shape.seq}, {shape.n_microbatches} "
                               f"microbatches, simulated pipeline degree {shape.pipeline_degree}, "
                               f"schedule {sched_name}{' g=%d' % args.group if args.group else ''} rank 0; "
                               f"value is at offload ratio {top:g}",
                   "copy_streams": args.copy_streams, "prefetch_passes": args.prefetch, "staged_copies": args.staged,
                   "weight_stream": args.weight_stream, "dropout": args.dropout, "select": select,
                   "slot_k": args.slot_k},
        "ratios": {str(k): v for k, v in ratios.items()},
        "k_eq1_measured_serial": k_meas, "k_eq1_measured_duplex": (k_meas / 2 if k_meas else None),
        # bf16 workloads: the matrix-core GEMM against the dense bf16 MFMA peak.  The fp32 debug workload (C1) runs the
        # shape-generic fp32 kernel, plain vector arithmetic, priced against the fp32 vector peak.
        "roofline": {"bound": "mfma" if dtype == "bf16" else "alu", "achieved": gemm["gemm_tflops"],
                     "peak": peak_tflops, "unit": "TFLOP/s",
                     "frac": (gemm["gemm_tflops"] / peak_tflops) if gemm["gemm_tflops"] else None,
                     "traffic": MEASURED_GEMM_TRAFFIC_BYTES.get(args.config),
                     "kernel": (f"gemm_mfma_kernel and its grouped form (every {args.profile_every}-th GEMM launch of "
                                f"the timed steps at ratio 0, which walks through all 9 launches of a layer, the "
                                f"four weight-gradient products being one: sum of 2MNK flops / sum of event-timed "
                                f"durations)") if dtype == "bf16" else
                               (f"gemm_generic_kernel, fp32 (every {args.profile_every}-th GEMM launch of the timed "
                                f"steps at ratio 0: sum of 2MNK flops / sum of event-timed durations)"),
                     "launches_timed_per_step": gemm["n_gemm_launches_timed"],
                     "busy_ms_per_step_estimate": gemm["gemm_busy_ms"]},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
