#!/usr/bin/env python3
"""Benchmark of the stage + activation-offload hot path on one MI355X.

A step is one po_run_schedule over all microbatches of the workload (every
forward, offload, reload and backward of the rank-local 1F1B schedule).  Inputs,
parameters and outputs are resident in HBM before the timed region; slab and
pinned-buffer pools are warm.  Prints ONE JSON line.

  value            stage tokens/s at offload ratio 1 (full offload), m*s / step time, on the headline workload (C2)
  ratios           tokens/s, ms/step, peak activation GB, resident units (measured, and the schedule model's in
                   cpu_baseline.schedule_model), overlap (exposed-copy and trace-based), host-link GB/s at ratios
                   0, 0.5, 1 and at "auto" = min(1, 1/k) with k from the measured transfer and compute times (Section 2)
  frontier         the same workload with a reload lead of one pass: the (lead, ratio) -> (peak GB, tokens/s) points
                   that trade throughput for memory where the default lead saves none (Section 2: selective offload
                   exists to cut peak memory)
  host_link        achieved D2H / H2D rate during the headline run against the link's peak per direction
  roofline         bf16 MFMA GEMM launches of the timed steps at ratio 0 (HIP events on the compute stream, recorded
                   by the library around every k-th GEMM launch, k = --profile-every) against 2.5 PFLOP/s;
  roofline_at_value_ratio   the same launches timed while the copies of the headline ratio run beside them
  k_le_1_workload  C5 (long context, Eq. 1's k below 1 on this machine) at ratio 0 and 1: the case in which full
                   offload is meant to be free (Section 1, below Eq. 1)
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
# PCIe 5.0 x16: 32 GT/s x 16 lanes x 128/130 encoding = 63.0 GB/s per direction before packet overhead.
HOST_LINK_PEAK_GB_PER_S = 63.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemm_hbm_traffic.txt")


def measured_gemm_traffic(workload):
    """HBM bytes per GEMM launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes (counters cannot be read
    from inside this script): the line of profiles/gemm_hbm_traffic.txt for the workload, written by
    `python -m paper_2503_01328_amd.profile_traffic`, with the commit it was measured at; None if not collected."""
    try:
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) >= 3 and f[0] == workload:
                return {"bytes_per_launch": int(f[1]), "measured_at_commit": f[2]}
    except OSError:
        pass
    return None


def model_flops_per_run(shape):
    """72 h^2 + 6 s h per token and layer (GEMMs forward + backward, causal attention), Eq. 1's T_c with the
    causal half of its attention term."""
    h, s = shape.hidden, shape.seq
    # QKV projection is h x (h + 2 hkv): 6 (1 + 2 hkv / h) h^2 instead of 18 h^2 of the 72 h^2
    qkv = 6.0 * h * (h + 2.0 * shape.kv_width)
    per_token_layer = 54.0 * h * h + qkv + 6.0 * s * h
    return per_token_layer * s * shape.n_layers * shape.n_microbatches


def gemm_algorithmic_bytes_per_launch(shape):
    """Bytes an average GEMM launch of a layer has to move at least (operands read once, results written once, the
    fp32 gradient accumulators read and written once): the nine launches of a layer and microbatch are the four
    forward products (the MLP's first one writes u and gelu(u), the two output projections read a residual), the
    four input-gradient products (the MLP's second one reads u and writes du and gelu(u)) and the grouped launch
    of the four weight-gradient products."""
    s, h, f, w = shape.seq, shape.hidden, shape.ffn, shape.hidden + 2 * shape.kv_width
    E = 2
    fwd = (s * h + h * w + s * w) * E + (s * h + h * h + 2 * s * h) * E + (s * h + h * f + 2 * s * f) * E + \
          (s * f + f * h + 2 * s * h) * E
    dgrad = (s * h + h * f + 3 * s * f) * E + (s * f + f * h + s * h) * E + (s * h + h * h + s * h) * E + \
            (s * w + w * h + s * h) * E
    weights = h * w + h * h + 2 * h * f
    wgrad = (s * f + s * h + s * h + s * f + 2 * s * h + s * h + s * w) * E + 2 * 4 * weights
    return (fwd + dgrad + wgrad) / 9.0


def cpu_baseline(shape, sched_name, select, ratios):
    """Times the oracle (float32 instantiation, as it stands) on one microbatch of the workload: as many of its
    layers as fit about 25 s at the 0.3 TFLOP/s the numpy oracle reaches on 16 cores (all 4 at C2, 1 at C3).
    The oracle's schedule model adds the number of units it expects resident at each measured (ratio, reload lead)."""
    import numpy as np

    from oracle import schedule_oracle as sch
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
    out = {"value": tokens_per_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
           "sample": f"1 microbatch x {n} of {shape.n_layers} layers (fp32 numpy oracle, forward+backward, "
                     f"{dt:.2f} s), scaled by the layer count"}
    # residency the schedule model expects (idealised: a copy takes no time, so the measured figures may hold one
    # unit more while a slab is in transit)
    if sched_name in ("1f1b", "1f1b-interleaved"):
        d, v, m = shape.pipeline_degree, shape.n_chunks, shape.n_microbatches
        passes = sch.one_f_one_b(d, 0, m) if sched_name == "1f1b" else sch.interleaved_one_f_one_b(d, 0, v, m)
        model = {}
        for label, (ratio, lead) in ratios.items():
            sel = sch.selected_units(m, v, ratio, select)
            r = sch.simulate(sch.with_offload(passes, sel, prefetch=lead))
            model[label] = {"ratio": ratio, "prefetch_passes": lead, "peak_resident_units": r["peak_resident"],
                            "peak_in_flight_units": r["peak_in_flight"]}
        out["schedule_model"] = model
    return out


def measure_ratios(po, torch, runner, shape, sched, ratio_list, steps, warmup, profile_every, auto_ratio):
    """Times `steps` runs of the schedule at every ratio of ratio_list (and at the "auto" ratio); returns
    {ratio or "auto": figures}."""
    tokens = shape.n_microbatches * shape.seq

    def measure(ratio):
        for _ in range(warmup):
            runner.run(sched, ratio)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        per = []
        for _ in range(steps):
            per.append(runner.run(sched, ratio))
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        agg = {k: sum(p[k] for p in per) / len(per) for k in
               ("compute_busy_s", "d2h_busy_s", "h2d_busy_s", "gemm_busy_s", "gemm_flops", "attn_busy_s",
                "attn_flops", "pack_busy_s", "copy_hidden_s")}
        last = per[-1]
        return dict(
            tokens_per_s=tokens / dt, ms_per_step=dt * 1e3, steps=steps,
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
            gemm_busy_ms=agg["gemm_busy_s"] * 1e3 * profile_every,  # timed sample scaled to all launches
            n_gemm_launches_timed=last["n_gemm_launches"],
            attn_tflops=agg["attn_flops"] / agg["attn_busy_s"] / 1e12 if agg["attn_busy_s"] else None,
            attn_busy_ms=agg["attn_busy_s"] * 1e3 * profile_every,
            mfu=model_flops_per_run(shape) / dt / (PEAK_BF16_TFLOPS * 1e12),
        )

    ratios = {}
    for ratio in ratio_list:
        ratios[ratio] = measure(ratio)
    top = max(ratios)
    if auto_ratio and top > 0.0:
        # Largest ratio whose transfers should still hide: k measured as the busier copy direction at the top
        # ratio over the step time at ratio 0 (both directions run at once on this machine), ratio = min(1, 1 / k).
        one = ratios[top]
        busy = [b for b in ((one["d2h_busy_ms"], one["h2d_busy_ms"])) if b]
        k_transfer = (max(busy) / ratios[0.0]["ms_per_step"]) if busy else None
        if k_transfer:
            auto = po.po_offload_ratio_for_k(k_transfer)
            ratios["auto"] = dict(ratios[top]) if auto >= 1.0 else measure(auto)
            ratios["auto"]["ratio"] = auto
            ratios["auto"]["k_transfer_measured"] = k_transfer
    if 0.0 in ratios:
        base = ratios[0.0]["ms_per_step"]
        for ratio, d in ratios.items():
            if ratio != 0.0 and d["copy_busy_ms"] > 0:
                d["overlap"] = max(0.0, min(1.0, 1.0 - (d["ms_per_step"] - base) / d["copy_busy_ms"]))
            else:
                d["overlap"] = None
            d["throughput_vs_no_offload"] = base / d["ms_per_step"]
    return ratios


def workload_text(name, shape, sched_name, group):
    kv = " (%d key/value heads)" % shape.n_kv_heads if shape.n_kv_heads else ""
    return (f"{name}: GPT stage, {shape.n_layers} layers, hidden {shape.hidden}, {shape.n_heads} heads{kv}, "
            f"FFN {shape.ffn}, seq {shape.seq}, {shape.n_microbatches} microbatches, simulated pipeline degree "
            f"{shape.pipeline_degree}, schedule {sched_name}{' g=%d' % group if group else ''} rank 0")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C2", help="workload: C1..C5 (default C2, the configuration the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-auto-ratio", action="store_true",
                    help="skip the extra measurement at the ratio min(1, 1/k) derived from the measured transfer times")
    ap.add_argument("--no-frontier", action="store_true",
                    help="skip the second pass over the workload with a reload lead of one pass")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the k <= 1 workload (C5 at ratio 0 and 1) that the default run adds to the line")
    ap.add_argument("--secondary-steps", type=int, default=2, help="timed steps per ratio of the k <= 1 workload")
    ap.add_argument("--copy-streams", type=int, default=2)
    ap.add_argument("--prefetch", type=int, default=2)
    ap.add_argument("--staged", type=int, default=0)
    ap.add_argument("--schedule", default="auto", choices=["auto", "1f1b", "1f1b-interleaved", "gis", "po"],
                    help="auto: 1F1B, or interleaved 1F1B for a workload with several chunks; gis: generalized "
                         "interleaved schedule with split backward (Sections 3.1, 3.2); po: the uniformly repeated "
                         "schedule (Section 2, Table 1), which selects whole chunks by lifespan")
    ap.add_argument("--profile-every", type=int, default=25,
                    help="bracket every k-th GEMM / attention launch of the timed steps with HIP events (1 = all; an "
                         "event pair idles the stream for a few microseconds; k = 25 keeps that below half a percent of "
                         "the C2 step, still times over a hundred GEMM launches in ten steps and, being coprime to the "
                         "launches of a layer, all of their shapes)")
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
    scheds = {"1f1b": po.PO_SCHED_1F1B, "1f1b-interleaved": po.PO_SCHED_1F1B_INTERLEAVED,
              "gis": po.PO_SCHED_GIS, "po": po.PO_SCHED_PO}
    sched = scheds[sched_name]
    select = args.select if args.select != "auto" else ("longest-lifespan" if sched_name == "po" else "alternate-mb")
    policy = {"alternate-mb": po.PO_SEL_ALTERNATE_MB, "longest-lifespan": po.PO_SEL_LONGEST_LIFESPAN}[select]
    common = dict(device_params=True, copy_streams=args.copy_streams, staged_copies=args.staged,
                  profile_kernels=args.profile_every, group=args.group, weight_stream=args.weight_stream,
                  dropout_p=args.dropout, dropout_seed=20250301, select_policy=policy, slot_k=args.slot_k)
    ratio_list = (0.0,) if args.only_ratio_0 else (0.0, 0.5, 1.0)

    with StageRunner(shape, prefetch_passes=args.prefetch, **common) as r:
        r.make_inputs_on_device()
        ratios = measure_ratios(po, torch, r, shape, sched, ratio_list, args.steps, args.warmup, args.profile_every,
                                not args.no_auto_ratio)
    top = max(k for k in ratios if k != "auto")  # 1.0 unless --only-ratio-0
    headline = ratios[top]

    frontier = None
    if not args.only_ratio_0 and not args.no_frontier and args.prefetch != 1:
        # the same workload with the reload issued one pass ahead of the backward instead of args.prefetch
        with StageRunner(shape, prefetch_passes=1, **common) as r:
            r.make_inputs_on_device()
            fr = measure_ratios(po, torch, r, shape, sched, (0.0, 0.5, 1.0), max(3, args.steps // 2), 2,
                                args.profile_every, False)
        keep = ("tokens_per_s", "ms_per_step", "steps", "peak_activation_gb", "peak_resident_units",
                "throughput_vs_no_offload", "d2h_gb_per_s", "h2d_gb_per_s")
        frontier = {"prefetch_passes": 1, "ratios": {str(k): {f: v[f] for f in keep} for k, v in fr.items() if k != 0.0}}

    secondary = None
    if (not args.only_ratio_0 and not args.no_secondary and args.config == "C2" and sched_name == "1f1b"
            and not args.kv_heads and not args.dropout):
        # the workload whose transfers fit under its compute on this machine (k <= 1): full offload should be free
        name2 = "C5"
        shape2 = syn.CONFIGS[name2]
        with StageRunner(shape2, prefetch_passes=args.prefetch, **common) as r:
            r.make_inputs_on_device()
            r2 = measure_ratios(po, torch, r, shape2, po.PO_SCHED_1F1B, (0.0, 1.0), args.secondary_steps, 1,
                                args.profile_every, False)
        bc2 = model_flops_per_run(shape2) / (r2[0.0]["ms_per_step"] * 1e-3)
        bo2 = (r2[1.0]["d2h_gb_per_s"] or 0) * 1e9
        keep = ("tokens_per_s", "ms_per_step", "steps", "peak_activation_gb", "peak_resident_units",
                "peak_in_flight_units", "throughput_vs_no_offload", "overlap", "overlap_trace", "d2h_gb_per_s",
                "h2d_gb_per_s", "gemm_tflops", "attn_tflops", "mfu")
        secondary = {
            "workload": workload_text(name2, shape2, "1f1b", 0),
            "warmup": 1, "prefetch_passes": args.prefetch,
            "k_eq1_measured_duplex": (po.po_offload_k(shape2.hidden, shape2.seq, bc2, bo2) / 2) if bo2 else None,
            "ratios": {str(k): {f: v.get(f) for f in keep} for k, v in r2.items()},
            "throughput_vs_no_offload_at_full_offload": r2[1.0]["throughput_vs_no_offload"],
        }

    # Eq. 1 with measured rates: compute rate = model flops / compute time at ratio 0, link rate = measured D2H
    bc = model_flops_per_run(shape) / (ratios[0.0]["ms_per_step"] * 1e-3)
    bo = (headline["d2h_gb_per_s"] or 0) * 1e9
    k_meas = po.po_offload_k(shape.hidden, shape.seq, bc, bo) if bo else None
    dtype = "bf16" if shape.dtype == "bf16" else "f32"
    peak_tflops = PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_F32_VECTOR_TFLOPS
    traffic = measured_gemm_traffic(args.config)
    kernel_text = ((f"gemm_mfma_kernel and its grouped form (every {args.profile_every}-th GEMM launch of the timed "
                    f"steps, which walks through all 9 launches of a layer, the four weight-gradient products being "
                    f"one: sum of 2MNK flops / sum of event-timed durations)") if dtype == "bf16" else
                   (f"gemm_generic_kernel, fp32 (every {args.profile_every}-th GEMM launch of the timed steps: sum of "
                    f"2MNK flops / sum of event-timed durations)"))

    def roofline_of(d, at_ratio):
        return {"bound": "mfma" if dtype == "bf16" else "alu", "achieved": d["gemm_tflops"], "peak": peak_tflops,
                "unit": "TFLOP/s", "frac": (d["gemm_tflops"] / peak_tflops) if d["gemm_tflops"] else None,
                "traffic": traffic["bytes_per_launch"] if traffic else None,
                "algorithmic_bytes_per_launch": gemm_algorithmic_bytes_per_launch(shape),
                "traffic_measured_at_commit": traffic["measured_at_commit"] if traffic else None,
                "kernel": kernel_text, "offload_ratio": at_ratio,
                "launches_timed_per_step": d["n_gemm_launches_timed"],
                "busy_ms_per_step_estimate": d["gemm_busy_ms"]}

    def link_of(rate):
        return {"achieved_gb_per_s": rate, "frac": (rate / HOST_LINK_PEAK_GB_PER_S) if rate else None}

    out = {
        "metric": "stage tokens/sec at offload ratio 0/0.5/1; peak activation HBM GB; overlap %",
        "value": headline["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": headline["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": workload_text(args.config, shape, sched_name, args.group) +
                               f"; value is at offload ratio {top:g}",
                   "copy_streams": args.copy_streams, "prefetch_passes": args.prefetch, "staged_copies": args.staged,
                   "weight_stream": args.weight_stream, "dropout": args.dropout, "select": select,
                   "slot_k": args.slot_k},
        "ratios": {str(k): v for k, v in ratios.items()},
        "frontier": frontier,
        "k_eq1_measured_serial": k_meas, "k_eq1_measured_duplex": (k_meas / 2 if k_meas else None),
        "host_link": {"peak_gb_per_s_per_direction": HOST_LINK_PEAK_GB_PER_S,
                      "peak_source": "PCIe 5.0 x16: 32 GT/s x 16 lanes x 128/130, before packet overhead",
                      "offload_ratio": top, "both_directions_busy": args.copy_streams == 2,
                      "d2h": link_of(headline["d2h_gb_per_s"]), "h2d": link_of(headline["h2d_gb_per_s"])},
        # bf16 workloads: the matrix-core GEMM against the dense bf16 MFMA peak.  The fp32 debug workload (C1) runs the
        # shape-generic fp32 kernel, plain vector arithmetic, priced against the fp32 vector peak.
        "roofline": roofline_of(ratios[0.0], 0.0),
        "roofline_at_value_ratio": roofline_of(headline, top) if top != 0.0 else None,
        "k_le_1_workload": secondary,
    }
    if not args.no_cpu_baseline:
        model_ratios = {str(k): ((v["ratio"] if k == "auto" else k), args.prefetch) for k, v in ratios.items()}
        if frontier:
            for k in frontier["ratios"]:
                model_ratios[f"lead1_{k}"] = (float(k), 1)
        out["cpu_baseline"] = cpu_baseline(shape, sched_name, select, model_ratios)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
