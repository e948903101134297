"""Per-kernel micro-benchmarks of the stage's building blocks at a workload's shapes.

    python -m paper_2503_01328_amd.microbench --config C3

Prints one line per kernel: algorithmic bytes or flops per launch, average launch time (HIP events on
the launch stream, inputs resident), achieved rate and the fraction of the bounding roofline
(HBM 8 TB/s, bf16 MFMA 2.5 PFLOP/s, and the measured host link for copies).
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as po
from . import inputs as syn

HBM_PEAK = 8.0e12
MFMA_PEAK = 2.5e15


def _time(fn, iters=20, warm=3):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / iters


def run(config: str, iters: int = 20):
    shape = syn.CONFIGS[config]
    dev = torch.device("cuda:0")
    s, h, f, a = shape.seq, shape.hidden, shape.ffn, shape.n_heads
    bf = torch.bfloat16
    E = 2
    rows = []

    def add(name, bound, work, secs, peak):
        rate = work / secs
        rows.append(dict(kernel=name, bound=bound, work=work, us=secs * 1e6, rate=rate, frac=rate / peak))

    g = torch.Generator(device=dev)
    g.manual_seed(1)
    rn = lambda *sz: torch.randn(*sz, device=dev, generator=g).to(bf)

    # LayerNorm forward / backward
    x, gain, shift, y = rn(s, h), rn(h), rn(h), torch.empty(s, h, device=dev, dtype=bf)
    t = _time(lambda: po.po_op_layernorm_forward(po.PO_BF16, x, gain, shift, y, s, h, 1e-5), iters)
    add("layernorm forward [s,h]", "hbm", 2 * s * h * E, t, HBM_PEAK)
    dn, dres, dx = rn(s, h), rn(s, h), torch.empty(s, h, device=dev, dtype=bf)
    dg, db = torch.zeros(h, device=dev), torch.zeros(h, device=dev)
    ws = torch.empty(po.po_op_layernorm_backward_workspace(s, h) // 4, device=dev)
    t = _time(lambda: po.po_op_layernorm_backward(po.PO_BF16, dn, x, gain, dres, dx, dg, db, ws, s, h, 1e-5), iters)
    add("layernorm backward [s,h] (dn, x, dres -> dx, dgain, dshift)", "hbm", 4 * s * h * E, t, HBM_PEAK)
    # bias gradient
    du = rn(s, f)
    acc = torch.zeros(f, device=dev)
    ws2 = torch.empty(po.po_op_colsum_workspace(s, f) // 4, device=dev)
    t = _time(lambda: po.po_op_colsum_accumulate(po.PO_BF16, du, acc, ws2, s, f), iters)
    add("column sums [s,f] (bias gradient)", "hbm", s * f * E, t, HBM_PEAK)
    # hidden dropout with a regenerated mask: out = residual + dropout(x)
    xo = torch.empty(s, h, device=dev, dtype=bf)
    t = _time(lambda: po.po_op_dropout(po.PO_BF16, dn, xo, s, h, 0.1, 1234, 0, 0, 0), iters)
    add("dropout [s,h] (Philox mask regenerated, x -> out)", "hbm", 2 * s * h * E, t, HBM_PEAK)
    # pack / unpack of one layer's saved set
    sizes = [s * h * E, s * 3 * h * E, s * h * E, s * h * E, s * f * E, a * s * 4]
    segs = [torch.empty(n, dtype=torch.uint8, device=dev) for n in sizes]
    packed = torch.empty(sum(sizes), dtype=torch.uint8, device=dev)
    seglist = [(t_, n) for t_, n in zip(segs, sizes)]
    t = _time(lambda: po.po_op_pack(seglist, packed), iters)
    add("pack one layer's saved set", "hbm", 2 * sum(sizes), t, HBM_PEAK)
    t = _time(lambda: po.po_op_unpack(seglist, packed), iters)
    add("unpack one layer's saved set", "hbm", 2 * sum(sizes), t, HBM_PEAK)
    del segs, packed
    # GEMMs of one layer
    gemms = {
        "gemm qkv forward": (0, 0, s, 3 * h, h, "out"), "gemm out-proj forward": (0, 0, s, h, h, "out"),
        "gemm fc1 forward (+gelu)": (0, 0, s, f, h, "gelu"), "gemm fc2 forward": (0, 0, s, h, f, "out"),
        "gemm fc2 dgrad (+gelu bwd)": (0, 1, s, f, h, "gelu_bwd"), "gemm fc1 dgrad": (0, 1, s, h, f, "out"),
        "gemm qkv dgrad": (0, 1, s, h, 3 * h, "out"), "gemm out-proj dgrad": (0, 1, s, h, h, "out"),
        "gemm fc2 wgrad": (1, 0, f, h, s, "acc"), "gemm fc1 wgrad": (1, 0, h, f, s, "acc"),
        "gemm qkv wgrad": (1, 0, h, 3 * h, s, "acc"), "gemm out-proj wgrad": (1, 0, h, h, s, "acc"),
    }
    for name, (ta, tb, M, N, K, kind) in gemms.items():
        A = rn(K, M) if ta else rn(M, K)
        B = rn(N, K) if tb else rn(K, N)
        kw = {}
        if kind == "acc":
            kw["acc_f32"] = torch.zeros(M, N, device=dev)
        else:
            kw["out"] = torch.empty(M, N, device=dev, dtype=bf)
            if kind == "gelu":
                kw["gelu_out"] = torch.empty(M, N, device=dev, dtype=bf)
            if kind == "gelu_bwd":
                kw["gelu_out"] = torch.empty(M, N, device=dev, dtype=bf)
                kw["gelu_u"] = rn(M, N)
        t = _time(lambda: po.po_op_gemm(po.PO_BF16, ta, tb, M, N, K, A, A.shape[1], B, B.shape[1], **kw), iters)
        add(f"{name} M={M} N={N} K={K}", "mfma", 2.0 * M * N * K, t, MFMA_PEAK)
        del A, B, kw
    # the four weight-gradient products of a layer as one grouped launch (what the stage runs)
    probs = []
    for M, N in ((f, h), (h, f), (h, h), (h, 3 * h)):
        probs.append((M, N, s, rn(s, M), M, rn(s, N), N, torch.zeros(M, N, device=dev), N))
    t = _time(lambda: po.po_op_gemm_grouped(probs), iters)
    add("gemm wgrad, four products in one grouped launch", "mfma", sum(2.0 * p[0] * p[1] * p[2] for p in probs), t,
        MFMA_PEAK)
    del probs
    # attention
    qkv, d_o = rn(s, 3 * h), rn(s, h)
    o = torch.empty(s, h, device=dev, dtype=bf)
    lse = torch.empty(a, s, device=dev)
    dqkv = torch.empty(s, 3 * h, device=dev, dtype=bf)
    delta = torch.empty(a, s, device=dev)
    t = _time(lambda: po.po_op_attention_forward(po.PO_BF16, qkv, o, lse, s, h, a), iters)
    add("attention forward (causal model flops 2 s^2 h)", "mfma", 2.0 * s * s * h, t, MFMA_PEAK)
    t = _time(lambda: po.po_op_attention_backward(po.PO_BF16, qkv, o, lse, d_o, dqkv, delta, s, h, a), iters)
    add("attention backward (causal model flops 4 s^2 h)", "mfma", 4.0 * s * s * h, t, MFMA_PEAK)
    # host link: one layer slab each way (both directions at once are measured inside the stage: bench.py)
    nbytes = sum(sizes)
    host_a = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    host_b = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    dev_a = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    dev_b = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def d2h():
        host_a.copy_(dev_a, non_blocking=True)

    def h2d():
        dev_b.copy_(host_b, non_blocking=True)

    t = _time(d2h, 5, 1)
    link = nbytes / t
    add("D2H copy of one layer slab (pinned)", "link", nbytes, t, link)
    t = _time(h2d, 5, 1)
    add("H2D copy of one layer slab (pinned)", "link", nbytes, t, nbytes / t)

    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C3")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    rows = run(args.config, args.iters)
    if args.json:
        print(json.dumps(rows))
        return
    print(f"workload {args.config}")
    for r in rows:
        unit = {"hbm": "GB/s", "mfma": "TFLOP/s", "link": "GB/s"}[r["bound"]]
        div = 1e12 if r["bound"] == "mfma" else 1e9
        frac = "" if r["bound"] == "link" else f"{100 * r['frac']:5.1f} % of {'8 TB/s' if r['bound'] == 'hbm' else '2.5 PFLOP/s'}"
        print(f"{r['kernel']:62s} {r['us']:10.1f} us {r['rate'] / div:9.1f} {unit:8s} {frac}")


if __name__ == "__main__":
    main()
