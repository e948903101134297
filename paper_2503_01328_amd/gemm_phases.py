"""Where a block of the bf16 matrix-core GEMM spends its time: prologue (first operand slices on their way), main
loop, epilogue, from the device's cycle counter in a measurement build of the kernel (-DPO_PHASE_TIMING, a library of
its own under _build/; the product library is not touched).

    python -m paper_2503_01328_amd.gemm_phases --build     # here, hipcc cross-compiles
    python -m paper_2503_01328_amd.gemm_phases             # on the MI355X

Per shape: the launch's duration (average of ten back-to-back launches between two events) and, for the block of tile
(0, 0), the three phases in microseconds, the main loop's cycles per 64-deep K slice against the MFMA issue time of that
slice (64 MFMAs of 32 cycles per wave for the 256 x 256 tile, 48 for 256 x 192, 16 for 128 x 128), and the clock the block ran at
(cycle counter over the constant 100 MHz counter).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import sys

from . import build as b

LIB = os.path.join(b.OBJ, "libpipeoffload_phases.so")


def build_variant() -> str:
    os.makedirs(b.OBJ, exist_ok=True)
    flags = [f for f in b.FLAGS if not f.startswith("-Rpass")]
    objs = []
    for src in b.SOURCES:
        obj = os.path.join(b.OBJ, os.path.splitext(src)[0] + ".o")
        if src == "gemm_mfma.hip":
            obj = os.path.join(b.OBJ, "gemm_mfma_phases.o")
            r = subprocess.run(["hipcc", *flags, "-DPO_PHASE_TIMING", "-c", os.path.join(b.CSRC, src), "-o", obj],
                               capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(r.stderr)
        elif not os.path.exists(obj):
            b.build(verbose=False)
        objs.append(obj)
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], capture_output=True,
                       text=True)
    if r.returncode != 0:
        raise RuntimeError(r.stderr)
    return LIB


def main(argv) -> int:
    if "--build" in argv:
        print("built", build_variant())
        return 0
    import torch

    if not os.path.exists(LIB):
        raise SystemExit("build the measurement library first: python -m paper_2503_01328_amd.gemm_phases --build")
    lib = C.CDLL(LIB)
    lib.po_op_gemm.restype = C.c_int
    lib.po_last_error.restype = C.c_char_p
    dev = torch.device("cuda:0")
    bf = torch.bfloat16
    rn = lambda *sh: (torch.randn(*sh, device=dev) * 0.5).to(bf)
    vp = lambda t: C.c_void_p(t.data_ptr() if t is not None else None)
    stream = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)

    def gemm(ta, tb, M, N, K, A, Bm, out):
        rc = lib.po_op_gemm(1, ta, tb, M, N, K, vp(A), A.shape[1], vp(Bm), Bm.shape[1], None, None, vp(out), None, None,
                            None, 0, stream)
        if rc:
            raise RuntimeError(lib.po_last_error().decode())

    print("shape | launch us | prologue us | main loop us | cycles per K slice (MFMA issue cycles) | epilogue us | clock GHz")
    for cfg, (s, h, f) in {"C2": (2048, 2048, 8192), "C3": (4096, 4096, 16384)}.items():
        shapes = {"qkv forward": (0, 0, s, 3 * h, h), "out-proj forward": (0, 0, s, h, h), "fc1 forward": (0, 0, s, f, h),
                  "fc2 forward": (0, 0, s, h, f), "fc1 dgrad": (0, 1, s, h, f), "qkv dgrad": (0, 1, s, h, 3 * h)}
        for name, (ta, tb, M, N, K) in shapes.items():
            A = rn(K, M) if ta else rn(M, K)
            Bm = rn(N, K) if tb else rn(K, N)
            out = torch.empty(M, N, device=dev, dtype=bf)
            for _ in range(3):
                gemm(ta, tb, M, N, K, A, Bm, out)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                gemm(ta, tb, M, N, K, A, Bm, out)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 100
            d = out.view(-1)[:8].view(torch.float32).cpu().tolist()
            clk = d[3] / 10.0
            bm, bn = C.c_int32(0), C.c_int32(0)
            lib.po_op_gemm_tile(M, N, C.byref(bm), C.byref(bn))
            ideal = (bm.value // 64) * (bn.value // 64) * 128  # MFMAs of a wave per slice x 32 cycles
            print(f"{cfg} {name} M={M} N={N} K={K} | {us:.1f} | {d[0] / clk / 1e3:.1f} | {d[1] / clk / 1e3:.1f} | "
                  f"{d[1] / (K // 64):.0f} ({ideal}) | {d[2] / clk / 1e3:.1f} | {clk:.2f}", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
