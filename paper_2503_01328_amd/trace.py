"""Prints the span timeline that the library appends to the file named by PIPEOFFLOAD_TRACE.

    PIPEOFFLOAD_TRACE=/tmp/run.txt python bench.py --steps 1 --warmup 1 --no-cpu-baseline
    python -m paper_2503_01328_amd.trace /tmp/run.txt [run index, default: the last run in the file]

One block per stream (compute passes, D2H copies, H2D copies): every span as [start-end] in milliseconds from the
first span of the run, with the gap to the span before it on the same stream, and the stream's busy time.  The
picture to look for is the paper's Figure 7: copies back to back on their streams while the compute stream has no
gaps; a gap on the compute stream in front of a backward pass is a reload that came too late.
"""
from __future__ import annotations

import sys

NAMES = {0: "compute", 1: "D2H", 2: "H2D", 3: "pack/unpack", 4: "GEMM launches (sampled)", 5: "attention launches (sampled)"}


def read_runs(path: str) -> list[list[tuple[int, float, float]]]:
    runs: list[list[tuple[int, float, float]]] = []
    for line in open(path):
        if line.startswith("#"):
            runs.append([])
            continue
        kind, start, stop = line.split()
        if not runs:
            runs.append([])
        runs[-1].append((int(kind), float(start), float(stop)))
    return [r for r in runs if r]


def render(run: list[tuple[int, float, float]], per_line: int = 8) -> str:
    out = []
    end = max(stop for _, _, stop in run)
    out.append(f"run of {end:.2f} ms, {len(run)} spans")
    for kind in sorted({k for k, _, _ in run}):
        spans = [(a, b) for k, a, b in run if k == kind]
        busy = sum(b - a for a, b in spans)
        out.append(f"{NAMES.get(kind, kind)}: {len(spans)} spans, busy {busy:.2f} ms")
        cells, prev = [], None
        for a, b in spans:
            gap = a - prev if prev is not None else a
            cells.append(f"[{a:7.2f}-{b:7.2f} gap {gap:5.2f}]")
            prev = b
        for i in range(0, len(cells), per_line):
            out.append("    " + " ".join(cells[i:i + per_line]))
    return "\n".join(out)


def main(argv: list[str]) -> int:
    if len(argv) < 2:
        print(__doc__)
        return 2
    runs = read_runs(argv[1])
    if not runs:
        print("no spans in", argv[1])
        return 1
    index = int(argv[2]) if len(argv) > 2 else len(runs) - 1
    print(render(runs[index]))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
