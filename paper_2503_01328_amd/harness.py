"""Glue between the seeded inputs (numpy), device memory (torch) and the binding.

Marshalling only: builds flat parameter buffers in the library's layout, uploads
inputs, calls the C ABI and downloads results.  Used by the tests, the smoke
check and the benchmark.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as po
from . import inputs as syn


def make_config(shape: syn.StageShape, **overrides) -> po.po_config:
    cfg = po.po_config_default(
        n_layers=shape.n_layers, n_chunks=shape.n_chunks, hidden=shape.hidden, n_heads=shape.n_heads,
        ffn=shape.ffn, seq=shape.seq, vocab=shape.vocab, dtype=po.PO_BF16 if shape.dtype == "bf16" else po.PO_F32,
        pipeline_degree=shape.pipeline_degree, rank=shape.rank, n_kv_heads=shape.n_kv_heads)
    for k, v in overrides.items():
        setattr(cfg, k, v)
    return cfg


def torch_dtype(cfg) -> torch.dtype:
    return torch.bfloat16 if cfg.dtype == po.PO_BF16 else torch.float32


def flatten_params(cfg, params: dict) -> np.ndarray:
    """fp32 flat array in the library's parameter layout."""
    flat = np.zeros(po.po_param_count(cfg), dtype=np.float32)
    for d in po.po_param_layout(cfg):
        src = params[d["name"]] if d["layer"] < 0 else params["layers"][d["layer"]][d["name"]]
        n = d["rows"] * d["cols"]
        flat[d["offset"]: d["offset"] + n] = np.asarray(src, dtype=np.float32).reshape(-1)
    return flat


def unflatten(cfg, flat: np.ndarray) -> dict:
    """Inverse of flatten_params: {'layers': [dict per layer], 'wte', 'wpe'}."""
    out = {"layers": [dict() for _ in range(cfg.n_layers)]}
    for d in po.po_param_layout(cfg):
        n = d["rows"] * d["cols"]
        a = flat[d["offset"]: d["offset"] + n]
        a = a.reshape(d["cols"]) if d["rows"] == 1 and d["layer"] >= 0 else a.reshape(d["rows"], d["cols"])
        if d["layer"] < 0:
            out[d["name"]] = a
        else:
            out["layers"][d["layer"]][d["name"]] = a
    return out


def upload(a: np.ndarray, cfg, device="cuda:0") -> torch.Tensor:
    if a.dtype == np.int32:
        return torch.from_numpy(np.ascontiguousarray(a)).to(device)
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return t.to(torch_dtype(cfg)).contiguous()


def download(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


class StageRunner:
    """Owns a stage plus the caller-side buffers (parameters, gradients, unit inputs and outputs)."""

    def __init__(self, shape: syn.StageShape, seed: int = 1234, device="cuda:0", params: dict | None = None,
                 n_microbatches: int | None = None, device_params: bool = False, **cfg_overrides):
        self.shape = shape
        self.seed = seed
        self.device = torch.device(device)
        self.cfg = make_config(shape, **cfg_overrides)
        self.m = n_microbatches if n_microbatches is not None else shape.n_microbatches
        self.v = shape.n_chunks
        if device_params:  # large configurations: draw the parameters on the device
            self.params_np = None
            self.params = random_device_params(self.cfg, self.device, seed)
        else:
            self.params_np = params if params is not None else syn.stage_params(shape, seed)
            flat = flatten_params(self.cfg, self.params_np)
            self.params = torch.from_numpy(flat).to(self.device).to(torch_dtype(self.cfg)).contiguous()
        self.grads = torch.zeros(self.params.shape[0], dtype=torch.float32, device=self.device)
        torch.cuda.synchronize()
        self.stage = po.po_stage_create(self.cfg, torch.cuda.current_stream(self.device))
        po.po_bind_params(self.stage, self.params, self.grads)
        self.x = self.y = self.dy = self.dx = None

    def close(self):
        if self.stage is not None:
            po.po_stage_destroy(self.stage)
            self.stage = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def unit_index(self, mb, chunk):
        return chunk * self.m + mb

    def make_inputs(self, x_np: dict | None = None, dy_np: dict | None = None):
        """Uploads seeded inputs for every (mb, chunk); allocates outputs."""
        s, h = self.shape.seq, self.shape.hidden
        n = self.m * self.v
        self.x, self.dy, self.y, self.dx = [None] * n, [None] * n, [None] * n, [None] * n
        dt = torch_dtype(self.cfg)
        for c in range(self.v):
            for j in range(self.m):
                i = self.unit_index(j, c)
                xa = x_np[(j, c)] if x_np is not None else syn.unit_input(self.shape, j, c, self.seed)
                da = dy_np[(j, c)] if dy_np is not None else syn.unit_upstream_grad(self.shape, j, c, self.seed)
                self.x[i] = upload(xa, self.cfg, self.device)
                self.dy[i] = upload(da, self.cfg, self.device)
                self.y[i] = torch.empty(s, h, dtype=dt, device=self.device)
                embed = self.shape.vocab > 0 and c == 0
                self.dx[i] = None if embed else torch.empty(s, h, dtype=dt, device=self.device)
        torch.cuda.synchronize()

    def make_inputs_on_device(self, seed: int = 0):
        """Random inputs generated directly on the device (benchmarking of large configurations)."""
        s, h = self.shape.seq, self.shape.hidden
        n = self.m * self.v
        g = torch.Generator(device=self.device)
        g.manual_seed(self.seed + seed)
        dt = torch_dtype(self.cfg)
        vocab = self.shape.vocab
        self.x, self.dx = [], []
        for i in range(n):
            embed = vocab > 0 and i < self.m  # units of chunk 0 take token ids and have no input gradient
            if embed:
                self.x.append(torch.randint(0, vocab, (s,), generator=g, device=self.device, dtype=torch.int32))
                self.dx.append(None)
            else:
                self.x.append(torch.randn(s, h, generator=g, device=self.device, dtype=torch.float32).to(dt))
                self.dx.append(torch.empty(s, h, dtype=dt, device=self.device))
        self.dy = [torch.randn(s, h, generator=g, device=self.device, dtype=torch.float32).to(dt) for _ in range(n)]
        self.y = [torch.empty(s, h, dtype=dt, device=self.device) for _ in range(n)]
        torch.cuda.synchronize()

    def zero_grads(self):
        self.grads.zero_()
        torch.cuda.synchronize()

    def run(self, schedule=po.PO_SCHED_1F1B, ratio=0.0) -> dict:
        return po.po_run_schedule(self.stage, schedule, self.m, ratio, self.x, self.y, self.dy, self.dx)

    def results(self):
        """(y {(mb, chunk): np}, dx {(mb, chunk): np or None}, grads dict) as fp32 numpy."""
        torch.cuda.synchronize()
        y, dx = {}, {}
        for c in range(self.v):
            for j in range(self.m):
                i = self.unit_index(j, c)
                y[(j, c)] = download(self.y[i])
                dx[(j, c)] = None if self.dx[i] is None else download(self.dx[i])
        return y, dx, unflatten(self.cfg, self.grads.cpu().numpy())


def random_device_params(cfg, device="cuda:0", seed=1234) -> torch.Tensor:
    """N(0, 0.02) parameters with LayerNorm gains around one, generated on the device (large configurations)."""
    n = po.po_param_count(cfg)
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    flat = torch.randn(n, generator=g, device=device, dtype=torch.float32) * 0.02
    for d in po.po_param_layout(cfg):
        if d["name"] in ("ln1_g", "ln2_g"):
            flat[d["offset"]: d["offset"] + d["cols"]] += 1.0
    return flat.to(torch_dtype(cfg)).contiguous()


def max_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| over one tensor."""
    denom = float(np.abs(ref).max())
    if denom == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got.astype(np.float64) - ref.astype(np.float64)).max() / denom)


def rel_l2_err(got: np.ndarray, ref: np.ndarray) -> float:
    """||got - ref||_2 / ||ref||_2 over one tensor."""
    g, r = got.astype(np.float64), ref.astype(np.float64)
    denom = float(np.sqrt((r * r).sum()))
    num = float(np.sqrt(((g - r) ** 2).sum()))
    return num if denom == 0.0 else num / denom


def check_parity(got: np.ndarray, ref: np.ndarray, tol: float, what: str) -> tuple:
    """Asserts both error norms of one tensor against `tol` and prints them (pytest -s shows the lines; a failure
    shows them anyway): the per-tensor max norm max|got - ref| / max|ref| and the relative L2 norm."""
    mx, l2 = max_rel_err(got, ref), rel_l2_err(got, ref)
    print(f"parity {what}: max-norm {mx:.3e}  rel-L2 {l2:.3e}  (tolerance {tol:g})")
    assert mx < tol, f"{what}: max|got - ref| / max|ref| = {mx:.3e} >= {tol:g}"
    assert l2 < tol, f"{what}: ||got - ref|| / ||ref|| = {l2:.3e} >= {tol:g}"
    return mx, l2

