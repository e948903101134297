"""Thin ctypes binding of libpipeoffload.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
include/pipeoffload.h) and does nothing but convert arguments: torch tensors
become raw device pointers, Python lists become C arrays.  All computation runs
in the HIP library.  There is no fallback: if the library has not been built,
importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

# PyTorch ships its own HIP runtime.  It has to be loaded before this library, so that both
# resolve to ONE runtime in the process: with two, kernel launches from here see no device.
import torch  # noqa: F401  (device memory and streams come from torch anyway)

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpipeoffload.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it with `python -m paper_2503_01328_amd.build` "
        "(or __graft_entry__.build()); there is no non-HIP fallback")
lib = C.CDLL(_LIB_PATH)

PO_F32, PO_BF16 = 0, 1
PO_SCHED_1F1B, PO_SCHED_1F1B_INTERLEAVED, PO_SCHED_GIS, PO_SCHED_PO = 0, 1, 2, 3
PO_SEL_ALTERNATE_MB, PO_SEL_LONGEST_LIFESPAN = 0, 1
PO_OK, PO_E_INVAL, PO_E_STATE, PO_E_DEVICE_OOM, PO_E_HOST_OOM, PO_E_HIP = 0, -1, -2, -3, -4, -5
OP_KINDS = ("F", "B", "OFFLOAD", "RELOAD", "W")


class po_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_chunks", "hidden", "n_heads", "ffn", "seq", "vocab", "dtype", "pipeline_degree", "rank",
        "prefetch_passes", "copy_streams", "select_policy", "staged_copies", "debug_poison", "profile_kernels",
        "group", "weight_stream", "n_kv_heads", "min_gap_passes")] + [
        ("ln_eps", C.c_float), ("dropout_p", C.c_float), ("slot_k", C.c_float), ("host_pool_cap_bytes", C.c_uint64),
        ("device_pool_cap_bytes", C.c_uint64), ("dropout_seed", C.c_uint64)]


class po_param_desc(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("layer", C.c_int32), ("reserved", C.c_int32),
                ("offset_elems", C.c_int64), ("rows", C.c_int64), ("cols", C.c_int64)]


class po_op(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mb", C.c_int32), ("chunk", C.c_int32), ("ratio", C.c_float)]


class po_stats(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("wall_s", "tokens_per_s", "compute_busy_s", "d2h_busy_s", "h2d_busy_s",
                                           "pack_busy_s", "compute_span_s", "gemm_busy_s", "gemm_flops",
                                           "attn_busy_s", "attn_flops", "copy_hidden_s")] + \
               [(n, C.c_uint64) for n in ("bytes_d2h", "bytes_h2d", "peak_slab_bytes", "pool_bytes_allocated",
                                          "host_bytes_allocated", "workspace_bytes")] + \
               [(n, C.c_int32) for n in ("peak_resident_units", "peak_in_flight_units", "n_compute_passes",
                                         "n_offloads", "n_reloads", "n_gemm_launches")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


EXPORTS = {
    "po_config_default": (None, [C.POINTER(po_config)]),
    "po_last_error": (C.c_char_p, []),
    "po_param_count": (C.c_int, [C.POINTER(po_config), C.POINTER(C.c_int64)]),
    "po_param_layout": (C.c_int, [C.POINTER(po_config), C.POINTER(po_param_desc), C.POINTER(C.c_int32)]),
    "po_saved_bytes_per_layer": (C.c_int, [C.POINTER(po_config), C.POINTER(C.c_uint64)]),
    "po_schedule_ops": (C.c_int, [C.c_int32] * 6 + [C.c_float, C.c_int32, C.c_int32, C.c_int32, C.POINTER(po_op),
                                                    C.POINTER(C.c_int32)]),
    "po_schedule_ops_slots": (C.c_int, [C.c_int32] * 6 + [C.c_double, C.POINTER(po_op), C.POINTER(C.c_int32)]),
    "po_offload_k": (C.c_double, [C.c_int32, C.c_int32, C.c_double, C.c_double]),
    "po_offload_ratio_for_k": (C.c_double, [C.c_double]),
    "po_stage_create": (C.c_int, [C.POINTER(po_config), C.c_void_p, C.POINTER(C.c_void_p)]),
    "po_stage_destroy": (None, [C.c_void_p]),
    "po_bind_params": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "po_stage_forward": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "po_stage_backward": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "po_stage_backward_input": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "po_stage_backward_weight": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32]),
    "po_offload": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_float]),
    "po_reload": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32]),
    "po_run_schedule": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.POINTER(C.c_void_p),
                                  C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                  C.POINTER(po_stats)]),
    "po_synchronize": (C.c_int, [C.c_void_p]),
    "po_stage_reset": (C.c_int, [C.c_void_p]),
    "po_get_stats": (C.c_int, [C.c_void_p, C.POINTER(po_stats)]),
    "po_op_layernorm_forward": (C.c_int, [C.c_int32] + [C.c_void_p] * 4 + [C.c_int32, C.c_int32, C.c_float,
                                                                          C.c_void_p]),
    "po_op_layernorm_backward_workspace": (C.c_uint64, [C.c_int32, C.c_int32]),
    "po_op_layernorm_backward": (C.c_int, [C.c_int32] + [C.c_void_p] * 8 + [C.c_int32, C.c_int32, C.c_float,
                                                                           C.c_void_p]),
    "po_op_gemm": (C.c_int, [C.c_int32] * 6 + [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32] + [C.c_void_p] * 6 +
                   [C.c_int32, C.c_void_p]),
    "po_op_gemm_grouped": (C.c_int, [C.c_int32] + [C.POINTER(C.c_int32)] * 3 + [C.POINTER(C.c_void_p), C.POINTER(C.c_int32)] * 2 +
                           [C.POINTER(C.c_void_p), C.POINTER(C.c_int32), C.c_void_p]),
    "po_op_gemm_tile": (C.c_int, [C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "po_op_attention_forward": (C.c_int, [C.c_int32] + [C.c_void_p] * 3 + [C.c_int32] * 5 + [C.c_void_p]),
    "po_op_attention_backward": (C.c_int, [C.c_int32] + [C.c_void_p] * 7 + [C.c_int32] * 5 + [C.c_void_p]),
    "po_op_dropout": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_uint64,
                                C.c_int32, C.c_int32, C.c_int32, C.c_void_p]),
    "po_set_dropout_seed": (C.c_int, [C.c_void_p, C.c_uint64]),
    "po_op_colsum_workspace": (C.c_uint64, [C.c_int32, C.c_int32]),
    "po_op_colsum_accumulate": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                          C.c_void_p]),
    "po_op_colsum_accumulate_static": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]),
    "po_op_pack": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(C.c_uint64), C.c_int32, C.c_void_p, C.c_void_p]),
    "po_op_unpack": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(C.c_uint64), C.c_int32, C.c_void_p, C.c_void_p]),
}
for _name, (_res, _args) in EXPORTS.items():
    _f = getattr(lib, _name)
    _f.restype = _res
    _f.argtypes = _args


class PipeOffloadError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"pipeoffload error {code}: {text}")
        self.code = code


def _check(rc):
    if rc != 0:
        raise PipeOffloadError(rc, po_last_error())


def po_last_error() -> str:
    return lib.po_last_error().decode()


def _ptr(t):
    """Raw pointer of a torch tensor (device or host), an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def po_config_default(**overrides) -> po_config:
    cfg = po_config()
    lib.po_config_default(C.byref(cfg))
    for k, v in overrides.items():
        if not hasattr(cfg, k):
            raise AttributeError(k)
        setattr(cfg, k, v)
    return cfg


def po_param_count(cfg) -> int:
    n = C.c_int64()
    _check(lib.po_param_count(C.byref(cfg), C.byref(n)))
    return n.value


def po_param_layout(cfg):
    n = C.c_int32(0)
    _check(lib.po_param_layout(C.byref(cfg), None, C.byref(n)))
    arr = (po_param_desc * n.value)()
    _check(lib.po_param_layout(C.byref(cfg), arr, C.byref(n)))
    return [dict(name=d.name.decode(), layer=d.layer, offset=d.offset_elems, rows=d.rows, cols=d.cols) for d in arr]


def po_saved_bytes_per_layer(cfg) -> int:
    b = C.c_uint64()
    _check(lib.po_saved_bytes_per_layer(C.byref(cfg), C.byref(b)))
    return b.value


def po_schedule_ops(schedule, d, rank, v, m, ratio, policy=0, prefetch=2, group=0, min_gap=0):
    n = C.c_int32(0)
    _check(lib.po_schedule_ops(schedule, d, rank, v, m, group, ratio, policy, prefetch, min_gap, None, C.byref(n)))
    arr = (po_op * n.value)()
    _check(lib.po_schedule_ops(schedule, d, rank, v, m, group, ratio, policy, prefetch, min_gap, arr, C.byref(n)))
    return [(OP_KINDS[o.kind], o.mb, o.chunk) for o in arr]


def po_schedule_ops_slots(d, rank, v, m, n_offload_chunks, k, group=0):
    n = C.c_int32(0)
    _check(lib.po_schedule_ops_slots(d, rank, v, m, group, n_offload_chunks, k, None, C.byref(n)))
    arr = (po_op * n.value)()
    _check(lib.po_schedule_ops_slots(d, rank, v, m, group, n_offload_chunks, k, arr, C.byref(n)))
    return [(OP_KINDS[o.kind], o.mb, o.chunk) for o in arr]


def po_offload_ratio_for_k(k) -> float:
    return lib.po_offload_ratio_for_k(k)


def po_offload_k(h, s, compute_flops_per_s, link_bytes_per_s) -> float:
    return lib.po_offload_k(h, s, compute_flops_per_s, link_bytes_per_s)


def po_stage_create(cfg, stream=None):
    out = C.c_void_p()
    _check(lib.po_stage_create(C.byref(cfg), _stream(stream), C.byref(out)))
    return out


def po_stage_destroy(stage):
    lib.po_stage_destroy(stage)


def po_bind_params(stage, params, grads):
    _check(lib.po_bind_params(stage, _ptr(params), _ptr(grads)))


def po_stage_forward(stage, mb, chunk, x_in, y_out):
    _check(lib.po_stage_forward(stage, mb, chunk, _ptr(x_in), _ptr(y_out)))


def po_stage_backward(stage, mb, chunk, dy, dx):
    _check(lib.po_stage_backward(stage, mb, chunk, _ptr(dy), _ptr(dx)))


def po_stage_backward_input(stage, mb, chunk, dy, dx):
    _check(lib.po_stage_backward_input(stage, mb, chunk, _ptr(dy), _ptr(dx)))


def po_stage_backward_weight(stage, mb, chunk):
    _check(lib.po_stage_backward_weight(stage, mb, chunk))


def po_offload(stage, mb, chunk, ratio):
    _check(lib.po_offload(stage, mb, chunk, ratio))


def po_reload(stage, mb, chunk):
    _check(lib.po_reload(stage, mb, chunk))


def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else t.data_ptr()
    return arr


def po_run_schedule(stage, schedule, n_microbatches, offload_ratio, x_in, y_out, dy, dx) -> dict:
    """x_in, y_out, dy, dx: lists of tensors indexed [chunk * m + mb] (dx entries may be None)."""
    st = po_stats()
    _check(lib.po_run_schedule(stage, schedule, n_microbatches, offload_ratio, _ptr_array(x_in), _ptr_array(y_out),
                               _ptr_array(dy), _ptr_array(dx), C.byref(st)))
    return st.as_dict()


def po_synchronize(stage):
    _check(lib.po_synchronize(stage))


def po_stage_reset(stage):
    _check(lib.po_stage_reset(stage))


def po_get_stats(stage) -> dict:
    st = po_stats()
    _check(lib.po_get_stats(stage, C.byref(st)))
    return st.as_dict()


def po_op_layernorm_forward(dtype, x, gain, shift, y, rows, h, eps, stream=None):
    _check(lib.po_op_layernorm_forward(dtype, _ptr(x), _ptr(gain), _ptr(shift), _ptr(y), rows, h, eps,
                                       _stream(stream)))


def po_op_layernorm_backward_workspace(rows, h) -> int:
    return lib.po_op_layernorm_backward_workspace(rows, h)


def po_op_layernorm_backward(dtype, dn, x, gain, dres, dx, dgain, dshift, partials, rows, h, eps, stream=None):
    _check(lib.po_op_layernorm_backward(dtype, _ptr(dn), _ptr(x), _ptr(gain), _ptr(dres), _ptr(dx), _ptr(dgain),
                                        _ptr(dshift), _ptr(partials), rows, h, eps, _stream(stream)))


def po_op_gemm(dtype, trans_a, trans_b, M, N, K, A, lda, B, ldb, bias=None, residual=None, out=None, gelu_out=None,
               gelu_u=None, acc_f32=None, force_generic=0, stream=None):
    _check(lib.po_op_gemm(dtype, trans_a, trans_b, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(bias), _ptr(residual),
                          _ptr(out), _ptr(gelu_out), _ptr(gelu_u), _ptr(acc_f32), force_generic, _stream(stream)))


def po_op_gemm_grouped(problems, stream=None):
    """problems: list of (M, N, K, A [K, M], lda, B [K, N], ldb, acc_f32 [M, N], ldc); acc_f32 += A^T B for each."""
    n = len(problems)
    ints = lambda k: (C.c_int32 * n)(*[p[k] for p in problems])
    ptrs = lambda k: _ptr_array([p[k] for p in problems])
    _check(lib.po_op_gemm_grouped(n, ints(0), ints(1), ints(2), ptrs(3), ints(4), ptrs(5), ints(6), ptrs(7), ints(8),
                                  _stream(stream)))


def po_op_gemm_tile(M, N):
    """(tile rows, tile columns) of the bf16 matrix-core GEMM for an M x N result; (0, 0) if it has none."""
    bm, bn = C.c_int32(0), C.c_int32(0)
    _check(lib.po_op_gemm_tile(M, N, C.byref(bm), C.byref(bn)))
    return bm.value, bn.value


def po_op_attention_forward(dtype, qkv, o, lse, s, h, n_heads, force_generic=0, stream=None, n_kv_heads=0):
    _check(lib.po_op_attention_forward(dtype, _ptr(qkv), _ptr(o), _ptr(lse), s, h, n_heads, n_kv_heads,
                                       force_generic, _stream(stream)))


def po_op_attention_backward(dtype, qkv, o, lse, d_o, dqkv, delta, s, h, n_heads, force_generic=0, stream=None,
                             n_kv_heads=0, partials=None):
    _check(lib.po_op_attention_backward(dtype, _ptr(qkv), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dqkv), _ptr(delta),
                                        _ptr(partials), s, h, n_heads, n_kv_heads, force_generic, _stream(stream)))


def po_op_dropout(dtype, x, out, rows, cols, p, seed, layer, site, mb, stream=None):
    _check(lib.po_op_dropout(dtype, _ptr(x), _ptr(out), rows, cols, p, seed, layer, site, mb, _stream(stream)))


def po_set_dropout_seed(stage, seed):
    _check(lib.po_set_dropout_seed(stage, seed))


def po_op_colsum_workspace(rows, n) -> int:
    return lib.po_op_colsum_workspace(rows, n)


def po_op_colsum_accumulate(dtype, x, acc, workspace, rows, n, stream=None):
    _check(lib.po_op_colsum_accumulate(dtype, _ptr(x), _ptr(acc), _ptr(workspace), rows, n, _stream(stream)))


def po_op_colsum_accumulate_static(dtype, x, acc, rows, n, stream=None):
    _check(lib.po_op_colsum_accumulate_static(dtype, _ptr(x), _ptr(acc), rows, n, _stream(stream)))


def po_op_pack(segments, packed, stream=None):
    """segments: list of (tensor_or_ptr, n_bytes)."""
    ptrs = (C.c_void_p * len(segments))(*[(s if isinstance(s, int) else s.data_ptr()) for s, _ in segments])
    sizes = (C.c_uint64 * len(segments))(*[b for _, b in segments])
    _check(lib.po_op_pack(ptrs, sizes, len(segments), _ptr(packed), _stream(stream)))


def po_op_unpack(segments, packed, stream=None):
    ptrs = (C.c_void_p * len(segments))(*[(s if isinstance(s, int) else s.data_ptr()) for s, _ in segments])
    sizes = (C.c_uint64 * len(segments))(*[b for _, b in segments])
    _check(lib.po_op_unpack(ptrs, sizes, len(segments), _ptr(packed), _stream(stream)))
