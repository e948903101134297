"""Parity of the single HIP operations against the CPU oracle, through the C ABI.

Tolerances (max |got - ref| / max |ref| per tensor): 1e-4 in fp32, 2e-2 in bf16.
The oracle is fed the values the kernel is fed (bf16-rounded where bf16)."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as so
from paper_2503_01328_amd import binding as po
from paper_2503_01328_amd import inputs as syn
from paper_2503_01328_amd.harness import check_parity, max_rel_err

pytestmark = pytest.mark.gpu

DT = {"f32": (po.PO_F32, torch.float32, 1e-4), "bf16": (po.PO_BF16, torch.bfloat16, 2e-2)}


def _dev(a, tdt, dev):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(tdt).contiguous()


def _rand(rng, shape, dtype, scale=1.0, shift=0.0):
    a = (rng.standard_normal(shape) * scale + shift).astype(np.float32)
    return syn.round_to_bf16(a) if dtype == "bf16" else a


def _np(t):
    return t.to(torch.float32).cpu().numpy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,h", [(1, 64), (7, 256), (130, 1024), (33, 5120), (5, 2048), (3, 3584), (4, 8192)])
def test_layernorm_forward_and_backward(gpu_device, dtype, rows, h):
    code, tdt, tol = DT[dtype]
    rng = np.random.default_rng(rows * 1000 + h)
    x = _rand(rng, (rows, h), dtype, 2.0, 0.5)
    g = _rand(rng, (h,), dtype, 0.1, 1.0)
    b = _rand(rng, (h,), dtype, 0.1)
    dn = _rand(rng, (rows, h), dtype)
    dres = _rand(rng, (rows, h), dtype)
    xd, gd, bd, dnd, dresd = (_dev(a, tdt, gpu_device) for a in (x, g, b, dn, dres))
    y = torch.empty_like(xd)
    po.po_op_layernorm_forward(code, xd, gd, bd, y, rows, h, 1e-5)
    ref, cache = so.layernorm_forward(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), 1e-5)
    assert max_rel_err(_np(y), ref) < tol
    ws = torch.empty(po.po_op_layernorm_backward_workspace(rows, h) // 4, dtype=torch.float32, device=gpu_device)
    dx = torch.empty_like(xd)
    dg0 = rng.standard_normal(h).astype(np.float32)
    db0 = rng.standard_normal(h).astype(np.float32)
    dg, db = torch.from_numpy(dg0).to(gpu_device), torch.from_numpy(db0).to(gpu_device)
    po.po_op_layernorm_backward(code, dnd, xd, gd, dresd, dx, dg, db, ws, rows, h, 1e-5)
    rdx, rdg, rdb = so.layernorm_backward(dn.astype(np.float64), cache, g.astype(np.float64))
    assert max_rel_err(_np(dx), rdx + dres) < tol
    assert max_rel_err(_np(dg) - dg0, rdg) < max(tol, 1e-4)  # fp32 accumulators added into existing values
    assert max_rel_err(_np(db) - db0, rdb) < max(tol, 1e-4)
    # without a residual
    po.po_op_layernorm_backward(code, dnd, xd, gd, None, dx, dg, db, ws, rows, h, 1e-5)
    assert max_rel_err(_np(dx), rdx) < tol


GEMM_SHAPES_GENERIC = [(1, 1, 1), (5, 7, 3), (64, 64, 16), (70, 130, 45), (128, 256, 256)]


def _gemm_case(gpu_device, dtype, ta, tb, M, N, K, epilogue, force_generic):
    code, tdt, tol = DT[dtype]
    rng = np.random.default_rng(M * 7 + N * 3 + K + ta * 2 + tb)
    A = _rand(rng, (K, M) if ta else (M, K), dtype)
    B = _rand(rng, (N, K) if tb else (K, N), dtype, 0.05)
    Ad, Bd = _dev(A, tdt, gpu_device), _dev(B, tdt, gpu_device)
    a64 = (A.T if ta else A).astype(np.float64)
    b64 = (B.T if tb else B).astype(np.float64)
    ref = a64 @ b64
    lda, ldb = A.shape[1], B.shape[1]
    kw = dict(force_generic=force_generic)
    if epilogue == "plain":
        out = torch.empty(M, N, dtype=tdt, device=gpu_device)
        po.po_op_gemm(code, ta, tb, M, N, K, Ad, lda, Bd, ldb, out=out, **kw)
        assert max_rel_err(_np(out), ref) < tol
    elif epilogue == "bias_residual":
        bias = _rand(rng, (N,), dtype)
        res = _rand(rng, (M, N), dtype)
        out = torch.empty(M, N, dtype=tdt, device=gpu_device)
        po.po_op_gemm(code, ta, tb, M, N, K, Ad, lda, Bd, ldb, bias=_dev(bias, tdt, gpu_device),
                      residual=_dev(res, tdt, gpu_device), out=out, **kw)
        assert max_rel_err(_np(out), ref + bias + res) < tol
    elif epilogue == "bias_gelu":
        bias = _rand(rng, (N,), dtype)
        out = torch.empty(M, N, dtype=tdt, device=gpu_device)
        g = torch.empty(M, N, dtype=tdt, device=gpu_device)
        po.po_op_gemm(code, ta, tb, M, N, K, Ad, lda, Bd, ldb, bias=_dev(bias, tdt, gpu_device), out=out,
                      gelu_out=g, **kw)
        assert max_rel_err(_np(out), ref + bias) < tol
        assert max_rel_err(_np(g), so.gelu(_np(out).astype(np.float64))) < tol  # gelu of the stored (rounded) u
    elif epilogue == "gelu_backward":
        u = _rand(rng, (M, N), dtype, 1.5)
        out = torch.empty(M, N, dtype=tdt, device=gpu_device)
        g = torch.empty(M, N, dtype=tdt, device=gpu_device)
        po.po_op_gemm(code, ta, tb, M, N, K, Ad, lda, Bd, ldb, out=out, gelu_out=g,
                      gelu_u=_dev(u, tdt, gpu_device), **kw)
        assert max_rel_err(_np(out), ref * so.gelu_derivative(u.astype(np.float64))) < tol
        assert max_rel_err(_np(g), so.gelu(u.astype(np.float64))) < tol
    elif epilogue == "accumulate":
        acc0 = rng.standard_normal((M, N)).astype(np.float32)
        acc = torch.from_numpy(acc0).to(gpu_device)
        po.po_op_gemm(code, ta, tb, M, N, K, Ad, lda, Bd, ldb, acc_f32=acc, **kw)
        assert max_rel_err(_np(acc) - acc0, ref) < max(tol, 2e-4)
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("shape", GEMM_SHAPES_GENERIC)
def test_gemm_generic_all_forms(gpu_device, dtype, ta, tb, shape):
    _gemm_case(gpu_device, dtype, ta, tb, *shape, "plain", 1)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("epilogue", ["bias_residual", "bias_gelu", "gelu_backward", "accumulate"])
def test_gemm_generic_epilogues(gpu_device, dtype, epilogue):
    _gemm_case(gpu_device, dtype, 0, 0, 70, 130, 45, epilogue, 1)


# MFMA path: 128-tiles (M, N multiples of 128), 256-tiles (>= 192 tiles of 256 x 256) and 256 x 192 tiles (N a
# multiple of 192 and a round of them cheaper), K multiple of 64 (one, two, three and many slices)
MFMA_SHAPES = [(128, 128, 64), (256, 384, 192), (384, 128, 1024), (4096, 3328, 128), (2048, 6144, 64),
               (4096, 3072, 192), (4096, 6144, 128), (2048, 6144, 512)]


def test_gemm_mfma_shapes_cover_every_tile():
    assert {po.po_op_gemm_tile(M, N) for M, N, _ in MFMA_SHAPES} == {(128, 128), (256, 256), (256, 192)}


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("shape", MFMA_SHAPES)
def test_gemm_mfma_all_forms(gpu_device, ta, tb, shape):
    _gemm_case(gpu_device, "bf16", ta, tb, *shape, "plain", 0)


@pytest.mark.parametrize("epilogue", ["bias_residual", "bias_gelu", "gelu_backward", "accumulate"])
@pytest.mark.parametrize("shape", [(256, 384, 192), (4096, 3328, 128), (2048, 6144, 192)])
def test_gemm_mfma_epilogues(gpu_device, epilogue, shape):
    form = {"accumulate": (1, 0), "gelu_backward": (0, 1)}.get(epilogue, (0, 0))
    _gemm_case(gpu_device, "bf16", *form, *shape, epilogue, 0)


def test_gemm_grouped_equals_single_launches_and_the_oracle(gpu_device):
    """Four weight-gradient products of different shapes in one launch: each accumulator equals, bit for bit, what
    the single launch of that product leaves, and the fp64 product within the bf16 tolerance.  Tile counts
    8 + 24 + 4 + 257 = 293 make two rounds, the second one ragged."""
    rng = np.random.default_rng(11)
    shapes = [(512, 1024, 192), (2048, 768, 64), (256, 1024, 128), (256, 65792, 64)]
    probs, single, refs, acc0s = [], [], [], []
    for M, N, K in shapes:
        A = _rand(rng, (K, M), "bf16")
        B = _rand(rng, (K, N), "bf16", 0.05)
        acc0 = rng.standard_normal((M, N)).astype(np.float32)
        Ad, Bd = _dev(A, torch.bfloat16, gpu_device), _dev(B, torch.bfloat16, gpu_device)
        acc = torch.from_numpy(acc0).to(gpu_device)
        alone = torch.from_numpy(acc0).to(gpu_device)
        po.po_op_gemm(po.PO_BF16, 1, 0, M, N, K, Ad, M, Bd, N, acc_f32=alone)
        probs.append((M, N, K, Ad, M, Bd, N, acc, N))
        single.append(alone)
        refs.append(A.T.astype(np.float64) @ B.astype(np.float64))
        acc0s.append(acc0)
    po.po_op_gemm_grouped(probs)
    torch.cuda.synchronize()
    for p, alone, ref, acc0 in zip(probs, single, refs, acc0s):
        assert torch.equal(p[7], alone)
        assert max_rel_err(_np(p[7]) - acc0, ref) < 2e-2
    # one problem alone, fewer tiles than compute units
    M, N, K = 256, 512, 64
    A = _rand(rng, (K, M), "bf16")
    B = _rand(rng, (K, N), "bf16")
    acc = torch.zeros(M, N, device=gpu_device)
    po.po_op_gemm_grouped([(M, N, K, _dev(A, torch.bfloat16, gpu_device), M, _dev(B, torch.bfloat16, gpu_device), N,
                            acc, N)])
    assert max_rel_err(_np(acc), A.T.astype(np.float64) @ B.astype(np.float64)) < 2e-2
    with pytest.raises(po.PipeOffloadError):  # 384 is no multiple of 256
        po.po_op_gemm_grouped([(384, 512, 64, acc, 384, acc, 512, acc, 512)])
    with pytest.raises(po.PipeOffloadError):
        po.po_op_gemm_grouped([(256, 512, 64, acc, 256, acc, 512, acc, 512)] * 5)


def test_gemm_rejects_bad_arguments(gpu_device):
    a = torch.zeros(64, 64, device=gpu_device)
    with pytest.raises(po.PipeOffloadError):
        po.po_op_gemm(po.PO_F32, 0, 0, 64, 64, 64, a, 32, a, 64, out=a)  # lda too small
    with pytest.raises(po.PipeOffloadError):
        po.po_op_gemm(po.PO_F32, 0, 0, 64, 64, 64, a, 64, a, 64)  # no output
    with pytest.raises(po.PipeOffloadError):
        po.po_op_gemm(9, 0, 0, 64, 64, 64, a, 64, a, 64, out=a)  # bad dtype
    with pytest.raises(po.PipeOffloadError):
        po.po_op_gemm(po.PO_F32, 0, 0, 0, 64, 64, a, 64, a, 64, out=a)  # empty


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("s,h,a", [(1, 64, 1), (5, 64, 2), (64, 128, 2), (65, 256, 4), (200, 256, 2), (130, 512, 2)])
@pytest.mark.parametrize("force_generic", [1, 0])
def test_attention_forward_and_backward(gpu_device, dtype, s, h, a, force_generic):
    _attention_case(gpu_device, dtype, s, h, a, force_generic)


# shapes the matrix-core kernels take: head size 64 / 128, s a multiple of 128; the last two
# are large enough in (s / 256) * heads to select the forward kernel's 256-row blocks (both head sizes)
@pytest.mark.parametrize("s,h,a", [(128, 128, 2), (256, 256, 2), (384, 128, 1), (640, 192, 3), (512, 16384, 256),
                                   (512, 32768, 256)])
def test_attention_mfma(gpu_device, s, h, a):
    _attention_case(gpu_device, "bf16", s, h, a, 0)


def _attention_case(gpu_device, dtype, s, h, a, force_generic, akv=0, with_partials=False):
    code, tdt, tol = DT[dtype]
    rng = np.random.default_rng(s * 31 + h + a + 7 * akv)
    dh = h // a
    hkv = (akv or a) * dh
    group = a // (akv or a)
    qkv = _rand(rng, (s, h + 2 * hkv), dtype)
    d_o = _rand(rng, (s, h), dtype)
    qd, dod = _dev(qkv, tdt, gpu_device), _dev(d_o, tdt, gpu_device)
    o = torch.empty(s, h, dtype=tdt, device=gpu_device)
    lse = torch.empty(a, s, dtype=torch.float32, device=gpu_device)
    po.po_op_attention_forward(code, qd, o, lse, s, h, a, force_generic, n_kv_heads=akv)
    q64 = qkv.astype(np.float64)
    q, k, v = q64[:, :h], q64[:, h:h + hkv], q64[:, h + hkv:]
    ro, probs = so.attention_forward(q, k, v, a)
    assert max_rel_err(_np(o), ro) < tol
    # log-sum-exp of the scaled, masked scores: a plain definition
    for t in range(a):
        kt = k[:, (t // group) * dh:(t // group + 1) * dh]
        sc = (q[:, t * dh:(t + 1) * dh] @ kt.T) / np.sqrt(dh)
        sc = np.where(np.triu(np.ones((s, s), dtype=bool), 1), -np.inf, sc)
        ref_lse = np.log(np.exp(sc - sc.max(1, keepdims=True)).sum(1)) + sc.max(1)
        assert np.abs(_np(lse[t]) - ref_lse).max() < 1e-3 * max(1.0, np.abs(ref_lse).max())
    dqkv = torch.empty(s, h + 2 * hkv, dtype=tdt, device=gpu_device)
    delta = torch.empty(a, s, dtype=torch.float32, device=gpu_device)
    partials = torch.empty(s, 2 * h, dtype=tdt, device=gpu_device) if with_partials else None
    po.po_op_attention_backward(code, qd, o, lse, dod, dqkv, delta, s, h, a, force_generic, n_kv_heads=akv,
                                partials=partials)
    rdq, rdk, rdv = so.attention_backward(d_o.astype(np.float64), q, k, v, probs, a)
    got = _np(dqkv)
    check_parity(got[:, :h], rdq, tol, "dQ")
    check_parity(got[:, h:h + hkv], rdk, tol, "dK")
    check_parity(got[:, h + hkv:], rdv, tol, "dV")


# grouped-query attention: key/value heads shared by groups of query heads
@pytest.mark.parametrize("dtype,s,h,a,akv,force_generic", [
    ("f32", 37, 128, 4, 2, 1), ("f32", 70, 192, 6, 1, 1), ("bf16", 130, 256, 4, 2, 1),
    ("bf16", 128, 256, 4, 2, 0), ("bf16", 384, 512, 4, 1, 0), ("bf16", 256, 512, 8, 2, 0),
    ("bf16", 640, 768, 6, 3, 0), ("bf16", 512, 1024, 16, 4, 0), ("bf16", 256, 256, 4, 4, 0),
    # 17 row blocks x 16 heads: more dQ blocks than CUs but fewer dK/dV blocks, so without the workspace the two
    # backward kernels have different block forms and go out as two launches; with it, as one launch of four-wave blocks
    ("bf16", 2176, 1024, 16, 2, 0)])
@pytest.mark.parametrize("with_partials", [False, True], ids=["direct", "per-head-then-sum"])
def test_grouped_query_attention(gpu_device, dtype, s, h, a, akv, force_generic, with_partials):
    _attention_case(gpu_device, dtype, s, h, a, force_generic, akv, with_partials)


def test_grouped_query_attention_rejects_bad_groups(gpu_device):
    t = torch.zeros(128, 3 * 256, dtype=torch.bfloat16, device=gpu_device)
    o = torch.zeros(128, 256, dtype=torch.bfloat16, device=gpu_device)
    lse = torch.zeros(4, 128, device=gpu_device)
    with pytest.raises(po.PipeOffloadError):
        po.po_op_attention_forward(po.PO_BF16, t, o, lse, 128, 256, 4, 0, n_kv_heads=3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,n", [(1, 2), (37, 130), (300, 1024)])
def test_colsum_accumulate(gpu_device, dtype, rows, n):
    code, tdt, tol = DT[dtype]
    rng = np.random.default_rng(rows + n)
    x = _rand(rng, (rows, n), dtype)
    acc0 = rng.standard_normal(n).astype(np.float32)
    acc = torch.from_numpy(acc0).to(gpu_device)
    ws = torch.empty(po.po_op_colsum_workspace(rows, n) // 4, dtype=torch.float32, device=gpu_device)
    po.po_op_colsum_accumulate(code, _dev(x, tdt, gpu_device), acc, ws, rows, n)
    assert max_rel_err(_np(acc) - acc0, x.astype(np.float64).sum(0)) < 1e-4


def test_pack_unpack_roundtrip_is_bit_exact(gpu_device):
    rng = np.random.default_rng(0)
    sizes = [16, 4096 + 16, 0, 1 << 20, 48, 3 * 16384 + 32]  # bytes, multiples of 16, one empty
    segs = [torch.from_numpy(rng.integers(0, 256, size=n, dtype=np.uint8)).to(gpu_device) for n in sizes]
    total = sum(sizes)
    packed = torch.zeros(total, dtype=torch.uint8, device=gpu_device)
    po.po_op_pack([(t if t.numel() else 0, n) for t, n in zip(segs, sizes)], packed)
    want = np.concatenate([t.cpu().numpy() for t in segs])
    assert np.array_equal(packed.cpu().numpy(), want)  # byte-exact: oracle = concatenation
    outs = [torch.zeros_like(t) for t in segs]
    po.po_op_unpack([(t if t.numel() else 0, n) for t, n in zip(outs, sizes)], packed)
    for a, b in zip(outs, segs):
        assert torch.equal(a, b)
    with pytest.raises(po.PipeOffloadError):
        po.po_op_pack([(segs[0], 8)], packed)  # not a multiple of 16
    po.po_op_pack([], packed)  # empty is a no-op


# ---- dropout with regenerated masks ------------------------------------------------------------------------------
@pytest.mark.parametrize("rows,cols,p,seed,layer,site,mb", [(37, 130, 0.1, 1234, 0, 0, 0), (64, 256, 0.25, 2 ** 40 + 7, 3, 1, 5),
                                                            (5, 7, 0.5, 1, 11, 0, 2), (300, 1024, 0.9, 99, 1, 1, 31)])
def test_dropout_mask_is_the_oracle_mask_bit_for_bit(gpu_device, rows, cols, p, seed, layer, site, mb):
    p = float(np.float32(p))  # the probability the library sees is the fp32 value
    x = torch.ones(rows, cols, dtype=torch.float32, device=gpu_device)
    out = torch.empty_like(x)
    po.po_op_dropout(po.PO_F32, x, out, rows, cols, p, seed, layer, site, mb)
    keep = so.dropout_keep_mask(seed, layer, site, mb, rows, cols, p)
    got = _np(out)
    assert np.array_equal(got != 0, keep)
    assert np.all(got[keep] == np.float32(1.0 / (1.0 - p)))
    # bf16 values through the same mask
    rng = np.random.default_rng(rows)
    v = _rand(rng, (rows, cols), "bf16")
    xb = _dev(v, torch.bfloat16, gpu_device)
    ob = torch.empty_like(xb)
    po.po_op_dropout(po.PO_BF16, xb, ob, rows, cols, p, seed, layer, site, mb)
    assert max_rel_err(_np(ob), v.astype(np.float64) * keep / (1.0 - p)) < 1e-2
