"""Pins for the stage-math oracle: everything here is checked against something
other than the oracle's own formulas (finite differences, an independently
composed torch-CPU model with autograd, brute-force loops, closed forms)."""
import math

import numpy as np
import pytest
import torch

from oracle import stage_oracle as so
from paper_2503_01328_amd import inputs as syn

TINY = syn.StageShape(n_layers=2, n_chunks=1, hidden=8, n_heads=2, ffn=16, seq=5, dtype="f32")


def _loss(params, shape, x, dy, vocab=0):
    y, _, _ = so.run_stage(params, shape.n_layers, shape.n_chunks, shape.n_heads, x, dy, vocab=vocab)
    return sum(float((y[u] * dy[u]).sum()) for u in y)


def _tiny_problem(shape, m=2, seed=7, scale=8.0):
    params = syn.stage_params(shape, seed)
    # larger weights than N(0, 0.02) so that every path carries signal at h = 8
    for p in params["layers"]:
        for k in p:
            if not k.startswith("ln"):
                p[k] = (p[k] * scale).astype(np.float64)
            else:
                p[k] = p[k].astype(np.float64)
    for k in ("wte", "wpe"):
        if k in params:
            params[k] = (params[k] * 20).astype(np.float64)
    x = {(j, c): syn.unit_input(shape, j, c, seed) for j in range(m) for c in range(shape.n_chunks)}
    x = {u: (a if a.dtype == np.int32 else a.astype(np.float64)) for u, a in x.items()}
    dy = {(j, c): syn.unit_upstream_grad(shape, j, c, seed).astype(np.float64) for j in range(m) for c in range(shape.n_chunks)}
    return params, x, dy


def test_finite_differences_every_parameter_and_input():
    shape = TINY
    params, x, dy = _tiny_problem(shape)
    _, dx, grads = so.run_stage(params, shape.n_layers, 1, shape.n_heads, x, dy)
    eps = 1e-6
    rng = np.random.default_rng(0)
    for l, p in enumerate(params["layers"]):
        for name, a in p.items():
            flat = a.reshape(-1)
            for idx in rng.choice(flat.size, size=min(6, flat.size), replace=False):
                old = flat[idx]
                flat[idx] = old + eps
                lp = _loss(params, shape, x, dy)
                flat[idx] = old - eps
                lm = _loss(params, shape, x, dy)
                flat[idx] = old
                fd = (lp - lm) / (2 * eps)
                an = grads["layers"][l][name].reshape(-1)[idx]
                assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (l, name, idx, fd, an)
    for u in x:
        flat = x[u].reshape(-1)
        for idx in rng.choice(flat.size, size=8, replace=False):
            old = flat[idx]
            flat[idx] = old + eps
            lp = _loss(params, shape, x, dy)
            flat[idx] = old - eps
            lm = _loss(params, shape, x, dy)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            an = dx[u].reshape(-1)[idx]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an))


def test_finite_differences_embedding():
    shape = syn.StageShape(1, 1, 8, 2, 16, 6, vocab=5, dtype="f32")
    params, x, dy = _tiny_problem(shape)
    assert x[(0, 0)].dtype == np.int32
    _, dx, grads = so.run_stage(params, 1, 1, 2, x, dy, vocab=5)
    assert dx[(0, 0)] is None
    eps = 1e-6
    rng = np.random.default_rng(1)
    for name in ("wte", "wpe"):
        flat = params[name].reshape(-1)
        for idx in rng.choice(flat.size, size=12, replace=False):
            old = flat[idx]
            flat[idx] = old + eps
            lp = _loss(params, shape, x, dy, vocab=5)
            flat[idx] = old - eps
            lm = _loss(params, shape, x, dy, vocab=5)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            an = grads[name].reshape(-1)[idx]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, idx)
    # repeated tokens must accumulate: a token that never occurs has zero gradient
    tok = x[(0, 0)]
    for t in range(5):
        if t not in set(tok.tolist()) and t not in set(x[(1, 0)].tolist()):
            assert np.all(grads["wte"][t] == 0)


def _torch_layer(x, p, a, eps):
    """Independent composition of the same layer from torch library routines."""
    import torch.nn.functional as F

    h = x.shape[1]
    dh = h // a
    n1 = F.layer_norm(x, (h,), p["ln1_g"], p["ln1_b"], eps)
    qkv = F.linear(n1, p["w_qkv"].t(), p["b_qkv"])
    q, k, v = qkv.split(h, dim=1)
    s = x.shape[0]
    hd = lambda t: t.reshape(s, a, dh).transpose(0, 1).unsqueeze(0)
    o = F.scaled_dot_product_attention(hd(q), hd(k), hd(v), is_causal=True)
    o = o.squeeze(0).transpose(0, 1).reshape(s, h)
    x1 = x + F.linear(o, p["w_o"].t(), p["b_o"])
    n2 = F.layer_norm(x1, (h,), p["ln2_g"], p["ln2_b"], eps)
    u = F.linear(n2, p["w_fc1"].t(), p["b_fc1"])
    return x1 + F.linear(F.gelu(u, approximate="tanh"), p["w_fc2"].t(), p["b_fc2"])


def test_against_torch_library_model_with_autograd():
    shape = syn.StageShape(2, 1, 32, 4, 64, 24, dtype="f32")
    params, x, dy = _tiny_problem(shape, m=2, seed=3, scale=5.0)
    y, dx, grads = so.run_stage(params, 2, 1, 4, x, dy)
    tp = [{k: torch.tensor(a, dtype=torch.float64, requires_grad=True) for k, a in p.items()} for p in params["layers"]]
    total = 0
    for u in sorted(x):
        xt = torch.tensor(x[u], dtype=torch.float64, requires_grad=True)
        t = xt
        for p in tp:
            t = _torch_layer(t, p, 4, 1e-5)
        np.testing.assert_allclose(t.detach().numpy(), y[u], rtol=1e-10, atol=1e-10)
        loss = (t * torch.tensor(dy[u])).sum()
        (gx,) = torch.autograd.grad(loss, xt, retain_graph=True)
        np.testing.assert_allclose(gx.numpy(), dx[u], rtol=1e-9, atol=1e-10)
        total = total + loss
    total.backward()
    for l, p in enumerate(tp):
        for k, t in p.items():
            np.testing.assert_allclose(t.grad.numpy(), grads["layers"][l][k], rtol=1e-9, atol=1e-10, err_msg=f"{l}.{k}")


def test_attention_brute_force_loops():
    rng = np.random.default_rng(5)
    s, a, dh = 6, 2, 3
    q, k, v = (rng.standard_normal((s, a * dh)) for _ in range(3))
    o, probs = so.attention_forward(q, k, v, a)
    for t in range(a):
        for i in range(s):
            w = [math.exp(sum(q[i, t * dh + e] * k[j, t * dh + e] for e in range(dh)) / math.sqrt(dh)) for j in range(i + 1)]
            z = sum(w)
            for e in range(dh):
                ref = sum(w[j] / z * v[j, t * dh + e] for j in range(i + 1))
                assert abs(ref - o[i, t * dh + e]) < 1e-12
            assert abs(probs[t][i].sum() - 1) < 1e-12
            assert np.all(probs[t][i, i + 1:] == 0)
        assert probs[t][0, 0] == 1.0


def test_causality_future_inputs_do_not_change_past_outputs():
    shape = TINY
    params, x, dy = _tiny_problem(shape, m=1)
    y0, _ = so.unit_forward(params, [0, 1], x[(0, 0)], 2)
    x2 = x[(0, 0)].copy()
    x2[3:] += 1.0
    y1, _ = so.unit_forward(params, [0, 1], x2, 2)
    np.testing.assert_array_equal(y0[:3], y1[:3])
    assert np.abs(y0[3:] - y1[3:]).max() > 1e-3


def test_identity_stage_when_output_projections_are_zero():
    shape = TINY
    params, x, dy = _tiny_problem(shape, m=1)
    for p in params["layers"]:
        for k in ("w_o", "b_o", "w_fc2", "b_fc2"):
            p[k][...] = 0
    y, dx, grads = so.run_stage(params, 2, 1, 2, x, dy)
    np.testing.assert_array_equal(y[(0, 0)], x[(0, 0)])
    np.testing.assert_array_equal(dx[(0, 0)], dy[(0, 0)])
    assert np.all(grads["layers"][0]["w_qkv"] == 0)  # nothing upstream of a zero projection learns


def test_single_token_layer_reduces_to_mlp_with_residual():
    # with s = 1 the softmax is 1 and O = v: x1 = x + (LN1(x) Wv + bv) Wo + bo
    shape = syn.StageShape(1, 1, 8, 2, 16, 1, dtype="f32")
    params, x, dy = _tiny_problem(shape, m=1)
    p = params["layers"][0]
    xx = x[(0, 0)]
    h = 8
    mu, var = xx.mean(), xx.var()
    n1 = (xx - mu) / math.sqrt(var + 1e-5) * p["ln1_g"] + p["ln1_b"]
    vv = n1 @ p["w_qkv"][:, 2 * h:] + p["b_qkv"][2 * h:]
    x1 = xx + vv @ p["w_o"] + p["b_o"]
    n2 = (x1 - x1.mean()) / math.sqrt(x1.var() + 1e-5) * p["ln2_g"] + p["ln2_b"]
    u = n2 @ p["w_fc1"] + p["b_fc1"]
    g = np.array([[0.5 * t * (1 + math.tanh(math.sqrt(2 / math.pi) * (t + 0.044715 * t ** 3))) for t in u[0]]])
    ref = x1 + g @ p["w_fc2"] + p["b_fc2"]
    y, _ = so.unit_forward(params, [0], xx, 2)
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    # q and k cannot matter when there is a single key
    _, _, grads = so.run_stage(params, 1, 1, 2, x, dy)
    assert np.abs(grads["layers"][0]["w_qkv"][:, : 2 * h]).max() < 1e-14
    assert np.abs(grads["layers"][0]["w_qkv"][:, 2 * h:]).max() > 1e-6


def test_layernorm_moments_and_backward_orthogonality():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 16)) * 3 + 1
    n, cache = so.layernorm_forward(x, np.ones(16), np.zeros(16), 1e-5)
    assert np.abs(n.mean(axis=1)).max() < 1e-12
    np.testing.assert_allclose(n.var(axis=1), x.var(axis=1) / (x.var(axis=1) + 1e-5), rtol=1e-12)
    dn = rng.standard_normal((7, 16))
    dx, dg, db = so.layernorm_backward(dn, cache, np.ones(16))
    assert np.abs(dx.sum(axis=1)).max() < 1e-12
    # with eps = 0 the normalised row has unit second moment and dx is orthogonal to it
    _, cache = so.layernorm_forward(x, np.ones(16), np.zeros(16), 0.0)
    dx, dg, db = so.layernorm_backward(dn, cache, np.ones(16))
    assert np.abs((dx * cache[0]).sum(axis=1)).max() < 1e-12
    np.testing.assert_allclose(db, dn.sum(axis=0))


def test_gelu_values_and_derivative():
    # values of the tanh form at a few points, computed by hand from its definition
    assert so.gelu(np.array([0.0]))[0] == 0.0
    assert abs(so.gelu(np.array([1.0]))[0] - 0.8411919906082768) < 1e-15
    assert abs(so.gelu(np.array([-1.0]))[0] + 0.15880800939172324) < 1e-15
    assert abs(so.gelu(np.array([10.0]))[0] - 10.0) < 1e-12
    u = np.linspace(-4, 4, 41)
    fd = (so.gelu(u + 1e-6) - so.gelu(u - 1e-6)) / 2e-6
    np.testing.assert_allclose(so.gelu_derivative(u), fd, atol=1e-8)
    torch_ref = torch.nn.functional.gelu(torch.tensor(u), approximate="tanh").numpy()
    np.testing.assert_allclose(so.gelu(u), torch_ref, rtol=1e-13, atol=1e-15)


def test_gradient_is_additive_over_microbatches():
    shape = TINY
    params, x, dy = _tiny_problem(shape, m=3)
    _, _, total = so.run_stage(params, 2, 1, 2, x, dy)
    parts = [so.run_stage(params, 2, 1, 2, {u: x[u]}, {u: dy[u]})[2] for u in sorted(x)]
    for l in range(2):
        for k in total["layers"][l]:
            np.testing.assert_allclose(total["layers"][l][k], sum(p["layers"][l][k] for p in parts), rtol=1e-12, atol=1e-14)


def test_two_chunks_compose_to_the_unchunked_stage():
    shape2 = syn.StageShape(2, 2, 8, 2, 16, 5, dtype="f32")
    params, x1, dy1 = _tiny_problem(TINY, m=1)
    y_full, dx_full, g_full = so.run_stage(params, 2, 1, 2, x1, dy1)
    # chunk 0 alone, then chunk 1 fed chunk 0's output; backward in reverse
    y0, tape0 = so.unit_forward(params, [0], x1[(0, 0)], 2)
    y1, tape1 = so.unit_forward(params, [1], y0, 2)
    np.testing.assert_allclose(y1, y_full[(0, 0)], rtol=1e-13)
    d1, g1 = so.unit_backward(params, tape1, dy1[(0, 0)], 2)
    d0, g0 = so.unit_backward(params, tape0, d1, 2)
    np.testing.assert_allclose(d0, dx_full[(0, 0)], rtol=1e-12)
    # and through run_stage's chunk interface
    y, dx, g = so.run_stage(params, 2, 2, 2, {(0, 0): x1[(0, 0)], (0, 1): y0}, {(0, 0): d1, (0, 1): dy1[(0, 0)]})
    np.testing.assert_allclose(dx[(0, 0)], dx_full[(0, 0)], rtol=1e-12)
    for l in range(2):
        for k in g_full["layers"][l]:
            np.testing.assert_allclose(g["layers"][l][k], g_full["layers"][l][k], rtol=1e-11, atol=1e-14)
    assert shape2.layers_per_chunk == 1


def test_float32_instantiation_agrees_with_float64():
    shape = syn.StageShape(2, 1, 64, 4, 256, 32, dtype="f32")
    params = syn.stage_params(shape, 11)
    x = {(0, 0): syn.unit_input(shape, 0, 0, 11)}
    dy = {(0, 0): syn.unit_upstream_grad(shape, 0, 0, 11)}
    y64, dx64, g64 = so.run_stage(params, 2, 1, 4, x, dy, dtype=np.float64)
    y32, dx32, g32 = so.run_stage(params, 2, 1, 4, x, dy, dtype=np.float32)
    assert y32[(0, 0)].dtype == np.float32
    rel = lambda a, b: np.abs(a - b).max() / np.abs(b).max()
    assert rel(y32[(0, 0)], y64[(0, 0)]) < 1e-5
    assert rel(dx32[(0, 0)], dx64[(0, 0)]) < 1e-5
    for l in range(2):
        for k in g64["layers"][l]:
            assert rel(g32["layers"][l][k], g64["layers"][l][k]) < 2e-5, (l, k)


def test_bf16_rounding_helper_is_round_to_nearest_even():
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 3.14159], dtype=np.float32)
    r = syn.round_to_bf16(a)
    ref = torch.tensor(a).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, ref)
    np.testing.assert_array_equal(syn.bf16_bits_to_f32(syn.bf16_bits(r)), r)


# ---- grouped-query attention (Table 2: query groups) ----------------------------------------------------------
GQA_TINY = syn.StageShape(n_layers=2, n_chunks=1, hidden=16, n_heads=4, ffn=32, seq=6, dtype="f32", n_kv_heads=2)


def _replicate_kv(params, shape):
    """The multi-head model that computes the same function: every query head gets its own copy of its group's
    key and value projection columns."""
    h, dh, a, akv = shape.hidden, shape.head_dim, shape.n_heads, shape.kv_heads
    group, hkv = a // akv, shape.kv_width
    out = {"layers": []}
    for p in params["layers"]:
        q = dict(p)
        w, b = p["w_qkv"], p["b_qkv"]
        cols = list(range(h))
        for block in (h, h + hkv):
            for t in range(a):
                cols += list(range(block + (t // group) * dh, block + (t // group + 1) * dh))
        q["w_qkv"], q["b_qkv"] = w[:, cols].copy(), b[cols].copy()
        out["layers"].append(q)
    return out


def test_grouped_query_attention_equals_multi_head_with_replicated_kv_weights():
    shape = GQA_TINY
    params, x, dy = _tiny_problem(shape, m=2, seed=11, scale=6.0)
    assert params["layers"][0]["w_qkv"].shape == (16, 16 + 2 * 8)
    y, dx, g = so.run_stage(params, shape.n_layers, 1, shape.n_heads, x, dy)
    ym, dxm, gm = so.run_stage(_replicate_kv(params, shape), shape.n_layers, 1, shape.n_heads, x, dy)
    h, dh, group, hkv = 16, 4, 2, 8
    for u in y:
        np.testing.assert_allclose(y[u], ym[u], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(dx[u], dxm[u], rtol=1e-11, atol=1e-12)
    for l in range(shape.n_layers):
        for k in g["layers"][l]:
            if k in ("w_qkv", "b_qkv"):
                continue
            np.testing.assert_allclose(g["layers"][l][k], gm["layers"][l][k], rtol=1e-10, atol=1e-12, err_msg=k)
        # a shared key/value column receives the sum of the gradients of its copies (chain rule through the copy)
        for name in ("w_qkv", "b_qkv"):
            full = gm["layers"][l][name]
            got = g["layers"][l][name]
            np.testing.assert_allclose(got[..., :h], full[..., :h], rtol=1e-10, atol=1e-12)
            for blk in range(2):
                for kvh in range(2):
                    want = sum(full[..., h + blk * h + t * dh: h + blk * h + (t + 1) * dh]
                               for t in range(kvh * group, (kvh + 1) * group))
                    np.testing.assert_allclose(got[..., h + blk * hkv + kvh * dh: h + blk * hkv + (kvh + 1) * dh], want,
                                               rtol=1e-10, atol=1e-12)


def test_grouped_query_attention_finite_differences():
    shape = GQA_TINY
    params, x, dy = _tiny_problem(shape, m=1, seed=5, scale=6.0)
    _, dx, grads = so.run_stage(params, shape.n_layers, 1, shape.n_heads, x, dy)
    eps = 1e-6
    rng = np.random.default_rng(1)
    for l, p in enumerate(params["layers"]):
        for name in ("w_qkv", "b_qkv", "w_o"):
            flat = p[name].reshape(-1)
            for idx in rng.choice(flat.size, size=10, replace=False):
                old = flat[idx]
                flat[idx] = old + eps
                lp = _loss(params, shape, x, dy)
                flat[idx] = old - eps
                lm = _loss(params, shape, x, dy)
                flat[idx] = old
                an = grads["layers"][l][name].reshape(-1)[idx]
                assert abs((lp - lm) / (2 * eps) - an) <= 1e-6 * max(1.0, abs(an)), (l, name, idx)


def test_grouped_query_attention_against_torch_sdpa():
    import torch.nn.functional as F

    s, a, akv, dh = 7, 6, 2, 4
    rng = np.random.default_rng(2)
    q, k, v = rng.standard_normal((s, a * dh)), rng.standard_normal((s, akv * dh)), rng.standard_normal((s, akv * dh))
    do = rng.standard_normal((s, a * dh))
    o, probs = so.attention_forward(q, k, v, a)
    dq, dk, dv = so.attention_backward(do, q, k, v, probs, a)
    tq, tk, tv = (torch.tensor(t, requires_grad=True) for t in (q, k, v))
    hd = lambda t, n: t.reshape(s, n, dh).transpose(0, 1)
    to = F.scaled_dot_product_attention(hd(tq, a), hd(tk, akv).repeat_interleave(a // akv, dim=0),
                                        hd(tv, akv).repeat_interleave(a // akv, dim=0), is_causal=True)
    to = to.transpose(0, 1).reshape(s, a * dh)
    np.testing.assert_allclose(to.detach().numpy(), o, rtol=1e-12, atol=1e-12)
    (to * torch.tensor(do)).sum().backward()
    for got, want in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-11, atol=1e-12)


# ---- dropout with regenerated masks (Appendix C: dropout is recomputed) ---------------------------------------
def test_philox4x32_10_known_answers():
    # the three known-answer vectors distributed with the reference implementation of Philox (Random123):
    # zero counter and key, all-ones, and the digits of pi
    cases = [((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
             ((0xffffffff,) * 4, (0xffffffff,) * 2, (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
             ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
              (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1))]
    for ctr, key, want in cases:
        assert tuple(int(x) for x in so.philox4x32_10(ctr, key)) == want


def test_dropout_mask_statistics_and_addressing():
    p = 0.1
    m = so.dropout_keep_mask(1234, 3, 1, 5, 512, 384, p)
    assert m.shape == (512, 384) and abs(m.mean() - 0.9) < 5e-3
    # rows, columns, layers, sites, microbatches and seeds all give different, uncorrelated masks
    others = [so.dropout_keep_mask(1234, 3, 0, 5, 512, 384, p), so.dropout_keep_mask(1234, 4, 1, 5, 512, 384, p),
              so.dropout_keep_mask(1234, 3, 1, 6, 512, 384, p), so.dropout_keep_mask(1235, 3, 1, 5, 512, 384, p),
              so.dropout_keep_mask(2 ** 40 + 1234, 3, 1, 5, 512, 384, p)]
    for o in others:
        both_dropped = (~m & ~o).mean()
        assert abs(both_dropped - p * p) < 3e-3
    assert abs((~m[:-1] & ~m[1:]).mean() - p * p) < 3e-3 and abs((~m[:, :-1] & ~m[:, 1:]).mean() - p * p) < 3e-3
    # element (r, c) is word c % 4 of the block at counter (c // 4, r, 2 layer + site, mb)
    w = so.philox4x32_10((np.uint32(70 // 4), np.uint32(9), np.uint32(7), np.uint32(5)), (1234, 0))
    assert m[9, 70] == (int(w[70 % 4]) >= so.dropout_threshold(p))
    # a sub-block is the same function of the absolute position; p = 0 keeps everything
    assert np.array_equal(so.dropout_keep_mask(1234, 3, 1, 5, 100, 50, p), m[:100, :50])
    assert so.dropout_keep_mask(1, 0, 0, 0, 8, 8, 0.0).all()


def test_dropout_stage_finite_differences_and_expectation():
    shape = TINY
    params, x, dy = _tiny_problem(shape, m=2)
    kw = dict(dropout_p=0.3, seed=99)
    y, dx, grads = so.run_stage(params, shape.n_layers, 1, shape.n_heads, x, dy, **kw)
    y0, _, _ = so.run_stage(params, shape.n_layers, 1, shape.n_heads, x, dy)
    assert any(np.abs(y[u] - y0[u]).max() > 1e-3 for u in y)  # the masks do something
    loss = lambda: sum(float((v * dy[u]).sum()) for u, v in
                       so.run_stage(params, shape.n_layers, 1, shape.n_heads, x, dy, **kw)[0].items())
    eps = 1e-6
    rng = np.random.default_rng(3)
    for l, p in enumerate(params["layers"]):
        for name in ("w_o", "b_o", "w_fc2", "b_fc2", "w_qkv", "w_fc1", "ln2_g"):
            flat = p[name].reshape(-1)
            for idx in rng.choice(flat.size, size=5, replace=False):
                old = flat[idx]
                flat[idx] = old + eps
                lp = loss()
                flat[idx] = old - eps
                lm = loss()
                flat[idx] = old
                an = grads["layers"][l][name].reshape(-1)[idx]
                assert abs((lp - lm) / (2 * eps) - an) <= 1e-6 * max(1.0, abs(an)), (l, name, idx)
    u = (0, 0)
    flat = x[u].reshape(-1)
    for idx in rng.choice(flat.size, size=8, replace=False):
        old = flat[idx]
        flat[idx] = old + eps
        lp = loss()
        flat[idx] = old - eps
        lm = loss()
        flat[idx] = old
        assert abs((lp - lm) / (2 * eps) - dx[u].reshape(-1)[idx]) <= 1e-6 * max(1.0, abs(dx[u].reshape(-1)[idx]))


def test_dropout_layer_against_torch_with_the_same_masks():
    import torch.nn.functional as F

    shape = syn.StageShape(1, 1, 32, 4, 64, 24, dtype="f32")
    params, x, dy = _tiny_problem(shape, m=1, seed=4, scale=5.0)
    prob, seed = 0.25, 7
    y, dx, grads = so.run_stage(params, 1, 1, 4, x, dy, dropout_p=prob, seed=seed)
    m1 = torch.tensor(so.dropout_keep_mask(seed, 0, 0, 0, 24, 32, prob), dtype=torch.float64) / (1 - prob)
    m2 = torch.tensor(so.dropout_keep_mask(seed, 0, 1, 0, 24, 32, prob), dtype=torch.float64) / (1 - prob)
    p = {k: torch.tensor(a, dtype=torch.float64, requires_grad=True) for k, a in params["layers"][0].items()}
    xt = torch.tensor(x[(0, 0)], dtype=torch.float64, requires_grad=True)
    h, a, dh, s = 32, 4, 8, 24
    n1 = F.layer_norm(xt, (h,), p["ln1_g"], p["ln1_b"], 1e-5)
    q, k, v = F.linear(n1, p["w_qkv"].t(), p["b_qkv"]).split(h, dim=1)
    hd = lambda t: t.reshape(s, a, dh).transpose(0, 1).unsqueeze(0)
    o = F.scaled_dot_product_attention(hd(q), hd(k), hd(v), is_causal=True).squeeze(0).transpose(0, 1).reshape(s, h)
    x1 = xt + F.linear(o, p["w_o"].t(), p["b_o"]) * m1
    n2 = F.layer_norm(x1, (h,), p["ln2_g"], p["ln2_b"], 1e-5)
    out = x1 + F.linear(F.gelu(F.linear(n2, p["w_fc1"].t(), p["b_fc1"]), approximate="tanh"), p["w_fc2"].t(), p["b_fc2"]) * m2
    np.testing.assert_allclose(out.detach().numpy(), y[(0, 0)], rtol=1e-10, atol=1e-10)
    (out * torch.tensor(dy[(0, 0)])).sum().backward()
    np.testing.assert_allclose(xt.grad.numpy(), dx[(0, 0)], rtol=1e-9, atol=1e-10)
    for kname, t in p.items():
        np.testing.assert_allclose(t.grad.numpy(), grads["layers"][0][kname], rtol=1e-9, atol=1e-10, err_msg=kname)
