"""CPU oracle for one pipeline stage's transformer-layer forward and backward.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module;
it exists so that tests, the smoke check and the benchmark's CPU-baseline leg
have an independent statement of what the HIP path must compute.  It shares no
code with the HIP path and never reads anything the HIP path produced.

What it computes.  The paper's offload method is exact (Section 5, convergence
paragraph: the schedules change when tensors live where, never their values;
Appendix C: LayerNorm and GeLU are recomputed in backward, which is the same
function evaluated twice).  The oracle is therefore the plain definition:
the gradients of a GPT-style pre-LayerNorm decoder stage (Section 5: GPT-3-like
models), summed over microbatches, with no notion of offload, recomputation,
tiling or fusion.  Every function below is the textbook formula written with
numpy array operations; matmul is used as a library primitive.

Readings of points the paper leaves open (each is also listed in the design
notes): pre-LN decoder layer; LayerNorm with gain and shift, biased variance,
eps inside the square root; linear layers with bias; GeLU in its tanh form;
causal softmax attention scaled by 1/sqrt(head_dim), multi-head, or grouped-query
when the QKV projection is narrower than 3h (Table 2's query groups); dropout
off by default, on request the two hidden dropouts (after the attention and
the MLP output projections) with regenerated masks; no final LayerNorm; learned token + position embedding when the stage
is the first one.

Precision: ``dtype`` is numpy float64 by default (reference), float32 on
request (the "plain fp32 CPU stage" used as timed CPU baseline).

Pins (tests/test_oracle_*.py): central finite differences of every parameter
and of the input in float64; an independently composed torch-CPU forward with
autograd; brute-force Python loops for attention on tiny shapes; closed forms
(identity stage, s = 1, LayerNorm moments and orthogonality, softmax rows,
causality); additivity over microbatches; chunk composition.
"""
from __future__ import annotations

import math

import numpy as np

SQRT_2_OVER_PI = math.sqrt(2.0 / math.pi)
GELU_CUBIC = 0.044715


# --------------------------------------------------------------------------- #
# LayerNorm (recomputed in backward by the method, Appendix C; here: plain)
# --------------------------------------------------------------------------- #
def layernorm_forward(x, gain, shift, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + x.dtype.type(eps))
    xhat = (x - mu) * rstd
    return xhat * gain + shift, (xhat, rstd)


def layernorm_backward(dn, cache, gain):
    xhat, rstd = cache
    dxhat = dn * gain
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True) - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, (dn * xhat).sum(axis=0), dn.sum(axis=0)


# --------------------------------------------------------------------------- #
# GeLU, tanh form (recomputed in backward by the method, Appendix C)
# --------------------------------------------------------------------------- #
def gelu(u):
    return 0.5 * u * (1.0 + np.tanh(SQRT_2_OVER_PI * (u + GELU_CUBIC * u ** 3)))


def gelu_derivative(u):
    t = np.tanh(SQRT_2_OVER_PI * (u + GELU_CUBIC * u ** 3))
    dz = SQRT_2_OVER_PI * (1.0 + 3.0 * GELU_CUBIC * u ** 2)
    return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * dz


# --------------------------------------------------------------------------- #
# Causal multi-head attention (the s-dependent term of Eq. 1's compute time)
# --------------------------------------------------------------------------- #
def attention_forward(q, k, v, n_heads):
    """q: [s, h]; k, v: [s, h_kv] with h_kv = n_kv_heads * dh.  Query head t owns
    columns [t*dh, (t+1)*dh) of q and reads key/value head t // (n_heads // n_kv_heads)
    (grouped-query attention, Table 2's "query groups"; n_kv_heads = n_heads is plain
    multi-head attention).  Returns O [s, h] and the per-head probability matrices
    (kept only by the oracle)."""
    s, h = q.shape
    dh = h // n_heads
    group = n_heads // (k.shape[1] // dh)
    scale = q.dtype.type(1.0 / math.sqrt(dh))
    o = np.empty_like(q)
    probs = []
    future = np.triu(np.ones((s, s), dtype=bool), k=1)  # j > i
    for t in range(n_heads):
        c = slice(t * dh, (t + 1) * dh)
        ckv = slice((t // group) * dh, (t // group + 1) * dh)
        sc = (q[:, c] @ k[:, ckv].T) * scale
        sc = np.where(future, -np.inf, sc)
        sc = sc - sc.max(axis=-1, keepdims=True)
        p = np.exp(sc)
        p = p / p.sum(axis=-1, keepdims=True)
        o[:, c] = p @ v[:, ckv]
        probs.append(p.astype(q.dtype))
    return o, probs


def attention_backward(do, q, k, v, probs, n_heads):
    s, h = q.shape
    dh = h // n_heads
    group = n_heads // (k.shape[1] // dh)
    scale = q.dtype.type(1.0 / math.sqrt(dh))
    dq, dk, dv = np.empty_like(q), np.zeros_like(k), np.zeros_like(v)
    for t in range(n_heads):  # a key/value head collects the gradients of its query heads in head order
        c = slice(t * dh, (t + 1) * dh)
        ckv = slice((t // group) * dh, (t // group + 1) * dh)
        p = probs[t]
        dv[:, ckv] += p.T @ do[:, c]
        dp = do[:, c] @ v[:, ckv].T
        ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
        dq[:, c] = (ds @ k[:, ckv]) * scale
        dk[:, ckv] += (ds.T @ q[:, c]) * scale
    return dq, dk, dv


# --------------------------------------------------------------------------- #
# Dropout whose mask is a function of (seed, layer, site, microbatch, position),
# so that the backward regenerates it instead of storing it (Appendix C: dropout
# is among the recomputed operations).  The generator is the published
# counter-based Philox4x32-10 (Salmon et al., SC'11); the HIP path implements the
# same generator on its own.
# --------------------------------------------------------------------------- #
_PHILOX_M0, _PHILOX_M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key):
    """counter: four uint32 arrays (broadcastable), key: two uint32 scalars.  Ten
    rounds of: (hi, lo) products of words 0 and 2 with the two multipliers, mixed
    with words 1 and 3 and the round key; the key advances by the Weyl constants."""
    c = [np.asarray(x, dtype=np.uint32) for x in counter]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = c[0].astype(np.uint64) * _PHILOX_M0
        p1 = c[2].astype(np.uint64) * _PHILOX_M1
        hi0, lo0 = (p0 >> np.uint64(32)).astype(np.uint32), p0.astype(np.uint32)
        hi1, lo1 = (p1 >> np.uint64(32)).astype(np.uint32), p1.astype(np.uint32)
        c = [hi1 ^ c[1] ^ np.uint32(k0), lo1, hi0 ^ c[3] ^ np.uint32(k1), lo0]
        k0, k1 = (k0 + _PHILOX_W0) & 0xFFFFFFFF, (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return c


def dropout_threshold(p):
    """An element is kept iff its 32-bit random word is >= this value."""
    return min(int(math.floor(p * 2.0 ** 32 + 0.5)), 2 ** 32 - 1)


def dropout_keep_mask(seed, layer, site, mb, rows, cols, p):
    """Boolean [rows, cols] keep mask of one dropout site (0: after the attention
    output projection, 1: after the MLP output projection) of global layer
    ``layer`` for microbatch ``mb``.  Element (r, c) uses word c % 4 of
    Philox4x32-10 with counter (c // 4, r, 2 * layer + site, mb) and key
    (seed mod 2^32, seed div 2^32)."""
    r = np.arange(rows, dtype=np.uint32)[:, None]
    c4 = np.arange((cols + 3) // 4, dtype=np.uint32)[None, :]
    words = philox4x32_10((c4, r, np.uint32(2 * layer + site), np.uint32(mb)), (seed & 0xFFFFFFFF, seed >> 32))
    w = np.stack([np.broadcast_to(x, (rows, c4.shape[1])) for x in words], axis=-1).reshape(rows, -1)[:, :cols]
    return w >= np.uint32(dropout_threshold(p))


# --------------------------------------------------------------------------- #
# One decoder layer
# --------------------------------------------------------------------------- #
def layer_forward(x, p, n_heads, eps, drop=None):
    """drop: None, or (keep mask of site 0, keep mask of site 1, 1 / (1 - p)): the two
    projections' outputs (bias included) are masked and rescaled before the residual
    is added."""
    h = x.shape[1]
    n1, ln1 = layernorm_forward(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = n1 @ p["w_qkv"] + p["b_qkv"]
    h_kv = (qkv.shape[1] - h) // 2  # w_qkv is [h, h + 2 h_kv]: query block, key block, value block
    q, k, v = qkv[:, :h], qkv[:, h:h + h_kv], qkv[:, h + h_kv:]
    o, probs = attention_forward(q, k, v, n_heads)
    z1 = o @ p["w_o"] + p["b_o"]
    if drop is not None:
        z1 = z1 * drop[0] * x.dtype.type(drop[2])
    x1 = x + z1
    n2, ln2 = layernorm_forward(x1, p["ln2_g"], p["ln2_b"], eps)
    u = n2 @ p["w_fc1"] + p["b_fc1"]
    g = gelu(u)
    z2 = g @ p["w_fc2"] + p["b_fc2"]
    if drop is not None:
        z2 = z2 * drop[1] * x.dtype.type(drop[2])
    y = x1 + z2
    cache = dict(n1=n1, ln1=ln1, q=q, k=k, v=v, probs=probs, o=o, n2=n2, ln2=ln2, u=u, g=g, drop=drop)
    return y, cache


def layer_backward(dy, p, c, n_heads):
    grads = {}
    drop = c.get("drop")
    # y = x1 + D2(g W2 + b2)
    dz2 = dy if drop is None else dy * drop[1] * dy.dtype.type(drop[2])
    grads["w_fc2"] = c["g"].T @ dz2
    grads["b_fc2"] = dz2.sum(axis=0)
    dg = dz2 @ p["w_fc2"].T
    du = dg * gelu_derivative(c["u"])
    grads["w_fc1"] = c["n2"].T @ du
    grads["b_fc1"] = du.sum(axis=0)
    dn2 = du @ p["w_fc1"].T
    dx1_ln, grads["ln2_g"], grads["ln2_b"] = layernorm_backward(dn2, c["ln2"], p["ln2_g"])
    dx1 = dy + dx1_ln
    # x1 = x + D1(O Wo + bo)
    dz1 = dx1 if drop is None else dx1 * drop[0] * dx1.dtype.type(drop[2])
    grads["w_o"] = c["o"].T @ dz1
    grads["b_o"] = dz1.sum(axis=0)
    do = dz1 @ p["w_o"].T
    dq, dk, dv = attention_backward(do, c["q"], c["k"], c["v"], c["probs"], n_heads)
    dqkv = np.concatenate([dq, dk, dv], axis=1)
    grads["w_qkv"] = c["n1"].T @ dqkv
    grads["b_qkv"] = dqkv.sum(axis=0)
    dn1 = dqkv @ p["w_qkv"].T
    dx_ln, grads["ln1_g"], grads["ln1_b"] = layernorm_backward(dn1, c["ln1"], p["ln1_g"])
    return dx1 + dx_ln, grads


# --------------------------------------------------------------------------- #
# One unit = one (microbatch, chunk): Lu consecutive layers, optional embedding
# --------------------------------------------------------------------------- #
def _cast_layer(p, dtype):
    return {k: np.asarray(a, dtype=dtype) for k, a in p.items()}


def unit_forward(params, layer_ids, x_in, n_heads, eps=1e-5, dtype=np.float64, embed=False, dropout=None):
    """x_in: [s, h] activations, or int tokens [s] when ``embed``.  Returns
    (y, tape) where the tape is what unit_backward needs."""
    tape = {"layers": [], "embed": None}
    if embed:
        tok = np.asarray(x_in)
        wte = np.asarray(params["wte"], dtype=dtype)
        wpe = np.asarray(params["wpe"], dtype=dtype)
        x = wte[tok] + wpe[: tok.shape[0]]
        tape["embed"] = tok
    else:
        x = np.asarray(x_in, dtype=dtype)
    for l in layer_ids:
        p = _cast_layer(params["layers"][l], dtype)
        drop = None
        if dropout is not None:  # (p, seed, mb)
            prob, seed, mb = dropout
            rows, cols = x.shape
            drop = (dropout_keep_mask(seed, l, 0, mb, rows, cols, prob), dropout_keep_mask(seed, l, 1, mb, rows, cols, prob),
                    1.0 / (1.0 - prob))
        x, cache = layer_forward(x, p, n_heads, eps, drop)
        tape["layers"].append((l, p, cache))
    return x, tape


def unit_backward(params, tape, dy, n_heads, dtype=np.float64):
    """Returns (dx or None if the unit starts with the embedding, grads) with
    grads = {'layers': {layer_id: {name: array}}, 'wte': ..., 'wpe': ...}."""
    d = np.asarray(dy, dtype=dtype)
    grads = {"layers": {}}
    for l, p, cache in reversed(tape["layers"]):
        d, g = layer_backward(d, p, cache, n_heads)
        grads["layers"][l] = g
    if tape["embed"] is not None:
        tok = tape["embed"]
        dwte = np.zeros(np.asarray(params["wte"]).shape, dtype=dtype)
        np.add.at(dwte, tok, d)
        dwpe = np.zeros(np.asarray(params["wpe"]).shape, dtype=dtype)
        dwpe[: tok.shape[0]] += d
        grads["wte"], grads["wpe"] = dwte, dwpe
        return None, grads
    return d, grads


def run_stage(params, n_layers, n_chunks, n_heads, x_in, dy, vocab=0, eps=1e-5, dtype=np.float64, dropout_p=0.0,
              seed=0):
    """Whole job of one rank: every (chunk, mb) unit forward and backward,
    parameter gradients summed over microbatches in microbatch order.

    x_in, dy: dicts keyed (mb, chunk).  Chunk c owns layers [c*Lu, (c+1)*Lu)
    and is an independent function with its own input and upstream gradient
    (in a real pipeline the other ranks sit between two chunks of one rank).

    Returns y {(mb, chunk): [s, h]}, dx {(mb, chunk): [s, h] or None}, grads
    {'layers': [dict per layer], 'wte', 'wpe'}.  dropout_p > 0 applies the two hidden
    dropouts of every layer with masks derived from (seed, layer, site, mb).
    """
    lu = n_layers // n_chunks
    y, dx = {}, {}
    total = {"layers": [None] * n_layers}
    for (mb, chunk) in sorted(x_in.keys()):
        ids = list(range(chunk * lu, (chunk + 1) * lu))
        embed = vocab > 0 and chunk == 0
        out, tape = unit_forward(params, ids, x_in[(mb, chunk)], n_heads, eps, dtype, embed,
                                 (dropout_p, seed, mb) if dropout_p > 0.0 else None)
        y[(mb, chunk)] = out
        d, g = unit_backward(params, tape, dy[(mb, chunk)], n_heads, dtype)
        dx[(mb, chunk)] = d
        for l, gl in g["layers"].items():
            if total["layers"][l] is None:
                total["layers"][l] = {k: a.copy() for k, a in gl.items()}
            else:
                for k, a in gl.items():
                    total["layers"][l][k] += a
        for name in ("wte", "wpe"):
            if name in g:
                total[name] = total.get(name, 0) + g[name]
    return y, dx, total
