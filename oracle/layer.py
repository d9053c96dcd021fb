"""CPU oracle for the three passes of one pipeline chunk: F, B and W.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP path is checked
against; nothing in the product path may import it.  It shares no code with the HIP kernels.

The paper (Section 2.1) splits the work of a stage for one microbatch into
  F  - the forward pass,
  B  - "backward for the activations": gradients w.r.t. the stage input,
  W  - "backward for the weights": gradients w.r.t. the parameters, which may be deferred,
and notes that ordinary 1F1B is the special case where B and W always run back to back.  The model
is GPT-like (Section 4.1); the paper does not print the layer, so the layer below is the standard
pre-LayerNorm GPT block under these readings: tanh-form GeLU, LayerNorm with biased variance and
eps inside the square root, biases on all four linear maps, causal mask, no dropout.  LayerNorm
gain/bias gradients are produced by B (they fall out of the same row pass as the LayerNorm input
gradient); the four weight matrices' and their biases' gradients are produced by W.

Everything is written with numpy in float64 by default (dtype selectable), one formula per line,
with the full s x s attention matrix materialised per head.  Matmul is the only library primitive.

Parity pins (tests/test_oracle_layer.py): central finite differences in fp64; PyTorch-CPU fp64
autograd through torch's own layer_norm / gelu / softmax routines; causality; softmax row sums;
LayerNorm output moments; db = column sums.
"""
from __future__ import annotations

import math

import numpy as np

PARAM_NAMES = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2",
)


# --------------------------------------------------------------------------- elementary maps

def layer_norm(x, gamma, beta, eps):
    """y = gamma * (x - mean) * rstd + beta over the last axis; returns (y, xhat, rstd)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, xhat, rstd


def layer_norm_input_grad(dy, xhat, rstd, gamma):
    """Gradient of layer_norm w.r.t. x, plus (dgamma, dbeta)."""
    g = dy * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    return dx, (dy * xhat).sum(axis=0), dy.sum(axis=0)


_K0 = math.sqrt(2.0 / math.pi)
_K1 = 0.044715


def gelu(u):
    return 0.5 * u * (1.0 + np.tanh(_K0 * (u + _K1 * u ** 3)))


def gelu_grad(u):
    t = np.tanh(_K0 * (u + _K1 * u ** 3))
    return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * _K0 * (1.0 + 3.0 * _K1 * u * u)


def _softmax_rows(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def attention(qkv, heads, causal, batch=1):
    """Multi-head self-attention on packed [tokens, 3h] (columns q | k | v, heads contiguous).

    Returns (o [tokens, h], P list indexed [batch][head] of the s x s probability matrices,
    lse [batch, heads, s] = log-sum-exp of the scaled, masked scores).
    """
    tokens, h3 = qkv.shape
    h = h3 // 3
    dh = h // heads
    s = tokens // batch
    sigma = 1.0 / math.sqrt(dh)
    o = np.zeros((tokens, h), dtype=qkv.dtype)
    probs = []
    lse = np.zeros((batch, heads, s), dtype=qkv.dtype)
    for b in range(batch):
        rows = slice(b * s, (b + 1) * s)
        per_head = []
        for hd in range(heads):
            q = qkv[rows, hd * dh:(hd + 1) * dh]
            k = qkv[rows, h + hd * dh:h + (hd + 1) * dh]
            v = qkv[rows, 2 * h + hd * dh:2 * h + (hd + 1) * dh]
            sc = sigma * (q @ k.T)
            if causal:
                sc = np.where(np.tril(np.ones((s, s), dtype=bool)), sc, -np.inf)
            mx = sc.max(axis=-1, keepdims=True)
            lse[b, hd] = (mx + np.log(np.exp(sc - mx).sum(axis=-1, keepdims=True)))[:, 0]
            p = _softmax_rows(sc)
            o[rows, hd * dh:(hd + 1) * dh] = p @ v
            per_head.append(p)
        probs.append(per_head)
    return o, probs, lse


def attention_input_grad(do, qkv, probs, heads, batch=1):
    """Gradient of attention() w.r.t. the packed qkv."""
    tokens, h3 = qkv.shape
    h = h3 // 3
    dh = h // heads
    s = tokens // batch
    sigma = 1.0 / math.sqrt(dh)
    dqkv = np.zeros_like(qkv)
    for b in range(batch):
        rows = slice(b * s, (b + 1) * s)
        for hd in range(heads):
            cq = slice(hd * dh, (hd + 1) * dh)
            ck = slice(h + hd * dh, h + (hd + 1) * dh)
            cv = slice(2 * h + hd * dh, 2 * h + (hd + 1) * dh)
            q, k, v = qkv[rows, cq], qkv[rows, ck], qkv[rows, cv]
            p = probs[b][hd]
            d_o = do[rows, cq]
            dp = d_o @ v.T
            ds = p * (dp - (p * dp).sum(axis=-1, keepdims=True))
            dqkv[rows, cv] = p.T @ d_o
            dqkv[rows, cq] = sigma * (ds @ k)
            dqkv[rows, ck] = sigma * (ds.T @ q)
    return dqkv


# --------------------------------------------------------------------------- one layer

def layer_forward(x, p, heads, causal=True, eps=1e-5, batch=1):
    """F for one layer.  Returns (x_out, saved) where saved holds what B and W read later."""
    a, xhat1, rstd1 = layer_norm(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = a @ p["w_qkv"] + p["b_qkv"]
    o, probs, lse = attention(qkv, heads, causal, batch)
    x_mid = x + o @ p["w_o"] + p["b_o"]
    c, xhat2, rstd2 = layer_norm(x_mid, p["ln2_g"], p["ln2_b"], eps)
    u = c @ p["w_1"] + p["b_1"]
    g = gelu(u)
    x_out = x_mid + g @ p["w_2"] + p["b_2"]
    saved = dict(x=x, xhat1=xhat1, rstd1=rstd1, a=a, qkv=qkv, probs=probs, lse=lse, o=o,
                 x_mid=x_mid, xhat2=xhat2, rstd2=rstd2, c=c, u=u, g=g)
    return x_out, saved


def layer_backward_input(dx_out, p, saved, heads, batch=1):
    """B for one layer.  Returns (dx, stash, ln_grads).

    stash holds the output-side gradients of the four linear maps (what W contracts with the saved
    inputs); ln_grads holds the LayerNorm gain/bias gradients, which B owns.
    """
    dg = dx_out @ p["w_2"].T
    du = dg * gelu_grad(saved["u"])
    dc = du @ p["w_1"].T
    dln2, dg2, db2 = layer_norm_input_grad(dc, saved["xhat2"], saved["rstd2"], p["ln2_g"])
    dx_mid = dx_out + dln2
    do = dx_mid @ p["w_o"].T
    dqkv = attention_input_grad(do, saved["qkv"], saved["probs"], heads, batch)
    da = dqkv @ p["w_qkv"].T
    dln1, dg1, db1 = layer_norm_input_grad(da, saved["xhat1"], saved["rstd1"], p["ln1_g"])
    dx = dx_mid + dln1
    stash = dict(dx_out=dx_out, du=du, dx_mid=dx_mid, dqkv=dqkv)
    ln_grads = dict(ln1_g=dg1, ln1_b=db1, ln2_g=dg2, ln2_b=db2)
    return dx, stash, ln_grads


def layer_backward_weight(saved, stash):
    """W for one layer: dW = X^T dY and db = column sums of dY for the four linear maps."""
    return dict(
        w_2=saved["g"].T @ stash["dx_out"], b_2=stash["dx_out"].sum(axis=0),
        w_1=saved["c"].T @ stash["du"], b_1=stash["du"].sum(axis=0),
        w_o=saved["o"].T @ stash["dx_mid"], b_o=stash["dx_mid"].sum(axis=0),
        w_qkv=saved["a"].T @ stash["dqkv"], b_qkv=stash["dqkv"].sum(axis=0),
    )


# --------------------------------------------------------------------------- one chunk (L layers)

def cast_params(params, dtype=np.float64):
    return [{k: np.asarray(v, dtype=dtype) for k, v in layer.items()} for layer in params]


def chunk_forward(x, params, heads, causal=True, eps=1e-5, batch=1):
    """F for a chunk: the layers in order.  Returns (y, saved_per_layer)."""
    saved = []
    for p in params:
        x, sv = layer_forward(x, p, heads, causal, eps, batch)
        saved.append(sv)
    return x, saved


def chunk_backward_input(dy, params, saved, heads, batch=1):
    """B for a chunk: the layers in reverse.  Returns (dx, stash_per_layer, ln_grads_per_layer)."""
    n = len(params)
    stash = [None] * n
    ln_grads = [None] * n
    for l in reversed(range(n)):
        dy, stash[l], ln_grads[l] = layer_backward_input(dy, params[l], saved[l], heads, batch)
    return dy, stash, ln_grads


def chunk_backward_weight(saved, stash):
    """W for a chunk.  Returns per-layer dict of weight and bias gradients."""
    return [layer_backward_weight(sv, st) for sv, st in zip(saved, stash)]


def zero_grads(params):
    return [{k: np.zeros_like(v) for k, v in layer.items()} for layer in params]


def accumulate(grads, *parts):
    """grads[l][name] += part[l][name] for every part (in the order given)."""
    for part in parts:
        for gl, pl in zip(grads, part):
            for k, v in pl.items():
                gl[k] += v


def chunk_activation_bytes(layers, hidden, heads, seq, elem_bytes, microbatch=1, ffn=None):
    """Bytes of activation one (chunk, microbatch) unit holds from F until W, by tensor:
    x, LN1 out, qkv (3), attention out, x_mid, LN2 out (8 [tokens, hidden] tensors) and u, g
    (2 [tokens, ffn] tensors; with ffn = 4 hidden that is 16 [tokens, hidden] in all) in the storage
    type, plus fp32 LayerNorm statistics (2 + 2 per token) and the attention log-sum-exp (heads per
    token).  After B the tensors x, qkv, x_mid, u are replaced one for one by the gradient tensors
    W needs (dx_out, d qkv, dx_mid, du), so the count stays the same."""
    tokens = seq * microbatch
    ffn = 4 * hidden if ffn is None else ffn
    return layers * ((8 * hidden + 2 * ffn) * tokens * elem_bytes + (4 + heads) * tokens * 4)


def chunk_stats_bytes(layers, heads, seq, microbatch=1):
    """The fp32 statistics part of chunk_activation_bytes; dead once B has run."""
    return layers * (4 + heads) * seq * microbatch * 4
