"""Pins for oracle/layer.py: finite differences, PyTorch-CPU fp64 autograd through torch's own
layer_norm / gelu / scaled_dot_product_attention routines, and structural invariants."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import synth
from oracle import layer as O

TINY = synth.ChunkCfg(layers=2, hidden=16, heads=2, ffn=64, seq=8, dtype="f32")
SMALL = synth.ChunkCfg(layers=2, hidden=64, heads=4, ffn=256, seq=48, dtype="f32")


def _setup(cfg, tag, scale_w=10.0):
    # weights scaled up so that every term of the gradient is far above fp64 difference noise
    params = O.cast_params(synth.chunk_params(cfg, tag))
    for layer in params:
        for k in ("w_qkv", "w_o", "w_1", "w_2", "b_qkv", "b_o", "b_1", "b_2"):
            layer[k] = layer[k] * scale_w
    x = synth.chunk_input(cfg, tag).astype(np.float64)
    dy = synth.upstream_grad(cfg, tag).astype(np.float64)
    return params, x, dy


def _fbw(cfg, params, x, dy):
    y, saved = O.chunk_forward(x, params, cfg.heads, cfg.causal, cfg.ln_eps, cfg.microbatch)
    dx, stash, ln_grads = O.chunk_backward_input(dy, params, saved, cfg.heads, cfg.microbatch)
    wg = O.chunk_backward_weight(saved, stash)
    grads = O.zero_grads(params)
    O.accumulate(grads, ln_grads, wg)
    return y, dx, grads


def test_finite_differences_input_and_weights():
    cfg = TINY
    params, x, dy = _setup(cfg, "fd")
    y, dx, grads = _fbw(cfg, params, x, dy)

    def loss(px, pp):
        out, _ = O.chunk_forward(px, pp, cfg.heads, cfg.causal, cfg.ln_eps)
        return float((out * dy).sum())

    eps = 1e-5
    rng = np.random.default_rng(0)
    # input gradient: every entry
    num = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        num[idx] = (loss(xp, params) - loss(xm, params)) / (2 * eps)
    assert np.linalg.norm(num - dx) / np.linalg.norm(dx) < 1e-7
    # every parameter tensor of every layer: a few random entries each
    for l in range(cfg.layers):
        for name in O.PARAM_NAMES:
            w = params[l][name]
            for _ in range(4):
                idx = tuple(rng.integers(0, s) for s in w.shape)
                keep = w[idx]
                w[idx] = keep + eps
                lp = loss(x, params)
                w[idx] = keep - eps
                lm = loss(x, params)
                w[idx] = keep
                fd = (lp - lm) / (2 * eps)
                assert abs(fd - grads[l][name][idx]) <= 1e-6 * max(1.0, abs(fd)), (l, name, idx)


def _torch_chunk(x, params, cfg):
    h, nh, dh = cfg.hidden, cfg.heads, cfg.head_dim
    b, s = cfg.microbatch, cfg.seq
    for p in params:
        a = TF.layer_norm(x, (h,), p["ln1_g"], p["ln1_b"], cfg.ln_eps)
        qkv = TF.linear(a, p["w_qkv"].T, p["b_qkv"])
        q, k, v = [t.reshape(b, s, nh, dh).transpose(1, 2) for t in qkv.split(h, dim=-1)]
        o = TF.scaled_dot_product_attention(q, k, v, is_causal=cfg.causal)
        o = o.transpose(1, 2).reshape(b * s, h)
        x = x + TF.linear(o, p["w_o"].T, p["b_o"])
        c = TF.layer_norm(x, (h,), p["ln2_g"], p["ln2_b"], cfg.ln_eps)
        u = TF.linear(c, p["w_1"].T, p["b_1"])
        x = x + TF.linear(TF.gelu(u, approximate="tanh"), p["w_2"].T, p["b_2"])
    return x


@pytest.mark.parametrize("cfg", [TINY, SMALL,
                                 synth.ChunkCfg(layers=1, hidden=32, heads=2, ffn=128, seq=12, microbatch=3, dtype="f32"),
                                 synth.ChunkCfg(layers=1, hidden=32, heads=4, ffn=96, seq=20, dtype="f32", causal=False)])
def test_f_b_w_reproduce_autograd(cfg):
    """F then B then W gives the forward output and every gradient that a monolithic
    reverse-mode backward through library routines gives (Section 2.1: B and W together are the
    ordinary backward pass)."""
    params, x, dy = _setup(cfg, "ag", scale_w=5.0)
    y, dx, grads = _fbw(cfg, params, x, dy)
    tp = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()} for p in params]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = _torch_chunk(tx, tp, cfg)
    ty.backward(torch.tensor(dy))
    assert np.allclose(y, ty.detach().numpy(), rtol=1e-10, atol=1e-10)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-10)
    for l in range(cfg.layers):
        for name in O.PARAM_NAMES:
            want = tp[l][name].grad.numpy()
            got = grads[l][name]
            assert np.linalg.norm(got - want) <= 1e-10 * max(1.0, np.linalg.norm(want)), (l, name)


def test_b_alone_matches_input_grad_and_w_is_separable():
    """B needs no weight gradient and W no further input: running W long after B, or for several
    microbatches in any order, accumulates the same sums."""
    cfg = TINY
    params, _, _ = _setup(cfg, "sep")
    saved, stash = {}, {}
    total = O.zero_grads(params)
    for j in range(3):
        x = synth.chunk_input(cfg, "sep", j).astype(np.float64)
        dy = synth.upstream_grad(cfg, "sep", j).astype(np.float64)
        _, saved[j] = O.chunk_forward(x, params, cfg.heads)
        _, stash[j], ln = O.chunk_backward_input(dy, params, saved[j], cfg.heads)
        _, _, g = _fbw(cfg, params, x, dy)
        O.accumulate(total, g)
    deferred = O.zero_grads(params)
    for j in (2, 0, 1):
        O.accumulate(deferred, O.chunk_backward_weight(saved[j], stash[j]))
    for l in range(cfg.layers):
        for name in ("w_qkv", "w_o", "w_1", "w_2", "b_qkv", "b_o", "b_1", "b_2"):
            assert np.allclose(deferred[l][name], total[l][name], rtol=1e-12, atol=1e-12)


def test_bias_grads_are_column_sums():
    cfg = TINY
    params, x, dy = _setup(cfg, "bias")
    _, saved = O.chunk_forward(x, params, cfg.heads)
    _, stash, _ = O.chunk_backward_input(dy, params, saved, cfg.heads)
    wg = O.chunk_backward_weight(saved, stash)
    top = cfg.layers - 1
    assert np.allclose(wg[top]["b_2"], dy.sum(axis=0))
    ones = np.ones((1, cfg.tokens))
    for name, key in (("b_1", "du"), ("b_o", "dx_mid"), ("b_qkv", "dqkv")):
        assert np.allclose(wg[top][name], (ones @ stash[top][key])[0])


def test_layer_norm_moments_and_softmax_rows():
    x = synth.matrix(("ln",), (37, 96)).astype(np.float64) * 3 + 1.5
    y, xhat, rstd = O.layer_norm(x, np.ones(96), np.zeros(96), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-12) and np.allclose(y.var(-1), 1, atol=1e-12)
    want = TF.layer_norm(torch.tensor(x), (96,), eps=1e-5).numpy()
    assert np.allclose(O.layer_norm(x, np.ones(96), np.zeros(96), 1e-5)[0], want, atol=1e-12)
    qkv = synth.matrix(("sm",), (24, 3 * 32)).astype(np.float64)
    o, probs, lse = O.attention(qkv, heads=2, causal=True)
    for p in probs[0]:
        assert np.allclose(p.sum(-1), 1.0)
        assert np.all(np.triu(p, 1) == 0)
    # log-sum-exp against its definition on one row
    q, k = qkv[:, :16], qkv[:, 32:48]
    row = (q[5] @ k[:6].T) / 4.0
    assert math.isclose(lse[0, 0, 5], math.log(np.exp(row).sum()), rel_tol=1e-12)


def test_gelu_closed_values_and_derivative():
    u = np.linspace(-6, 6, 241)
    want = TF.gelu(torch.tensor(u), approximate="tanh").numpy()
    assert np.allclose(O.gelu(u), want, atol=1e-14)
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert np.allclose(O.gelu(np.array([10.0, -10.0])), [10.0, 0.0], atol=1e-12)
    e = 1e-6
    assert np.allclose(O.gelu_grad(u), (O.gelu(u + e) - O.gelu(u - e)) / (2 * e), atol=1e-8)


def test_causality():
    """With the causal mask the output at position t does not depend on later inputs, and the
    input gradient at position t does not depend on earlier upstream gradients."""
    cfg = TINY
    params, x, dy = _setup(cfg, "causal")
    y, _ = O.chunk_forward(x, params, cfg.heads)
    x2 = x.copy()
    x2[5:] += 1.0
    y2, _ = O.chunk_forward(x2, params, cfg.heads)
    assert np.array_equal(y[:5], y2[:5]) and not np.allclose(y[5:], y2[5:])
    _, sv = O.chunk_forward(x, params, cfg.heads)
    dx, _, _ = O.chunk_backward_input(dy, params, sv, cfg.heads)
    dy2 = dy.copy()
    dy2[:3] += 1.0
    dx2, _, _ = O.chunk_backward_input(dy2, params, sv, cfg.heads)
    assert np.allclose(dx[3:], dx2[3:], rtol=0, atol=1e-12) and not np.allclose(dx[:3], dx2[:3])


def test_microbatch_rows_are_independent_sequences():
    cfg = synth.ChunkCfg(layers=1, hidden=16, heads=2, ffn=64, seq=6, microbatch=2, dtype="f32")
    params, x, _ = _setup(cfg, "mb")
    y, _ = O.chunk_forward(x, params, cfg.heads, batch=2)
    one = synth.ChunkCfg(layers=1, hidden=16, heads=2, ffn=64, seq=6, dtype="f32")
    y0, _ = O.chunk_forward(x[:6], params, one.heads)
    y1, _ = O.chunk_forward(x[6:], params, one.heads)
    assert np.allclose(y, np.concatenate([y0, y1]), atol=1e-13)


def test_activation_bytes_table():
    """16 storage-typed [s,h] tensors + fp32 statistics per layer.  A pin to THIS repository's tensor
    table (which tensors a unit holds between F and W), worked out by hand for the four workload
    shapes, e.g. 16 * 128 * 256 * 4 + (4 + 4) * 128 * 4 = 2 101 248; the paper fixes only the number
    of units (Section 2.2, Section 3.2), not the bytes of one."""
    assert O.chunk_activation_bytes(1, 256, 4, 128, 4) == 2101248
    assert O.chunk_activation_bytes(1, 2048, 16, 1024, 2) == 67190784
    assert O.chunk_activation_bytes(1, 4096, 32, 2048, 2) == 268730368
    assert O.chunk_activation_bytes(1, 5120, 40, 4096, 2) == 671809536
    _, saved = O.chunk_forward(np.zeros((8, 16)), O.cast_params(synth.chunk_params(TINY, "b")), 2)
    sv = saved[0]
    elems = sum(sv[k].size for k in ("x", "a", "qkv", "o", "x_mid", "c", "u", "g"))
    assert elems == 16 * 8 * 16
