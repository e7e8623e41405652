"""Pins for the oracle's Transformer-encoder step: finite differences on a tiny net, torch's autograd on a
small one (an independent library implementation of every operation), closed forms and invariants of
LayerNorm, GELU and softmax attention."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads as wl
from oracle import ops


def _f64(params):
    return {k: v.double().numpy().copy() for k, v in params.items()}


def test_finite_differences_full_backward():
    cfg = wl.get_config("tiny_encoder")
    p = _f64(wl.make_params(cfg, seed=4, perturbed=True))
    for name in p:                                  # spread the 0.02-scale weights so every path carries signal
        if name.endswith("weight") and p[name].ndim == 2:
            p[name] *= 12.0
    batch = wl.make_batch(cfg, seed=4)
    n_units = wl.unit_count(cfg)
    _, grads = oracle.spb_step(cfg, p, batch, n_units)
    assert set(grads) == set(p)
    for name, arr in p.items():
        fd = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            h = 1e-6 * max(1.0, abs(arr[idx]))
            keep = arr[idx]
            arr[idx] = keep + h
            up = oracle.spb_step(cfg, p, batch, 0)[0]
            arr[idx] = keep - h
            dn = oracle.spb_step(cfg, p, batch, 0)[0]
            arr[idx] = keep
            fd[idx] = (up - dn) / (2 * h)
        scale = max(np.abs(fd).max(), 1e-12)
        assert np.abs(fd - grads[name]).max() / scale < 2e-6, name


def _torch_encoder(cfg, tp, batch):
    ids = batch["x"].long().reshape(-1)
    b, s, nh, hid = cfg["batch"], cfg["seq"], cfg["heads"], cfg["hidden"]
    d = hid // nh
    x = F.embedding(ids, tp["embed.tok.weight"]) + tp["embed.pos.weight"].repeat(b, 1)
    for i in range(cfg["layers"]):
        pre = f"layer{i}."
        u = F.layer_norm(x, (hid,), tp[pre + "ln1.weight"], tp[pre + "ln1.bias"], 1e-5)
        qkv = F.linear(u, tp[pre + "attn.qkv.weight"], tp[pre + "attn.qkv.bias"]).view(b, s, 3, nh, d)
        q, k, v = (qkv[:, :, j].permute(0, 2, 1, 3) for j in range(3))
        prob = torch.softmax(q @ k.transpose(-1, -2) / math.sqrt(d), dim=-1)
        ctx = (prob @ v).permute(0, 2, 1, 3).reshape(b * s, hid)
        h = x + F.linear(ctx, tp[pre + "attn.out.weight"], tp[pre + "attn.out.bias"])
        v2 = F.layer_norm(h, (hid,), tp[pre + "ln2.weight"], tp[pre + "ln2.bias"], 1e-5)
        f = F.gelu(F.linear(v2, tp[pre + "ffn.w1.weight"], tp[pre + "ffn.w1.bias"]))
        x = h + F.linear(f, tp[pre + "ffn.w2.weight"], tp[pre + "ffn.w2.bias"])
    rows = batch["loss_rows"].long()
    y = F.layer_norm(x[rows], (hid,), tp["head.ln.weight"], tp["head.ln.bias"], 1e-5)
    logits = F.linear(y, tp["head.vocab.weight"], tp["head.vocab.bias"])
    return F.cross_entropy(logits, batch["labels"].long())


@pytest.mark.parametrize("name,k", [("small_encoder_bf16", 4), ("small_encoder_bf16", 2), ("tiny_encoder", 3)])
def test_torch_autograd_third_opinion(name, k):
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, 2, perturbed=True), wl.make_batch(cfg, 2)
    n_units = wl.unit_count(cfg)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    tp = {n: v.double().clone().requires_grad_(unit_of[n] >= n_units - k) for n, v in params.items()}
    loss_t = _torch_encoder(cfg, tp, batch)
    loss_t.backward()
    loss, g = oracle.spb_step(cfg, params, batch, k)
    assert abs(loss - loss_t.item()) < 1e-12
    assert set(g) == {n for n, t in tp.items() if t.requires_grad}
    for n in g:
        ref = tp[n].grad.numpy()
        assert np.abs(g[n] - ref).max() <= 1e-11 * max(1.0, np.abs(ref).max()), n


def test_layernorm_closed_forms_and_invariants():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 16)) * 3 + 1
    gamma, beta = rng.standard_normal(16), rng.standard_normal(16)
    y, cache = ops.layernorm_fwd(x, gamma, beta)
    xhat, _ = cache
    assert np.abs(xhat.mean(axis=1)).max() < 1e-14 and np.abs((xhat ** 2).mean(axis=1) - 1).max() < 1e-5
    ref = F.layer_norm(torch.from_numpy(x), (16,), torch.from_numpy(gamma), torch.from_numpy(beta), 1e-5).numpy()
    assert np.abs(y - ref).max() < 1e-13
    dy = rng.standard_normal((5, 16))
    dx, dg, db = ops.layernorm_bwd(dy, gamma, cache)
    assert np.abs(dx.sum(axis=1)).max() < 1e-13            # dx is orthogonal to the constant vector ...
    # ... and to xhat up to the epsilon in the variance: sum(dx * xhat) = rstd * sum(g * xhat) * (1 - mean(xhat^2))
    g = dy * gamma
    resid = cache[1][:, 0] * (g * xhat).sum(axis=1) * (1 - (xhat ** 2).mean(axis=1))
    assert np.abs((dx * xhat).sum(axis=1) - resid).max() < 1e-13 and np.abs(resid).max() < 1e-4
    assert np.allclose(db, dy.sum(axis=0)) and np.allclose(dg, (dy * xhat).sum(axis=0))
    # shifting or (for eps -> 0) scaling a row leaves the output unchanged
    y2, _ = ops.layernorm_fwd(x + 7.0, gamma, beta)
    assert np.abs(y - y2).max() < 1e-12


def test_gelu_values_and_derivative():
    assert ops.gelu_fwd(np.array([0.0]))[0] == 0.0 and ops.gelu_grad(np.array([0.0]))[0] == 0.5
    x = np.array([-6.0, -1.0, 1.0, 6.0])
    phi1 = 0.5 * (1 + math.erf(1 / math.sqrt(2)))            # Phi(1) = 0.8413447...
    assert abs(ops.gelu_fwd(x)[2] - phi1) < 1e-15 and abs(ops.gelu_fwd(x)[1] + (1 - phi1)) < 1e-15
    assert abs(ops.gelu_fwd(x)[3] - 6.0) < 1e-7 and abs(ops.gelu_fwd(x)[0]) < 1e-7
    xs = np.linspace(-5, 5, 101)
    assert np.abs(ops.gelu_fwd(xs) - F.gelu(torch.from_numpy(xs)).numpy()).max() < 1e-15
    h = 1e-6
    fd = (ops.gelu_fwd(xs + h) - ops.gelu_fwd(xs - h)) / (2 * h)
    assert np.abs(fd - ops.gelu_grad(xs)).max() < 1e-9
    # x + gelu(-x) = gelu(x): the function's odd part is x / 2
    assert np.abs(ops.gelu_fwd(xs) - ops.gelu_fwd(-xs) - xs).max() < 1e-14


def test_attention_gradient_rows_and_head_layout():
    rng = np.random.default_rng(9)
    s = rng.standard_normal((2, 3, 4, 4))
    p = ops.softmax_rows(s)
    assert np.abs(p.sum(axis=-1) - 1).max() < 1e-15
    dp = rng.standard_normal(p.shape)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    assert np.abs(ds.sum(axis=-1)).max() < 1e-15            # softmax is shift invariant along a row
    t = np.arange(2 * 4 * 6, dtype=np.float64).reshape(8, 6)   # batch 2, seq 4, heads 3, d 2
    h = ops.split_heads(t, 2, 4, 3)
    assert h.shape == (2, 3, 4, 2) and h[1, 2, 3, 1] == t[1 * 4 + 3, 2 * 2 + 1]
    assert np.array_equal(ops.merge_heads(h), t)


def test_embedding_gradient_adds_duplicates():
    cfg = wl.get_config("tiny_encoder")
    params, batch = wl.make_params(cfg, 0), wl.make_batch(cfg, 0)
    ids = batch["x"].reshape(-1).numpy()
    assert len(set(ids.tolist())) < len(ids)                  # this batch repeats a token
    _, g = oracle.spb_step(cfg, params, batch, wl.unit_count(cfg))
    unused = sorted(set(range(cfg["vocab"])) - set(ids.tolist()))
    assert np.all(g["embed.tok.weight"][unused] == 0)
    # every position's gradient lands in exactly one token row and one position row
    assert np.allclose(g["embed.tok.weight"].sum(axis=0), g["embed.pos.weight"].sum(axis=0))
