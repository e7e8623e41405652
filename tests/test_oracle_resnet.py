"""Pins for the oracle's residual-CNN step: the convolution definitions written as plain loops, adjoint
identities, reductions to a Linear layer, finite differences on tiny nets with both block kinds, stride 2,
projection shortcuts and the max-pool, and torch's autograd (conv2d, max_pool2d) on small nets."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads as wl
from oracle import ops


def _loops_conv(x, w, stride, pad):
    n, h, wd, ci = x.shape
    co, kr, ks, _ = w.shape
    ho, wo = (h + 2 * pad - kr) // stride + 1, (wd + 2 * pad - ks) // stride + 1
    y = np.zeros((n, ho, wo, co))
    for b, i, j, o, r, t, c in itertools.product(range(n), range(ho), range(wo), range(co), range(kr), range(ks), range(ci)):
        hi, wi = i * stride + r - pad, j * stride + t - pad
        if 0 <= hi < h and 0 <= wi < wd:
            y[b, i, j, o] += x[b, hi, wi, c] * w[o, r, t, c]
    return y


@pytest.mark.parametrize("kernel,stride,pad,size", [(1, 1, 0, 4), (1, 2, 0, 5), (3, 1, 1, 5), (3, 2, 1, 6), (3, 2, 1, 5), (7, 2, 3, 9)])
def test_convolution_against_loops_and_adjoints(kernel, stride, pad, size):
    rng = np.random.default_rng(kernel * 10 + stride)
    x = rng.standard_normal((2, size, size + 1, 3))            # non-square image, ci != co: a swapped index cannot pass
    w = rng.standard_normal((4, kernel, kernel, 3))
    y = ops.conv_fwd(x, w, stride, pad)
    assert np.abs(y - _loops_conv(x, w, stride, pad)).max() < 1e-12
    dy = rng.standard_normal(y.shape)
    dx = ops.conv_dgrad(dy, w, x.shape[1:3], stride, pad)
    dw = ops.conv_wgrad(x, dy, kernel, stride, pad)
    assert dx.shape == x.shape and dw.shape == w.shape
    lhs = np.vdot(y, dy)                                       # the convolution is linear in x and in w
    assert abs(lhs - np.vdot(x, dx)) < 1e-10 * max(1, abs(lhs))
    assert abs(lhs - np.vdot(w, dw)) < 1e-10 * max(1, abs(lhs))
    # one element of each gradient from the definition
    e = np.zeros_like(x); e[1, 2, 3, 1] = 1.0
    assert abs(np.vdot(_loops_conv(e, w, stride, pad), dy) - dx[1, 2, 3, 1]) < 1e-12
    e = np.zeros_like(w); e[2, kernel // 2, 0, 1] = 1.0
    assert abs(np.vdot(_loops_conv(x, e, stride, pad), dy) - dw[2, kernel // 2, 0, 1]) < 1e-12


def test_convolution_special_cases_reduce_to_a_linear_layer():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 4, 5, 6))
    w1 = rng.standard_normal((3, 1, 1, 6))
    lin = ops.linear_fwd(x.reshape(-1, 6), w1[:, 0, 0, :], np.zeros(3)).reshape(2, 4, 5, 3)
    assert np.abs(ops.conv_fwd(x, w1, 1, 0) - lin).max() < 1e-13
    w3 = np.zeros((3, 3, 3, 6)); w3[:, 1, 1, :] = w1[:, 0, 0, :]      # centre tap only
    assert np.abs(ops.conv_fwd(x, w3, 1, 1) - lin).max() < 1e-13
    assert np.abs(ops.conv_fwd(x, w1, 2, 0) - lin[:, ::2, ::2]).max() < 1e-13


def test_maxpool_and_avgpool():
    rng = np.random.default_rng(7)
    x = rng.permutation(2 * 7 * 6 * 3).reshape(2, 7, 6, 3).astype(np.float64)      # all distinct: no ties
    out, arg = ops.maxpool3x3s2_fwd(x)
    assert out.shape == (2, 4, 3, 3)
    for b, i, j, c in itertools.product(range(2), range(4), range(3), range(3)):
        win = [(x[b, hi, wi, c], hi * 6 + wi) for hi in range(2 * i - 1, 2 * i + 2) for wi in range(2 * j - 1, 2 * j + 2)
               if 0 <= hi < 7 and 0 <= wi < 6]
        assert (out[b, i, j, c], arg[b, i, j, c]) == max(win)
    dout = rng.standard_normal(out.shape)
    dx = ops.maxpool3x3s2_bwd(dout, arg, (7, 6))
    assert abs(dx.sum() - dout.sum()) < 1e-12                # every output gradient lands exactly once
    flat = x.reshape(2, 42, 3)
    for b, c in itertools.product(range(2), range(3)):       # finite differences of sum(dout * pool(x)) at the maxima
        for pos in np.unique(arg[b, :, :, c]):
            e = np.zeros_like(x); e.reshape(2, 42, 3)[b, pos, c] = 1e-3
            fd = (np.vdot(ops.maxpool3x3s2_fwd(x + e)[0], dout) - np.vdot(out, dout)) / 1e-3
            assert abs(fd - dx.reshape(2, 42, 3)[b, pos, c]) < 1e-9
    tie = np.zeros((1, 3, 3, 1))                              # all equal: the first position of the window wins
    _, arg_t = ops.maxpool3x3s2_fwd(tie)
    assert arg_t[0, 0, 0, 0] == 0 and arg_t[0, 1, 1, 0] == 4
    p = ops.avgpool_fwd(x)
    assert np.allclose(p, x.reshape(2, -1, 3).mean(axis=1))
    back = ops.avgpool_bwd(np.ones((2, 3)), (7, 6))
    assert back.shape == x.shape and np.allclose(back, 1.0 / 42)
    assert flat.shape == (2, 42, 3)


def test_affine_gradients():
    rng = np.random.default_rng(4)
    y, dz, s = rng.standard_normal((2, 3, 3, 5)), rng.standard_normal((2, 3, 3, 5)), rng.standard_normal(5)
    dy, ds, db = ops.affine_bwd(dz, y, s)
    assert np.allclose(dy, dz * s) and np.allclose(db, dz.reshape(-1, 5).sum(0)) and np.allclose(ds, (dz * y).reshape(-1, 5).sum(0))


@pytest.mark.parametrize("name", ["tiny_resnet_basic", "tiny_resnet_bottleneck"])
def test_finite_differences_full_backward(name):
    cfg = wl.get_config(name)
    p = {k: v.double().numpy().copy() for k, v in wl.make_params(cfg, seed=5, perturbed=True).items()}
    batch = wl.make_batch(cfg, seed=5)
    n_units = wl.unit_count(cfg)
    _, grads = oracle.spb_step(cfg, p, batch, n_units)
    assert set(grads) == set(p)
    for pname, arr in p.items():
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
        assert np.abs(fd - grads[pname]).max() / scale < 1e-6, pname


def _torch_resnet(cfg, tp, batch):
    lay = wl.resnet_layout(cfg)

    def conv_aff(x, name_c, name_a, stride, pad):
        w = tp[name_c + ".weight"].permute(0, 3, 1, 2)           # [Cout, R, S, Cin] -> torch's [Cout, Cin, R, S]
        y = F.conv2d(x, w, stride=stride, padding=pad)
        return y * tp[name_a + ".scale"].view(1, -1, 1, 1) + tp[name_a + ".shift"].view(1, -1, 1, 1)

    x = batch["x"].double().permute(0, 3, 1, 2)
    st = lay["stem"]
    x = torch.relu(conv_aff(x, "stem.conv", "stem.aff", st["stride"], st["pad"]))
    if st["pool"]:
        x = F.max_pool2d(x, 3, 2, 1)
    for blk in lay["blocks"]:
        pre = f"block{blk['index']}."
        spec = [(1, 0), (blk["stride"], 1), (1, 0)] if lay["bottleneck"] else [(blk["stride"], 1), (1, 1)]
        sc = conv_aff(x, pre + "proj", pre + "projaff", blk["stride"], 0) if blk["proj"] else x
        h = x
        for j, (s, pd) in enumerate(spec, start=1):
            h = conv_aff(h, f"{pre}conv{j}", f"{pre}aff{j}", s, pd)
            if j < len(spec):
                h = torch.relu(h)
        x = torch.relu(h + sc)
    pooled = x.mean(dim=(2, 3))
    logits = F.linear(pooled, tp["head.fc.weight"], tp["head.fc.bias"])
    return F.cross_entropy(logits, batch["labels"].long())


@pytest.mark.parametrize("name,k", [("small_resnet_basic_bf16", 5), ("small_resnet_basic_bf16", 2),
                                     ("small_resnet_bottleneck_bf16", 5), ("small_resnet_bottleneck_bf16", 3)])
def test_torch_autograd_third_opinion(name, k):
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, 3, perturbed=True), wl.make_batch(cfg, 3)
    n_units = wl.unit_count(cfg)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    tp = {n: v.double().clone().requires_grad_(unit_of[n] >= n_units - k) for n, v in params.items()}
    loss_t = _torch_resnet(cfg, tp, batch)
    loss_t.backward()
    loss, g = oracle.spb_step(cfg, params, batch, k)
    assert abs(loss - loss_t.item()) < 1e-10 * max(1.0, abs(loss))
    assert set(g) == {n for n, t in tp.items() if t.requires_grad}
    for n in g:
        ref = tp[n].grad.numpy()
        assert np.abs(g[n] - ref).max() <= 1e-10 * max(1.0, np.abs(ref).max()), n
