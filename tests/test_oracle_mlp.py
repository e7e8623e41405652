"""Pins for the oracle's perceptron step (Linear, ReLU, softmax cross-entropy,
truncated backward).  None of these retypes the oracle's formulas: they use
finite differences, closed forms, element-by-element loops, torch's autograd
and the suffix properties the paper states (Sec. 1-2)."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from oracle import ops


def _f64(params):
    return {k: v.double().numpy().copy() for k, v in params.items()}


def _loss_only(cfg, p, batch):
    return oracle.spb_step(cfg, p, batch, 0)[0]


def test_finite_differences_full_backward():
    cfg = wl.get_config("tiny_mlp_f32")
    p = _f64(wl.make_params(cfg, seed=3, perturbed=True))
    batch = wl.make_batch(cfg, seed=3)
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
            up = _loss_only(cfg, p, batch)
            arr[idx] = keep - h
            dn = _loss_only(cfg, p, batch)
            arr[idx] = keep
            fd[idx] = (up - dn) / (2 * h)
        scale = max(np.abs(fd).max(), 1e-12)
        assert np.abs(fd - grads[name]).max() / scale < 1e-6, name


@pytest.mark.parametrize("name", ["tiny_mlp_f32", "ragged_mlp_f32", "ragged_mlp_bf16", "tiny_encoder", "small_encoder_bf16",
                                  "tiny_resnet_bottleneck", "small_resnet_basic_bf16"])
@pytest.mark.parametrize("mode", ["exact", "bf16"])
def test_suffix_properties(name, mode):
    """Depth k returns exactly the top-k units' parameters; their values do not
    depend on where the walk stopped; the loss does not depend on k."""
    cfg = wl.get_config(name)
    q = oracle.identity if mode == "exact" else oracle.round_to_bf16
    p, batch = wl.make_params(cfg, 1, perturbed=True), wl.make_batch(cfg, 1)
    n_units = wl.unit_count(cfg)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    loss_full, full = oracle.spb_step(cfg, p, batch, n_units, q)
    assert set(full) == set(unit_of)
    for k in range(0, n_units + 1):
        loss, g = oracle.spb_step(cfg, p, batch, k, q)
        assert loss == loss_full
        assert set(g) == {n for n, u in unit_of.items() if u >= n_units - k}
        for n in g:
            assert np.array_equal(g[n], full[n]), (k, n)
    assert oracle.spb_step(cfg, p, batch, 0, q)[1] == {}
    with pytest.raises(ValueError):
        oracle.spb_step(cfg, p, batch, n_units + 1, q)
    with pytest.raises(ValueError):
        oracle.spb_step(cfg, p, batch, -1, q)


def test_cross_entropy_closed_forms():
    # With an all-zero last layer every class has probability 1/C: the loss is
    # ln C and the last bias gradient is 1/C minus the label frequency.
    for name in ["cfg1", "ragged_mlp_f32"]:
        cfg = wl.get_config(name)
        p, batch = _f64(wl.make_params(cfg, 0)), wl.make_batch(cfg, 0)
        last = wl.unit_count(cfg) - 1
        p[f"fc{last}.weight"][:] = 0.0
        p[f"fc{last}.bias"][:] = 0.0
        classes = cfg["dims"][-1]
        loss, g = oracle.spb_step(cfg, p, batch, 1)
        assert abs(loss - math.log(classes)) < 1e-12
        freq = np.bincount(batch["labels"].numpy(), minlength=classes) / cfg["batch"]
        assert np.allclose(g[f"fc{last}.bias"], 1.0 / classes - freq, atol=1e-14)
    rng = np.random.default_rng(5)
    z = rng.standard_normal((7, 11)) * 4
    y = rng.integers(0, 11, 7)
    loss, dz = ops.softmax_ce(z, y)
    assert np.abs(dz.sum(axis=1)).max() < 1e-15            # rows of the gradient sum to zero
    # shifting a row's logits by a constant changes nothing
    loss2, dz2 = ops.softmax_ce(z + rng.standard_normal((7, 1)) * 50, y)
    assert abs(loss - loss2) < 1e-12 and np.abs(dz - dz2).max() < 1e-13
    # two classes reduce to the logistic loss
    z2 = rng.standard_normal((6, 2))
    y2 = rng.integers(0, 2, 6)
    margin = np.where(y2 == 1, z2[:, 1] - z2[:, 0], z2[:, 0] - z2[:, 1])
    assert abs(ops.softmax_ce(z2, y2)[0] - np.mean(np.log1p(np.exp(-margin)))) < 1e-12
    # huge logits do not overflow
    big, _ = ops.softmax_ce(np.array([[1000.0, 0.0]]), np.array([1]))
    assert abs(big - 1000.0) < 1e-9


def test_linear_against_elementwise_loops():
    rng = np.random.default_rng(11)
    m, n, k = 3, 4, 5                     # all different: a transposed operand cannot pass
    x, w, b = rng.standard_normal((m, k)), rng.standard_normal((n, k)), rng.standard_normal(n)
    dz = rng.standard_normal((m, n))
    z = ops.linear_fwd(x, w, b)
    dw, db, dx = ops.linear_bwd(dz, x, w, True)
    for i in range(m):
        for j in range(n):
            assert abs(z[i, j] - (sum(x[i, t] * w[j, t] for t in range(k)) + b[j])) < 1e-12
    for j in range(n):
        assert abs(db[j] - sum(dz[i, j] for i in range(m))) < 1e-12
        for t in range(k):
            assert abs(dw[j, t] - sum(dz[i, j] * x[i, t] for i in range(m))) < 1e-12
    for i in range(m):
        for t in range(k):
            assert abs(dx[i, t] - sum(dz[i, j] * w[j, t] for j in range(n))) < 1e-12
    assert ops.linear_bwd(dz, x, w, False)[2] is None
    # adjoint identities: <linear(x), dz> = <x, dx> + <b, db> = <w, dw> + <b, db>
    zero_b = np.zeros(n)
    assert abs(np.vdot(ops.linear_fwd(x, w, zero_b), dz) - np.vdot(x, dx)) < 1e-12
    assert abs(np.vdot(ops.linear_fwd(x, w, zero_b), dz) - np.vdot(w, dw)) < 1e-12


def test_relu_derivative_at_zero_is_zero():
    z = np.array([-1.0, 0.0, -0.0, 2.0])
    assert np.array_equal(ops.relu_bwd(np.ones(4), z), [0.0, 0.0, 0.0, 1.0])
    assert np.array_equal(ops.relu_fwd(z), [0.0, 0.0, 0.0, 2.0])


@pytest.mark.parametrize("name,k", [("cfg1", 2), ("cfg1", 4), ("ragged_mlp_f32", 3)])
def test_torch_autograd_third_opinion(name, k):
    """torch's CPU autograd in float64 with the parameters below the cut frozen."""
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, 2, perturbed=True), wl.make_batch(cfg, 2)
    n_units = wl.unit_count(cfg)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    tp = {n: v.double().clone().requires_grad_(unit_of[n] >= n_units - k) for n, v in params.items()}
    h = batch["x"].double()
    for i in range(n_units):
        h = torch.nn.functional.linear(h, tp[f"fc{i}.weight"], tp[f"fc{i}.bias"])
        if i < n_units - 1:
            h = torch.relu(h)
    loss_t = torch.nn.functional.cross_entropy(h, batch["labels"].long())
    loss_t.backward()
    loss, g = oracle.spb_step(cfg, params, batch, k)
    assert abs(loss - loss_t.item()) < 1e-12
    for n, t in tp.items():
        if t.requires_grad:
            ref = t.grad.numpy()
            assert np.abs(g[n] - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max()), n
        else:
            assert n not in g


def test_bf16_mode_differs_from_exact_mode_by_storage_noise_only():
    """Rounding stored activations to bfloat16 perturbs the step but does not
    change what it computes: the loss moves by well under a percent, and every
    gradient stays within the spread that re-rounding a deep ReLU chain causes
    (a few percent of the tensor's largest entry per ReLU layer crossed, because
    a pre-activation that changes sign switches a whole term on or off)."""
    cfg = wl.get_config("ragged_mlp_bf16")
    p, batch = wl.make_params(cfg, 0), wl.make_batch(cfg, 0)
    n_units = wl.unit_count(cfg)
    la, ga = oracle.spb_step(cfg, p, batch, n_units)
    lb, gb = oracle.spb_step(cfg, p, batch, n_units, oracle.round_to_bf16)
    assert la != lb and abs(la - lb) / abs(la) < 5e-3
    top = f"fc{n_units - 1}.weight"           # no ReLU between it and the loss
    assert np.abs(ga[top] - gb[top]).max() / np.abs(ga[top]).max() < 1e-2
    for n in ga:
        assert np.abs(ga[n] - gb[n]).max() / np.abs(ga[n]).max() < 0.25
        assert np.linalg.norm(ga[n] - gb[n]) / np.linalg.norm(ga[n]) < 0.25
