"""Pins of the server-side aggregation oracle (Sec. 2: per-layer average over the contributing workers, learning
rate scaled with their number; Sec. 4.1: SGD with momentum and weight decay)."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl


def _setup(name, n_workers, seed=0):
    cfg = wl.get_config(name)
    specs = wl.tensor_specs(cfg)
    units = {n: u for n, _s, u, _i in specs}
    L = wl.unit_count(cfg)
    params = {n: t.double().numpy() for n, t in wl.make_params(cfg, seed, perturbed=True).items()}
    vel = {n: t.double().numpy() for n, t in wl.make_velocity(cfg, seed).items()}
    grads = [{n: t.double().numpy() for n, t in g.items()} for g in wl.make_worker_grads(cfg, seed, n_workers)]
    return cfg, units, L, params, vel, grads


def test_depth_rule_rounds_up_and_last_worker_is_full():
    assert oracle.worker_depths(8, 4) == [2, 4, 6, 8]
    assert oracle.worker_depths(10, 4) == [3, 5, 8, 10]
    assert oracle.worker_depths(3, 4) == [1, 2, 3, 3]
    for L in range(1, 20):
        for K in range(1, 9):
            d = oracle.worker_depths(L, K)
            assert d[-1] == L and d == sorted(d) and all(1 <= k <= L for k in d)
            assert all(k == -((-j * L) // K) for j, k in enumerate(d, start=1))


def test_full_depth_everywhere_is_plain_mean_sgd_with_torch_as_second_opinion():
    # all workers complete -> ordinary data-parallel SGD: mean gradient, unscaled rate (c = K)
    cfg, units, L, params, vel, grads = _setup("ragged_mlp_f32", 3)
    lr, mu, wd = 0.1, 0.9, 1e-4
    new_w, new_v = oracle.aggregate_update(units, L, params, vel, grads, [L, L, L], lr, mu, wd, True)
    for n in params:
        w = torch.tensor(params[n], dtype=torch.float64, requires_grad=True)
        opt = torch.optim.SGD([w], lr=lr, momentum=mu, weight_decay=wd)
        opt.state[w]["momentum_buffer"] = torch.tensor(vel[n], dtype=torch.float64).clone()
        w.grad = torch.tensor(sum(g[n] for g in grads) / 3.0)
        opt.step()
        np.testing.assert_allclose(new_w[n], w.detach().numpy(), rtol=0, atol=1e-14)
        np.testing.assert_allclose(new_v[n], opt.state[w]["momentum_buffer"].numpy(), rtol=0, atol=1e-14)


def test_hand_computed_two_workers():
    # L = 2 units, one scalar parameter each; worker 1 has depth 1 (top unit only), worker 2 depth 2
    units = {"low": 0, "top": 1}
    params = {"low": np.array([1.0]), "top": np.array([2.0])}
    vel = {"low": np.array([0.5]), "top": np.array([-0.25])}
    grads = [{"low": np.array([100.0]), "top": np.array([0.4])}, {"low": np.array([0.2]), "top": np.array([0.8])}]
    w, v = oracle.aggregate_update(units, 2, params, vel, grads, [1, 2], lr=0.1, momentum=0.9, weight_decay=0.01, scale_lr=True)
    # top: c = 2, g = 0.6, v = 0.9 * -0.25 + 0.6 + 0.01 * 2 = 0.395, rate 0.1 -> w = 2 - 0.0395
    assert v["top"][0] == pytest.approx(0.395) and w["top"][0] == pytest.approx(2 - 0.0395)
    # low: only worker 2 (worker 1's value must be ignored), c = 1, g = 0.2, v = 0.45 + 0.2 + 0.01 = 0.66, rate 0.05
    assert v["low"][0] == pytest.approx(0.66) and w["low"][0] == pytest.approx(1 - 0.05 * 0.66)
    w2, _ = oracle.aggregate_update(units, 2, params, vel, grads, [1, 2], lr=0.1, momentum=0.9, weight_decay=0.01, scale_lr=False)
    assert w2["low"][0] == pytest.approx(1 - 0.1 * 0.66)


def test_parameters_nobody_reached_are_untouched_and_contributor_counts_follow_the_suffixes():
    cfg, units, L, params, vel, grads = _setup("ragged_mlp_f32", 3)
    depths = [1, 2, 2]                      # units 0 and 1 of 4 are below every cut
    new_w, new_v = oracle.aggregate_update(units, L, params, vel, grads, depths, 0.1, 0.9, 1e-4, True)
    for n, u in units.items():
        who = oracle.contributors(u, L, depths)
        assert who == [j for j, k in enumerate(depths) if u >= L - k]
        if u < 2:
            assert who == [] and np.array_equal(new_w[n], params[n]) and np.array_equal(new_v[n], vel[n])
        else:
            assert len(who) == (3 if u == 3 else 2) and not np.array_equal(new_w[n], params[n])


def test_a_non_contributing_workers_gradient_does_not_leak_in():
    cfg, units, L, params, vel, grads = _setup("tiny_mlp_f32", 2)
    depths = [1, L]
    a, _ = oracle.aggregate_update(units, L, params, vel, grads, depths, 0.1, 0.9, 0.0, True)
    poisoned = [dict(grads[0]), grads[1]]
    for n, u in units.items():
        if u < L - 1:
            poisoned[0][n] = np.full_like(grads[0][n], np.nan)
    b, _ = oracle.aggregate_update(units, L, params, vel, poisoned, depths, 0.1, 0.9, 0.0, True)
    for n in params:
        assert np.array_equal(a[n], b[n])
