"""Server-side aggregation and update on the GPU against the oracle, through the C ABI (Sec. 2: per-layer average
over the contributing workers, rate scaled with their number; Sec. 4.1: SGD with momentum and weight decay)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2111_10672_amd as spb
import workloads as wl

pytestmark = pytest.mark.gpu


def _run(name, depths, scale_lr, seed=0, lr=0.05, mu=0.9, wd=1e-4):
    cfg = wl.get_config(name)
    params = wl.make_params(cfg, seed, perturbed=True)
    model = spb.SpbModel(cfg, params, "cuda:0")
    names = [i["name"] for i in model.infos]
    units = {i["name"]: i["unit"] for i in model.infos}
    vel = wl.make_velocity(cfg, seed)
    grads = wl.make_worker_grads(cfg, seed, len(depths))
    dev_vel = [vel[n].cuda() for n in names]
    # a worker's buffers below its cut are poisoned: they must never be read
    dev_grads = []
    for j, k in enumerate(depths):
        per = []
        for n in names:
            g = grads[j][n].cuda()
            if units[n] < model.n_units - k:
                g = torch.full_like(g, float("nan"))
            per.append(g)
        dev_grads.append(per)
    spb.spb_aggregate_update(model.handle, depths, dev_grads, dev_vel, lr, mu, wd, scale_lr, model.stream())
    torch.cuda.synchronize()
    q = oracle.round_to_bf16 if cfg["dtype"] == "bf16" else oracle.identity
    ref_w, ref_v = oracle.aggregate_update(units, model.n_units, {n: params[n].double().numpy() for n in names},
                                           {n: vel[n].double().numpy() for n in names},
                                           [{n: g[n].double().numpy() for n in names} for g in grads], depths, lr, mu, wd, scale_lr, q)
    for i, n in enumerate(names):
        w = model.params[i].double().cpu().numpy()
        v = dev_vel[i].double().cpu().numpy()
        assert np.isfinite(w).all() and np.isfinite(v).all(), n
        touched = bool(oracle.contributors(units[n], model.n_units, depths))
        if not touched:      # nobody reached it: bit-identical to the input
            assert np.array_equal(w, params[n].double().numpy()) and np.array_equal(v, vel[n].double().numpy()), n
            continue
        # float32 arithmetic on values of order 1: a few ulp; a bfloat16 parameter may land one rounding step away
        # where the float32 and float64 updates fall on different sides of a rounding boundary
        np.testing.assert_allclose(v, ref_v[n], rtol=0, atol=1e-6 * max(1.0, np.abs(ref_v[n]).max()), err_msg=n)
        if cfg["dtype"] == "bf16":
            assert (np.abs(w - ref_w[n]) <= 2.0 ** -7 * np.maximum(np.abs(ref_w[n]), 2.0 ** -126)).all(), n
            assert (w != ref_w[n]).mean() <= 1e-2, n
        else:
            np.testing.assert_allclose(w, ref_w[n], rtol=0, atol=1e-6 * max(1.0, np.abs(ref_w[n]).max()), err_msg=n)
    model.close()


@pytest.mark.parametrize("scale_lr", [True, False])
def test_mlp_f32_ragged_shapes(scale_lr):
    _run("ragged_mlp_f32", [1, 2, 4], scale_lr)        # last dim 7: tensors whose size is not a multiple of 4


def test_depth_rule_of_the_library_matches_the_oracle_and_full_depth_everywhere():
    cfg = wl.get_config("cfg2")
    m = spb.spb_model_create(spb.desc_from_config(cfg))
    L = wl.unit_count(cfg)
    for K in range(1, 9):
        assert [spb.spb_worker_depth(m, j, K) for j in range(1, K + 1)] == oracle.worker_depths(L, K)
    spb.spb_model_destroy(m)
    _run("ragged_mlp_bf16", [4, 4, 4, 4], True)


def test_cfg2_four_workers_at_the_paper_depth_rule():
    _run("cfg2", oracle.worker_depths(8, 4), True)


def test_some_parameters_unreached_and_eight_workers():
    _run("small_encoder_bf16", [0, 1, 1, 2, 2, 3, 3, 3], True)   # unit 0 (embedding) is below every cut
    _run("small_resnet_basic_bf16", [2, 3], False)


def test_emulated_iteration_of_three_workers_end_to_end():
    """Three workers' truncated steps on the GPU (own batches, depths ceil(j L / 3), own gradient buffers), then the
    server-side update, against the same iteration done by the oracle throughout."""
    cfg = wl.get_config("ragged_mlp_f32")
    params = wl.make_params(cfg, 0, perturbed=True)
    model = spb.SpbModel(cfg, params, "cuda:0")
    names = [i["name"] for i in model.infos]
    units = {i["name"]: i["unit"] for i in model.infos}
    L, K, lr, mu, wd = model.n_units, 3, 0.05, 0.9, 1e-4
    depths = [spb.spb_worker_depth(model.handle, j, K) for j in range(1, K + 1)]
    assert depths == oracle.worker_depths(L, K) == [2, 3, 4]
    vel = wl.make_velocity(cfg, 0)
    dev_vel = [vel[n].cuda() for n in names]
    batches = [wl.make_batch(cfg, 10 + j) for j in range(K)]
    worker_bufs = [[torch.full_like(g, float("nan")) for g in model.grads] for _ in range(K)]
    for j, k in enumerate(depths):
        spb.spb_bind_grads(model.handle, worker_bufs[j])
        model.step({n: t.cuda() for n, t in batches[j].items()}, k)
    spb.spb_aggregate_update(model.handle, depths, worker_bufs, dev_vel, lr, mu, wd, True, model.stream())
    torch.cuda.synchronize()
    ref_grads = [oracle.spb_step(cfg, params, batches[j], k)[1] for j, k in enumerate(depths)]
    old = {n: params[n].double().numpy() for n in names}
    ref_w, ref_v = oracle.aggregate_update(units, L, old, {n: vel[n].double().numpy() for n in names}, ref_grads, depths, lr, mu, wd, True)
    for i, n in enumerate(names):
        step_ref = ref_w[n] - old[n]
        step_gpu = model.params[i].double().cpu().numpy() - old[n]
        if not np.any(step_ref):
            assert not np.any(step_gpu), n
            continue
        # the step is a few 1e-3 of a weight stored in float32: its own rounding (6e-8 of the weight) sets the floor
        assert np.abs(step_gpu - step_ref).max() <= 1e-4 * np.abs(step_ref).max() + 2e-7 * np.abs(old[n]).max(), n
        np.testing.assert_allclose(dev_vel[i].double().cpu().numpy(), ref_v[n], rtol=0, atol=1e-4 * np.abs(ref_v[n]).max(), err_msg=n)
    model.close()
