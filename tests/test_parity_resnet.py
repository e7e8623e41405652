"""GPU parity of the residual-CNN SPB step against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2111_10672_amd as spb
import workloads as wl
from parity import check_gradients

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["small_resnet_basic_bf16", "small_resnet_bottleneck_bf16"])
@pytest.mark.parametrize("perturbed", [True, False])
def test_small_resnets_every_depth(name, perturbed):
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, 0, perturbed), wl.make_batch(cfg, 0)
    n_units = wl.unit_count(cfg)
    exact_loss, exact = oracle.spb_step(cfg, params, batch, n_units)
    ref_loss, ref = oracle.spb_step(cfg, params, batch, n_units, oracle.round_to_bf16)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    for k in range(n_units + 1):
        print(f"case {name} perturbed={perturbed} k={k}", flush=True)
        model = spb.SpbModel(cfg, params)
        try:
            dev = {n: t.cuda() for n, t in batch.items()}
            for g in model.grads:
                g.fill_(float("nan"))
            model.step(dev, k)
            torch.cuda.synchronize()
            assert abs(model.loss.item() - ref_loss) <= 5e-3 * abs(ref_loss), (model.loss.item(), ref_loss)
            gpu = {n: g.double().cpu().numpy() for n, g in model.grad_dict(k).items()}
            want = {n for n, u in unit_of.items() if u >= n_units - k}
            assert set(gpu) == want
            check_gradients(gpu, {n: ref[n] for n in want}, "bf16", {n: exact[n] for n in want})
            for info, g in zip(model.infos, model.grads):
                if info["unit"] < n_units - k:
                    assert torch.isnan(g).all(), f"{info['name']} was written below the cut"
        finally:
            model.close()


def test_mid_size_bottlenecks_element_by_element():
    """56x56 images at batch 8 through a 64 -> 256 bottleneck stage and a stride-2 128 -> 512 block: 25088 and 6272
    pixel rows, which take the 128-row and 256-row gathered tiles, the one-tap path at 64 and 128 channels, a
    stride-2 input gradient and weight gradients cut into many k-slices.  Every entry against the oracle."""
    name = "mid_resnet_bottleneck_bf16"
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, 0, True), wl.make_batch(cfg, 0)
    n_units = wl.unit_count(cfg)
    print(f"case {name}: oracle, exact", flush=True)
    _, exact = oracle.spb_step(cfg, params, batch, n_units)
    print(f"case {name}: oracle, bfloat16 storage", flush=True)
    ref_loss, ref = oracle.spb_step(cfg, params, batch, n_units, oracle.round_to_bf16)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    model = spb.SpbModel(cfg, params)
    try:
        dev = {n: t.cuda() for n, t in batch.items()}
        for k in (n_units, 2):
            print(f"case {name} k={k}", flush=True)
            for g in model.grads:
                g.fill_(float("nan"))
            model.step(dev, k)
            torch.cuda.synchronize()
            assert abs(model.loss.item() - ref_loss) <= 5e-3 * abs(ref_loss)
            gpu = {n: g.double().cpu().numpy() for n, g in model.grad_dict(k).items()}
            want = {n for n, u in unit_of.items() if u >= n_units - k}
            assert set(gpu) == want
            check_gradients(gpu, {n: ref[n] for n in want}, "bf16", {n: exact[n] for n in want}, label=f"{name} k={k}")
    finally:
        model.close()


def test_resnet_workspace_grows_with_depth():
    cfg = wl.get_config("small_resnet_bottleneck_bf16")
    m = spb.spb_model_create(spb.desc_from_config(cfg))
    sizes = [spb.spb_workspace_size(m, k) for k in range(wl.unit_count(cfg) + 1)]
    spb.spb_model_destroy(m)
    assert all(b >= a for a, b in zip(sizes, sizes[1:])) and sizes[-1] > sizes[0]


def test_resnet101_style_stack_at_table1_depths():
    """The 35-unit stack of the Table-1-shaped report, at toy widths, at a few of its depths."""
    cfg = wl.get_config("small_resnet101_bf16")
    params, batch = wl.make_params(cfg, 0, True), wl.make_batch(cfg, 0)
    n_units = wl.unit_count(cfg)
    assert n_units == 35
    _, exact = oracle.spb_step(cfg, params, batch, n_units)
    ref_loss, ref = oracle.spb_step(cfg, params, batch, n_units, oracle.round_to_bf16)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    model = spb.SpbModel(cfg, params)
    try:
        dev = {n: t.cuda() for n, t in batch.items()}
        for k in wl.depth_sweep(cfg):
            print(f"case small_resnet101_bf16 k={k}", flush=True)
            for g in model.grads:
                g.fill_(float("nan"))
            model.step(dev, k)
            torch.cuda.synchronize()
            assert abs(model.loss.item() - ref_loss) <= 5e-3 * abs(ref_loss)
            gpu = {n: g.double().cpu().numpy() for n, g in model.grad_dict(k).items()}
            want = {n for n, u in unit_of.items() if u >= n_units - k}
            assert set(gpu) == want
            check_gradients(gpu, {n: ref[n] for n in want}, "bf16", {n: exact[n] for n in want})
            for info, g in zip(model.infos, model.grads):
                if info["unit"] < n_units - k:
                    assert torch.isnan(g).all(), f"{info['name']} was written below the cut"
    finally:
        model.close()
