"""GPU parity of the perceptron SPB step against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2111_10672_amd as spb
import workloads as wl
from parity import check_gradients

pytestmark = pytest.mark.gpu

POISON = float("nan")


def _run(cfg, seed, k, perturbed, stash_k=None):
    params, batch = wl.make_params(cfg, seed, perturbed), wl.make_batch(cfg, seed)
    model = spb.SpbModel(cfg, params)
    dev = {n: t.cuda() for n, t in batch.items()}
    for g in model.grads:
        g.fill_(POISON)
    model.forward(dev, k if stash_k is None else stash_k)
    model.backward(k)
    torch.cuda.synchronize()
    return model, params, batch


def _compare(cfg, seed, k, perturbed=False):
    print(f"case {cfg['name']} seed={seed} k={k} perturbed={perturbed}", flush=True)
    model, params, batch = _run(cfg, seed, k, perturbed)
    try:
        exact_loss, exact = oracle.spb_step(cfg, params, batch, k)
        if cfg["dtype"] == "bf16":
            ref_loss, ref = oracle.spb_step(cfg, params, batch, k, oracle.round_to_bf16)
        else:
            ref_loss, ref = exact_loss, exact
        loss = model.loss.item()
        assert abs(loss - ref_loss) <= (1e-4 if cfg["dtype"] == "f32" else 5e-3) * abs(ref_loss), (loss, ref_loss)
        gpu = {n: g.double().cpu().numpy() for n, g in model.grad_dict(k).items()}
        report = []
        check_gradients(gpu, ref, cfg["dtype"], exact, report, label=f"{cfg['name']} seed={seed} k={k}")
        # below the cut: not listed and never written
        listed = set(gpu)
        for info, g in zip(model.infos, model.grads):
            if info["unit"] < model.n_units - k:
                assert info["name"] not in listed
                assert torch.isnan(g).all(), f"{info['name']} was written below the cut"
        return report
    finally:
        model.close()


@pytest.mark.parametrize("name", ["tiny_mlp_f32", "ragged_mlp_f32", "ragged_mlp_bf16", "one_layer_bf16", "many_class_mlp_bf16",
                                  "many_class_mlp_f32"])
def test_small_and_ragged_every_depth(name):
    cfg = wl.get_config(name)
    for k in range(wl.unit_count(cfg) + 1):
        _compare(cfg, 0, k, perturbed=True)
    _compare(cfg, 1, wl.unit_count(cfg), perturbed=False)


@pytest.mark.parametrize("name", ["wide_mlp_bf16", "big_tile_mlp_bf16"])
def test_wide_perceptron_through_the_large_tiles(name):
    """4096 rows against 768 / 3072 / 2304 columns, and 8192 x 4096 results: every product takes one of the large
    tiles.  The oracle runs once, at full depth; gradients above a cut do not depend on the cut, so depth 2 is checked
    against the same."""
    cfg = wl.get_config(name)
    n_units = wl.unit_count(cfg)
    params, batch = wl.make_params(cfg, 0, True), wl.make_batch(cfg, 0)
    print(f"case {name}: oracle, exact", flush=True)
    _, exact = oracle.spb_step(cfg, params, batch, n_units)
    print(f"case {name}: oracle, bfloat16 storage", flush=True)
    ref_loss, ref = oracle.spb_step(cfg, params, batch, n_units, oracle.round_to_bf16)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    for k in (n_units, 2):
        print(f"case {name} k={k}", flush=True)
        model, _, _ = _run(cfg, 0, k, True)
        try:
            assert abs(model.loss.item() - ref_loss) <= 5e-3 * abs(ref_loss)
            gpu = {n: g.double().cpu().numpy() for n, g in model.grad_dict(k).items()}
            want = {n for n, u in unit_of.items() if u >= n_units - k}
            assert set(gpu) == want
            check_gradients(gpu, {n: ref[n] for n in want}, "bf16", {n: exact[n] for n in want})
        finally:
            model.close()


@pytest.mark.parametrize("k", [0, 1, 2, 3, 4])
def test_cfg1_fp32(k):
    _compare(wl.get_config("cfg1"), 0, k)
    if k == 2:
        _compare(wl.get_config("cfg1"), 1, k, perturbed=True)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 6, 7, 8])
def test_cfg2_bf16_depth_sweep(k):
    report = _compare(wl.get_config("cfg2"), 0, k)
    worst = max(report, key=lambda r: r[2] / r[3])
    print(f"  k={k} worst {worst[0]} {worst[1]} err={worst[2]:.3e} bound={worst[3]:.3e}")


def test_listing_order_and_suffix_invariance_on_the_gpu():
    """Views come output end first; the values above the cut do not depend on the cut; the loss does not
    depend on the depth (bitwise: the same kernels run on the same data)."""
    cfg = wl.get_config("ragged_mlp_bf16")
    n_units = wl.unit_count(cfg)
    full_model, _, _ = _run(cfg, 0, n_units, True)
    full = {n: g.clone() for n, g in full_model.grad_dict(n_units).items()}
    full_loss = full_model.loss.clone()
    assert list(full) == [f"fc{u}.{p}" for u in range(n_units - 1, -1, -1) for p in ("weight", "bias")]
    full_model.close()
    for k in range(n_units + 1):
        for stash_k in {k, n_units}:
            m, _, _ = _run(cfg, 0, k, True, stash_k=stash_k)
            got = m.grad_dict(k)
            assert list(got) == list(full)[:2 * k]
            for n, g in got.items():
                assert torch.equal(g, full[n]), (k, n)
            assert torch.equal(m.loss, full_loss)
            m.close()


def test_zero_fill_on_request_and_error_paths():
    cfg = wl.get_config("ragged_mlp_f32")
    n_units = wl.unit_count(cfg)
    m, _, batch = _run(cfg, 0, 2, False)
    spb.spb_zero_absent_grads(m.handle, 2, m.stream())
    torch.cuda.synchronize()
    for info, g in zip(m.infos, m.grads):
        if info["unit"] < n_units - 2:
            assert (g == 0).all()
        else:
            assert torch.isfinite(g).all() and (g != 0).any()
    with pytest.raises(spb.SpbError) as e:              # deeper than the forward pass stashed for
        m.backward(3)
    assert e.value.code == -3
    dev = {n: t.cuda() for n, t in batch.items()}
    with pytest.raises(spb.SpbError) as e:              # workspace too small
        spb.spb_forward(m.handle, dev["x"], dev["labels"], None, n_units, m.workspace, 1024, m.loss, m.stream())
    assert e.value.code == -4
    with pytest.raises(spb.SpbError) as e:              # a failed forward invalidates the stash
        m.backward(1)
    assert e.value.code == -3
    with pytest.raises(spb.SpbError) as e:
        m.forward(dev, n_units + 1)
    assert e.value.code == -2
    m.forward(dev, 1)
    m.backward(0)                                       # legal, enqueues nothing
    assert spb.spb_grad_buffers(m.handle, 0) == []
    torch.cuda.synchronize()
    m.close()


def test_step_replays_identically_from_a_hip_graph():
    cfg = wl.get_config("cfg2")
    params, batch = wl.make_params(cfg, 0), wl.make_batch(cfg, 0)
    m = spb.SpbModel(cfg, params)
    dev = {n: t.cuda() for n, t in batch.items()}
    k = 5
    m.reserve(k)
    m.step(dev, k)
    torch.cuda.synchronize()
    eager = {n: g.clone() for n, g in m.grad_dict(k).items()}
    eager_loss = m.loss.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        m.step(dev, k)                                  # warm-up on the capture stream
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            m.step(dev, k)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        for g in m.grads:
            g.fill_(POISON)
        m.loss.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(m.loss, eager_loss)
        for n, g in m.grad_dict(k).items():
            assert torch.equal(g, eager[n]), n
    m.close()
