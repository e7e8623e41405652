"""GPU parity of the Transformer-encoder SPB step against the CPU oracle, through the C ABI."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2111_10672_amd as spb
import workloads as wl
from parity import check_gradients, rel_max

pytestmark = pytest.mark.gpu


def _step(cfg, params, batch, k):
    model = spb.SpbModel(cfg, params)
    dev = {n: t.cuda() for n, t in batch.items()}
    for g in model.grads:
        g.fill_(float("nan"))
    model.step(dev, k)
    torch.cuda.synchronize()
    return model


@pytest.mark.parametrize("name", ["small_encoder_bf16", "fused_attention_encoder_bf16", "fused_attention_short_bf16",
                                  "wide_encoder_512_bf16", "wide_encoder_1024_bf16", "big_vocab_encoder_bf16"])
@pytest.mark.parametrize("perturbed", [True, False])
def test_small_encoder_every_depth(perturbed, name):
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, 0, perturbed), wl.make_batch(cfg, 0)
    n_units = wl.unit_count(cfg)
    exact_loss, exact = oracle.spb_step(cfg, params, batch, n_units)
    ref_loss, ref = oracle.spb_step(cfg, params, batch, n_units, oracle.round_to_bf16)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    for k in range(n_units + 1):
        print(f"case {name} perturbed={perturbed} k={k}", flush=True)
        model = _step(cfg, params, batch, k)
        try:
            assert abs(model.loss.item() - ref_loss) <= 5e-3 * abs(ref_loss)
            gpu = {n: g.double().cpu().numpy() for n, g in model.grad_dict(k).items()}
            want = {n for n, u in unit_of.items() if u >= n_units - k}
            assert set(gpu) == want                       # the oracle's suffix property makes its depth-L values the reference
            check_gradients(gpu, {n: ref[n] for n in want}, "bf16", {n: exact[n] for n in want})
            for info, g in zip(model.infos, model.grads):
                if info["unit"] < n_units - k:
                    assert torch.isnan(g).all(), f"{info['name']} was written below the cut"
        finally:
            model.close()


def test_encoder_needs_loss_rows_and_replays_from_a_graph():
    cfg = wl.get_config("small_encoder_bf16")
    params, batch = wl.make_params(cfg, 1), wl.make_batch(cfg, 1)
    m = spb.SpbModel(cfg, params)
    dev = {n: t.cuda() for n, t in batch.items()}
    with pytest.raises(spb.SpbError) as e:
        m.forward({"x": dev["x"], "labels": dev["labels"]}, 1)
    assert e.value.code == -1
    k = 3
    m.step(dev, k)
    torch.cuda.synchronize()
    eager = {n: g.clone() for n, g in m.grad_dict(k).items()}
    eager_loss = m.loss.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        m.step(dev, k)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            m.step(dev, k)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        for g in m.grads:
            g.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(m.loss, eager_loss)
        for n, g in m.grad_dict(k).items():
            assert torch.equal(g, eager[n]), n
    m.close()
