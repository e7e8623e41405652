"""The backward pass launched eagerly runs weight gradients on a second stream of the library's own.  Every
kernel sums in a fixed order, so the gradients must come out bit for bit as in the single-stream order, which
the library keeps while kernels are being timed and while the caller's stream is being captured into a graph."""
import pytest
import torch

import paper_2111_10672_amd as spb
import workloads as wl

pytestmark = pytest.mark.gpu


def _grads(model, dev, k, how):
    for g in model.grads:
        g.fill_(float("nan"))
    if how == "graph":
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            model.step(dev, k)               # first call outside capture
            stream.synchronize()
            for g in model.grads:
                g.fill_(float("nan"))
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                model.step(dev, k)
            graph.replay()
            stream.synchronize()
    else:
        spb.spb_set_kernel_timing(model.handle, how == "timed")
        model.step(dev, k)
        torch.cuda.synchronize()
        spb.spb_set_kernel_timing(model.handle, False)
    return float(model.loss.item()), {n: g.clone() for n, g in model.grad_dict(k).items()}


@pytest.mark.parametrize("name", ["small_encoder_bf16", "fused_attention_encoder_bf16", "small_resnet_basic_bf16",
                                  "small_resnet_bottleneck_bf16", "small_resnet101_bf16", "ragged_mlp_f32"])
def test_two_stream_backward_gives_the_single_stream_bits(name):
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, 0, True), wl.make_batch(cfg, 0)
    n_units = wl.unit_count(cfg)
    model = spb.SpbModel(cfg, params)
    try:
        dev = {n: t.cuda() for n, t in batch.items()}
        for k in sorted({1, max(1, n_units // 2), n_units}):
            print(f"case {name} k={k}", flush=True)
            loss_a, eager = _grads(model, dev, k, "eager")
            for how in ("timed", "graph", "eager"):
                loss_b, other = _grads(model, dev, k, how)
                assert loss_a == loss_b
                assert set(eager) == set(other)
                for n in eager:
                    assert torch.equal(eager[n], other[n]), f"{name} k={k}: {n} differs between eager and {how}"
    finally:
        model.close()


@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_two_stream_backward_at_full_size(name):
    """At full size the two streams' kernels really overlap on the chip (tens of microseconds each); a buffer handed
    from one stream to the other too early shows up as a difference from the single-stream order."""
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, 0), wl.make_batch(cfg, 0)
    model = spb.SpbModel(cfg, params)
    try:
        dev = {n: t.cuda() for n, t in batch.items()}
        k = wl.depth_sweep(cfg)[-1]
        print(f"case {name} k={k}", flush=True)
        loss_a, serial = _grads(model, dev, k, "timed")
        for rep in range(3):
            loss_b, eager = _grads(model, dev, k, "eager")
            assert loss_a == loss_b
            for n in serial:
                assert torch.equal(serial[n], eager[n]), f"{name} k={k} repetition {rep}: {n} differs"
    finally:
        model.close()
