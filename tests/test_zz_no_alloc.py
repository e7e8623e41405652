"""The forward entry point that allocates nothing (spb_forward_static: the workspace is a fixed-size device array the
library holds) against spb_forward on a caller workspace: same kernels, so the loss and every gradient must be the
same bits.  Two steps in a row on the shared array, the second with a smaller model and batch, then the refusal of
a depth that does not fit."""
import pytest
import torch

import paper_2111_10672_amd as spb
import workloads as wl

pytestmark = pytest.mark.gpu


def _both_ways(name, k, seed):
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, seed, True), wl.make_batch(cfg, seed)
    dev = {n: t.cuda() for n, t in batch.items()}
    ref = spb.SpbModel(cfg, params)
    ref.step(dev, k)
    torch.cuda.synchronize()
    want = {n: g.clone() for n, g in ref.grad_dict(k).items()}
    want_loss = ref.loss.clone()
    ref.close()

    m = spb.SpbModel(cfg, params)
    assert spb.spb_workspace_size(m.handle, k) <= spb.SPB_STATIC_WORKSPACE_BYTES
    for g in m.grads:
        g.fill_(float("nan"))
    import gc
    gc.collect()                                   # tensors of earlier tests must not be freed inside the bracket below
    before = torch.cuda.memory_allocated()
    m.forward_static(dev, k)
    m.backward(k)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() <= before and m.workspace is None      # no caller workspace was ever made
    assert torch.equal(m.loss, want_loss), (name, m.loss.item(), want_loss.item())
    got = m.grad_dict(k)
    assert list(got) == list(want)
    for n, g in got.items():
        assert torch.equal(g, want[n]), (name, n)
    for info, g in zip(m.infos, m.grads):
        if info["unit"] < m.n_units - k:
            assert torch.isnan(g).all(), f"{info['name']} was written below the cut"
    m.close()


def test_static_workspace_forward_matches_the_caller_workspace_forward():
    print("case cfg2 k=8 on the static workspace", flush=True)
    _both_ways("cfg2", 8, 0)                      # 5.9 MB of the 8 MiB array, k-slices and all
    print("case ragged_mlp_bf16 k=3 on the static workspace (smaller, over the first call's leftovers)", flush=True)
    _both_ways("ragged_mlp_bf16", 3, 1)
    print("case cfg1 k=2 on the static workspace (float32)", flush=True)
    _both_ways("cfg1", 2, 0)


def test_static_workspace_refuses_what_does_not_fit():
    cfg = wl.get_config("wide_mlp_bf16")           # 4096 rows: tens of MB of activations
    m = spb.SpbModel(cfg, wl.make_params(cfg, 0))
    dev = {n: t.cuda() for n, t in wl.make_batch(cfg, 0).items()}
    assert spb.spb_workspace_size(m.handle, 2) > spb.SPB_STATIC_WORKSPACE_BYTES
    with pytest.raises(spb.SpbError) as e:
        m.forward_static(dev, 2)
    assert e.value.code == -4 and "static" in str(e.value)
    with pytest.raises(spb.SpbError) as e:          # the refused call left no stash behind
        m.backward(1)
    assert e.value.code == -3
    m.close()
