"""Full-size workloads on the GPU, in the launch configuration bench.py times, against sampled entries of the
oracle's gradients (tests/golden/*.json, written by tests/golden/make_golden.py from oracle/ alone).

Per gradient tensor the file holds 96 seeded entries, the largest magnitude and the Frobenius norm of the
oracle's result.  Checked here: the sampled entries (error measured against the tensor's largest magnitude),
the norm of the whole GPU tensor against the stored norm, the loss, and which parameters are listed.
"""
import json
import os

import numpy as np
import pytest
import torch

import paper_2111_10672_amd as spb
import workloads as wl
from parity import TOL

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_full_size_depth_sweep_against_golden_samples(name):
    seed = 0
    with open(os.path.join(GOLDEN, f"{name}_seed{seed}.json")) as f:
        gold = json.load(f)
    cfg = wl.get_config(name)
    n_units = wl.unit_count(cfg)
    assert gold["depth"] == n_units
    params, batch = wl.make_params(cfg, seed), wl.make_batch(cfg, seed)
    unit_of = {n: u for n, _s, u, _i in wl.tensor_specs(cfg)}
    model = spb.SpbModel(cfg, params)
    dev = {n: t.cuda() for n, t in batch.items()}
    tol = TOL[cfg["dtype"]]
    try:
        for k in wl.depth_sweep(cfg) + [n_units]:
            print(f"case {name} k={k}", flush=True)
            for g in model.grads:
                g.fill_(float("nan"))
            model.step(dev, k)
            torch.cuda.synchronize()
            assert abs(model.loss.item() - gold["loss"]) <= 5e-3 * abs(gold["loss"])
            got = model.grad_dict(k)
            assert set(got) == {n for n, u in unit_of.items() if u >= n_units - k}
            worst = (0.0, "")
            for pname, g in got.items():
                ref = gold["tensors"][pname]
                assert list(g.shape) == ref["shape"]
                assert torch.isfinite(g).all(), pname
                idx = torch.tensor(ref["index"], device=g.device)
                vals = g.reshape(-1)[idx].double().cpu().numpy()
                err = np.abs(vals - np.array(ref["value"])).max() / ref["max_abs"]
                bound = max(tol, ref["exact_rel_max"])
                assert err <= bound, f"{pname} k={k}: sampled rel_max {err:.3e} > {bound:.3e}"
                fro = float(torch.linalg.vector_norm(g.double()).item())
                ferr = abs(fro - ref["fro"]) / ref["fro"]
                fbound = max(tol, ref["exact_rel_fro"])
                assert ferr <= fbound, f"{pname} k={k}: norm off by {ferr:.3e} > {fbound:.3e}"
                worst = max(worst, (err / bound, pname))
            print(f"  worst sampled error / bound = {worst[0]:.3f} ({worst[1]})", flush=True)
            for info, g in zip(model.infos, model.grads):
                if info["unit"] < n_units - k:
                    assert torch.isnan(g).all(), f"{info['name']} was written below the cut"
    finally:
        model.close()
