"""Full-size workloads on the GPU, in the launch configuration bench.py times, end to end against stored entries of
the oracle's gradients (tests/golden/*.json, written by tests/golden/make_golden.py from oracle/ alone).

Per gradient tensor the file holds the oracle's values (storage-rounded mode, which gates, and exact mode) at 96
seeded entries plus the entries where a tiled kernel fails first: the last 8 x 8 corner, the last row and column,
and the first and last row and column of every band of 256.  Checked here per tensor, over those entries:
    max |g - ref| / max |ref| (the tensor's largest magnitude, stored)      and      ||g - ref|| / ||ref||
against the end-to-end bound of parity.py (2e-2, or the distance between the oracle's two modes where that is larger,
capped).  Every tensor beyond the flat 2e-2 is printed with its error against both modes.  Also checked: the loss,
which parameters are listed, and that nothing below the cut is written.  (Element-by-element checks of whole tensors
at these sizes, one unit at a time, are in test_parity_per_unit.py.)
"""
import json
import os

import numpy as np
import pytest
import torch

import paper_2111_10672_amd as spb
import workloads as wl
from parity import TOL, end_to_end_bound

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
            worst, beyond_flat, entries = (0.0, ""), [], 0
            for pname, g in got.items():
                ref = gold["tensors"][pname]
                assert list(g.shape) == ref["shape"]
                assert torch.isfinite(g).all(), pname
                idx = torch.tensor(ref["index"], device=g.device)
                vals = g.reshape(-1)[idx].double().cpu().numpy()
                want, exact = np.array(ref["value"]), np.array(ref["exact_value"])
                entries += len(want)
                scale_f = np.linalg.norm(want)
                err_m = np.abs(vals - want).max() / ref["max_abs"]
                err_f = np.linalg.norm(vals - want) / scale_f if scale_f > 0 else np.linalg.norm(vals)
                modes_f = np.linalg.norm(exact - want) / scale_f if scale_f > 0 else 0.0
                bound_m = end_to_end_bound(cfg["dtype"], ref["exact_rel_max"])
                bound_f = end_to_end_bound(cfg["dtype"], max(modes_f, ref["exact_rel_fro"]))
                if err_m > tol or err_f > tol:
                    beyond_flat.append(f"    {pname}: max measure {err_m:.3e} (vs exact oracle {np.abs(vals - exact).max() / ref['max_abs']:.3e}, "
                                       f"modes {ref['exact_rel_max']:.3e} apart, bound {bound_m:.3e}); Frobenius over the entries {err_f:.3e} "
                                       f"(vs exact {np.linalg.norm(vals - exact) / scale_f:.3e}, modes {modes_f:.3e} apart, bound {bound_f:.3e})")
                assert err_m <= bound_m, f"{pname} k={k}: max measure {err_m:.3e} > {bound_m:.3e}"
                assert err_f <= bound_f, f"{pname} k={k}: Frobenius measure over the stored entries {err_f:.3e} > {bound_f:.3e}"
                worst = max(worst, (max(err_m / bound_m, err_f / bound_f), pname))
            print(f"  {len(got)} tensors, {entries} stored entries; worst error / bound = {worst[0]:.3f} ({worst[1]}); "
                  f"{len(beyond_flat)} tensor(s) beyond the flat {tol:.0e}", flush=True)
            for line in beyond_flat:
                print(line, flush=True)
            for info, g in zip(model.infos, model.grads):
                if info["unit"] < n_units - k:
                    assert torch.isnan(g).all(), f"{info['name']} was written below the cut"
    finally:
        model.close()
