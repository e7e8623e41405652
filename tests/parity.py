"""Error measures and tolerances of the parity tests (test infrastructure).

Relative error of a gradient tensor is measured against the tensor's own scale, not element by
element (an element-wise ratio explodes wherever a ReLU zeroes the reference):
    rel_max = max_i |g_i - ref_i| / max_i |ref_i|        rel_fro = ||g - ref||_F / ||ref||_F
float32 workloads: both <= 1e-4 against the exact float64 oracle.
bfloat16 workloads: both <= 2e-2 against the oracle that rounds stored tensors to bfloat16 at the
same places as the HIP path.  A deep ReLU chain at small batch is not well-conditioned under that
rounding: a pre-activation that lands on the other side of zero, or of a rounding boundary, switches
whole terms of a gradient sum, and two correct bfloat16 implementations drift apart layer by layer.
Where the oracle's own two modes (exact, storage-rounded) differ by more than 2e-2 for a tensor, that
difference is the tensor's storage-noise floor and replaces 2e-2 as its bound.  A tensor whose
reference is identically zero must be exactly zero.
"""
from __future__ import annotations

import numpy as np

TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_max(g, ref):
    scale = np.abs(ref).max()
    return float(np.abs(g - ref).max() / scale) if scale > 0 else float(np.abs(g).max())


def rel_fro(g, ref):
    scale = np.linalg.norm(ref)
    return float(np.linalg.norm(g - ref) / scale) if scale > 0 else float(np.linalg.norm(g))


def check_gradients(gpu: dict, ref: dict, dtype: str, exact: dict | None = None, report=None):
    """gpu, ref, exact: name -> float64 arrays.  ref is the gated oracle; exact the float64 one (bf16 only)."""
    assert set(gpu) == set(ref), (sorted(gpu), sorted(ref))
    worst = 0.0
    for name in ref:
        g, r = np.asarray(gpu[name], dtype=np.float64), ref[name]
        assert g.shape == r.shape, name
        assert np.isfinite(g).all(), f"{name}: non-finite gradient"
        for measure in (rel_max, rel_fro):
            tol = TOL[dtype]
            if dtype == "bf16" and exact is not None:
                tol = max(tol, measure(exact[name], r))
            err = measure(g, r)
            worst = max(worst, err)
            if report is not None:
                report.append((name, measure.__name__, err, tol))
            assert err <= tol, f"{name}: {measure.__name__} = {err:.3e} > {tol:.3e}"
    return worst
