#!/usr/bin/env python3
"""Write tests/golden/<config>_seed<seed>.json: sampled entries of the oracle's gradients at full size.

Calls only workloads/ (seeded inputs) and oracle/ (the CPU reference); nothing from the HIP path.
The oracle runs once at full depth (its gradients above any cut equal the full-depth ones, the suffix
property the CPU tests pin), in the storage-rounded mode that gates bfloat16 workloads and in the exact
float64 mode.  Per gradient tensor the file keeps: shape, largest magnitude, Frobenius norm, the values at
seeded and tile-edge flat indices (see sample_indices), the exact mode's values at the same indices, and how far
the exact mode is from the gated one over the whole tensor (the tensor's storage-noise floor).

    python tests/golden/make_golden.py cfg5 0
"""
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
import workloads as wl  # noqa: E402

N_SAMPLES = 96


def sample_indices(name, shape, seed):
    """Flat indices at which a gradient tensor is kept: 96 seeded entries anywhere, plus the places where a tiled
    kernel goes wrong first, with the tensor seen as [shape[0], everything else]: the last 8 x 8 corner, 16 entries
    along the last row and the last column, and for every band of 256 rows (and of 256 columns) its first and its
    last row (column) at column (row) 0 and at a seeded one."""
    rng = np.random.Generator(np.random.Philox(key=(seed << 32) ^ (hash_name(name) & 0xFFFFFFFF)))
    numel = int(np.prod(shape))
    picked = set(int(i) for i in rng.choice(numel, size=min(N_SAMPLES, numel), replace=False))
    rows = int(shape[0])
    cols = numel // rows
    at = lambda r, c: picked.add(int(r) * cols + int(c))
    for r in range(max(0, rows - 8), rows):
        for c in range(max(0, cols - 8), cols):
            at(r, c)
    for c in np.unique(np.linspace(0, cols - 1, 16).astype(int)):
        at(rows - 1, c)
    for r in np.unique(np.linspace(0, rows - 1, 16).astype(int)):
        at(r, cols - 1)
    for r0 in range(0, rows, 256):
        c = int(rng.integers(cols))
        for r in (r0, min(rows, r0 + 256) - 1):
            at(r, 0)
            at(r, c)
    for c0 in range(0, cols, 256):
        r = int(rng.integers(rows))
        for c in (c0, min(cols, c0 + 256) - 1):
            at(0, c)
            at(r, c)
    return np.array(sorted(picked))


def hash_name(name):
    import zlib
    return zlib.crc32(name.encode())


def main():
    name, seed = sys.argv[1], int(sys.argv[2])
    cfg = wl.get_config(name)
    params, batch = wl.make_params(cfg, seed), wl.make_batch(cfg, seed)
    n_units = wl.unit_count(cfg)
    gated_mode = oracle.round_to_bf16 if cfg["dtype"] == "bf16" else oracle.identity
    t0 = time.time()
    loss, grads = oracle.spb_step(cfg, params, batch, n_units, gated_mode)
    print(f"gated mode done in {time.time() - t0:.0f} s, loss {loss}", flush=True)
    if cfg["dtype"] == "bf16":
        exact_loss, exact = oracle.spb_step(cfg, params, batch, n_units)
        print(f"exact mode done in {time.time() - t0:.0f} s, loss {exact_loss}", flush=True)
    else:
        exact_loss, exact = loss, grads
    out = {"config": name, "seed": seed, "depth": n_units, "loss": loss, "exact_loss": exact_loss, "tensors": {}}
    for pname, g in grads.items():
        flat = g.reshape(-1)
        idx = sample_indices(pname, g.shape, seed)
        max_abs, fro = float(np.abs(flat).max()), float(np.linalg.norm(flat))
        diff = exact[pname].reshape(-1) - flat
        out["tensors"][pname] = {
            "shape": list(g.shape), "max_abs": float(f"{max_abs:.10g}"), "fro": float(f"{fro:.10g}"),
            "index": idx.tolist(), "value": [float(f"{v:.10g}") for v in flat[idx]],
            "exact_value": [float(f"{v:.10g}") for v in exact[pname].reshape(-1)[idx]],
            "exact_rel_max": float(np.abs(diff).max() / max_abs) if max_abs > 0 else 0.0,
            "exact_rel_fro": float(np.linalg.norm(diff) / fro) if fro > 0 else 0.0,
        }
    path = os.path.join(HERE, f"{name}_seed{seed}.json")
    with open(path, "w") as f:
        json.dump(out, f)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
