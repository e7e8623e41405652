"""Parameter-server side of one SPB iteration on the CPU (oracle side, test infrastructure).

Sec. 2 of the paper: every worker sends the gradients of the suffix it backpropagated; the server averages each
layer's gradient over the workers that contributed to it, scales the learning rate with that number, and updates
its copy of the model.  Sec. 4.1 names the optimizer: SGD with momentum and weight decay.  Everything is float64;
`q` rounds a parameter to its storage type after the update (identity, or round_to_bf16).

Readings where the paper is silent: worker j of K backpropagates ceil(j L / K) units (rounded up, so that worker K
is always complete); the learning rate of a parameter with c contributors is lr * c / K; the update is
v <- mu v + (g + wd w), w <- w - rate v (no dampening, no Nesterov term); a parameter without contributors is left
as it is, velocity included.
"""
from __future__ import annotations

import math

import numpy as np


def worker_depths(n_units: int, n_workers: int) -> list:
    """Depth (units from the output end) of workers 1..K: ceil(j L / K)."""
    return [math.ceil(j * n_units / n_workers) for j in range(1, n_workers + 1)]


def contributors(unit: int, n_units: int, depths) -> list:
    """Indices of the workers whose suffix reaches down to `unit`."""
    return [j for j, k in enumerate(depths) if unit >= n_units - k]


def aggregate_update(param_units: dict, n_units: int, params: dict, velocity: dict, worker_grads: list, depths,
                     lr: float, momentum: float, weight_decay: float, scale_lr: bool, q=lambda a: a):
    """One server step.  param_units: name -> owning unit.  Returns (new params, new velocity) as float64 arrays."""
    new_w, new_v = {}, {}
    n_workers = len(depths)
    for name, unit in param_units.items():
        w = np.asarray(params[name], dtype=np.float64)
        v = np.asarray(velocity[name], dtype=np.float64)
        who = contributors(unit, n_units, depths)
        if not who:
            new_w[name], new_v[name] = w.copy(), v.copy()
            continue
        g = np.zeros_like(w)
        for j in who:
            g = g + np.asarray(worker_grads[j][name], dtype=np.float64)
        g = g / len(who)
        rate = lr * len(who) / n_workers if scale_lr else lr
        v = momentum * v + (g + weight_decay * w)
        new_v[name] = v
        new_w[name] = q(w - rate * v)
    return new_w, new_v
