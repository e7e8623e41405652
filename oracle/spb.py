"""The SPB worker step on the CPU (oracle side, test infrastructure).

Sec. 2 of the paper: a worker runs the complete forward pass to the loss, then
backpropagates over a fixed suffix of the network, starting at the output
layer, and hands over the gradients of that suffix only.  Because a layer's
gradient needs the gradients of every later layer (Sec. 1), the suffix is
visited in order from the output and the walk simply stops after k units.

`q` is the storage rounding: identity for the exact mode; round_to_bf16 for
the mode that mirrors a path which keeps activations and activation gradients
in bfloat16 between layers (arithmetic stays float64 either way).
"""
from __future__ import annotations

import numpy as np

from . import ops


def identity(a):
    return a


class LinearUnit:
    """Linear (+ReLU).  The last unit of a perceptron carries the loss instead."""

    def __init__(self, index, relu, loss):
        self.w, self.b = f"fc{index}.weight", f"fc{index}.bias"
        self.relu, self.loss = relu, loss
        self.param_names = [self.w, self.b]

    def forward(self, x, p, q, batch):
        self.x = x
        self.z = ops.linear_fwd(x, p[self.w], p[self.b])
        if self.loss:
            self.loss_value, self.dz_loss = ops.softmax_ce(self.z, batch["labels"])
            return self.loss_value
        return q(ops.relu_fwd(self.z)) if self.relu else q(self.z)

    def backward(self, dout, p, q, need_input_grad):
        if self.loss:
            dz = q(self.dz_loss)
        else:
            dz = q(ops.relu_bwd(dout, self.z)) if self.relu else dout
        dw, db, dx = ops.linear_bwd(dz, self.x, p[self.w], need_input_grad)
        return {self.w: dw, self.b: db}, dx


def build_units(cfg):
    fam = cfg["family"]
    if fam == "mlp":
        n = len(cfg["dims"]) - 1
        return [LinearUnit(i, relu=(i < n - 1), loss=(i == n - 1)) for i in range(n)]
    raise NotImplementedError(fam)


def _as_f64(t):
    if hasattr(t, "detach"):                      # torch tensor from the generators
        t = t.detach().cpu()
        t = t.double().numpy() if t.is_floating_point() else t.numpy()
    return np.asarray(t)


def spb_step(cfg, params, batch, k, q=identity):
    """One worker step at depth k.  Returns (loss, {param name: gradient}).

    The dictionary holds the parameters of the top k units and nothing else;
    k = 0 gives an empty dictionary, k = L ordinary backpropagation.
    """
    units = build_units(cfg)
    n_units = len(units)
    if not 0 <= k <= n_units:
        raise ValueError(f"depth {k} outside 0..{n_units}")
    p = {name: _as_f64(v) for name, v in params.items()}
    b = {name: _as_f64(v) for name, v in batch.items()}
    h = b["x"] if "x" in b else None
    for unit in units:                            # the forward pass is always complete
        h = unit.forward(h, p, q, b)
    loss = h
    grads = {}
    dout = None
    for index in range(n_units - 1, n_units - k - 1, -1):   # top k units, output end first
        lowest = index == n_units - k
        g, dout = units[index].backward(dout, p, q, need_input_grad=not lowest)
        grads.update(g)
    return loss, grads
