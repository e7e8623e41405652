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
    if fam in ("resnet_basic", "resnet_bottleneck"):
        from workloads import resnet_layout
        lay = resnet_layout(cfg)
        return [StemUnit(lay)] + [ResidualUnit(b, lay["bottleneck"]) for b in lay["blocks"]] + [PooledHeadUnit()]
    if fam == "encoder":
        return [EmbeddingUnit(cfg)] + [EncoderLayerUnit(i, cfg) for i in range(cfg["layers"])] + [MaskedHeadUnit()]
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
    h = b["x"]
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


class EmbeddingUnit:
    """x0[b, s, :] = tok[id[b, s], :] + pos[s, :].  Its gradient is a scatter-add of rows; it is the lowest
    unit, so it never forms an input gradient."""

    param_names = ["embed.tok.weight", "embed.pos.weight"]

    def __init__(self, cfg):
        self.seq = cfg["seq"]

    def forward(self, _x, p, q, batch):
        self.ids = batch["x"].reshape(-1)
        tok, pos = p["embed.tok.weight"], p["embed.pos.weight"]
        self.shapes = tok.shape, pos.shape
        n = self.ids.shape[0]
        return q(tok[self.ids] + pos[np.arange(n) % self.seq])

    def backward(self, dout, p, q, need_input_grad):
        dtok, dpos = np.zeros(self.shapes[0]), np.zeros(self.shapes[1])
        for row in range(dout.shape[0]):           # duplicates add up
            dtok[self.ids[row]] += dout[row]
            dpos[row % self.seq] += dout[row]
        return {"embed.tok.weight": dtok, "embed.pos.weight": dpos}, None


class EncoderLayerUnit:
    """Pre-LayerNorm Transformer layer: h = x + Out(Attn(LN1 x)); out = h + W2 gelu(W1 LN2 h + b1) + b2."""

    def __init__(self, index, cfg):
        self.pre = f"layer{index}."
        self.batch, self.seq, self.heads = cfg["batch"], cfg["seq"], cfg["heads"]
        self.d = cfg["hidden"] // cfg["heads"]
        self.param_names = [self.pre + n for n in (
            "ln1.weight", "ln1.bias", "attn.qkv.weight", "attn.qkv.bias", "attn.out.weight", "attn.out.bias",
            "ln2.weight", "ln2.bias", "ffn.w1.weight", "ffn.w1.bias", "ffn.w2.weight", "ffn.w2.bias")]

    def forward(self, x, p, q, batch):
        P = lambda n: p[self.pre + n]
        hidden = x.shape[1]
        u, self.ln1 = ops.layernorm_fwd(x, P("ln1.weight"), P("ln1.bias"))
        self.u = q(u)
        self.qkv = q(ops.linear_fwd(self.u, P("attn.qkv.weight"), P("attn.qkv.bias")))
        qh, kh, vh = (ops.split_heads(self.qkv[:, i * hidden:(i + 1) * hidden], self.batch, self.seq, self.heads) for i in range(3))
        scores = qh @ kh.transpose(0, 1, 3, 2) / np.sqrt(self.d)
        self.prob = q(ops.softmax_rows(scores))
        self.ctx = q(ops.merge_heads(self.prob @ vh))
        self.h = q(x + ops.linear_fwd(self.ctx, P("attn.out.weight"), P("attn.out.bias")))
        v, self.ln2 = ops.layernorm_fwd(self.h, P("ln2.weight"), P("ln2.bias"))
        self.v = q(v)
        z1 = ops.linear_fwd(self.v, P("ffn.w1.weight"), P("ffn.w1.bias"))
        self.dgelu = q(ops.gelu_grad(z1))    # what a path keeps of z1 for the backward pass: the GELU derivative itself
        self.f = q(ops.gelu_fwd(z1))
        return q(self.h + ops.linear_fwd(self.f, P("ffn.w2.weight"), P("ffn.w2.bias")))

    def backward(self, dout, p, q, need_input_grad):
        P = lambda n: p[self.pre + n]
        g = {}
        hidden = dout.shape[1]
        # feed-forward half
        g[self.pre + "ffn.w2.weight"], g[self.pre + "ffn.w2.bias"], df = ops.linear_bwd(dout, self.f, P("ffn.w2.weight"), True)
        dz1 = q(df * self.dgelu)
        g[self.pre + "ffn.w1.weight"], g[self.pre + "ffn.w1.bias"], dv = ops.linear_bwd(dz1, self.v, P("ffn.w1.weight"), True)
        dv = q(dv)
        dh_ln, g[self.pre + "ln2.weight"], g[self.pre + "ln2.bias"] = ops.layernorm_bwd(dv, P("ln2.weight"), self.ln2)
        dh = q(dout + dh_ln)                 # residual fan-in
        # attention half
        g[self.pre + "attn.out.weight"], g[self.pre + "attn.out.bias"], dctx = ops.linear_bwd(dh, self.ctx, P("attn.out.weight"), True)
        dctx = q(dctx)
        qh, kh, vh = (ops.split_heads(self.qkv[:, i * hidden:(i + 1) * hidden], self.batch, self.seq, self.heads) for i in range(3))
        do = ops.split_heads(dctx, self.batch, self.seq, self.heads)
        dvh = self.prob.transpose(0, 1, 3, 2) @ do
        dprob = do @ vh.transpose(0, 1, 3, 2)
        ds = q(self.prob * (dprob - (dprob * self.prob).sum(axis=-1, keepdims=True)) / np.sqrt(self.d))
        dqh = ds @ kh
        dkh = ds.transpose(0, 1, 3, 2) @ qh
        dqkv = q(np.concatenate([ops.merge_heads(t) for t in (dqh, dkh, dvh)], axis=1))
        g[self.pre + "attn.qkv.weight"], g[self.pre + "attn.qkv.bias"], du = ops.linear_bwd(dqkv, self.u, P("attn.qkv.weight"), True)
        du = q(du)
        dx_ln, g[self.pre + "ln1.weight"], g[self.pre + "ln1.bias"] = ops.layernorm_bwd(du, P("ln1.weight"), self.ln1)
        dx = q(dh + dx_ln) if need_input_grad else None
        return g, dx


class MaskedHeadUnit:
    """Final LayerNorm on the rows that carry a loss, vocabulary projection, softmax cross-entropy."""

    param_names = ["head.ln.weight", "head.ln.bias", "head.vocab.weight", "head.vocab.bias"]

    def forward(self, x, p, q, batch):
        self.rows, self.n_rows_total = batch["loss_rows"], x.shape[0]
        y, self.ln = ops.layernorm_fwd(x[self.rows], p["head.ln.weight"], p["head.ln.bias"])
        self.y = q(y)
        logits = ops.linear_fwd(self.y, p["head.vocab.weight"], p["head.vocab.bias"])
        self.loss_value, self.dz = ops.softmax_ce(logits, batch["labels"])
        return self.loss_value

    def backward(self, _dout, p, q, need_input_grad):
        g = {}
        dz = q(self.dz)
        g["head.vocab.weight"], g["head.vocab.bias"], dy = ops.linear_bwd(dz, self.y, p["head.vocab.weight"], True)
        dy = q(dy)
        dxr, g["head.ln.weight"], g["head.ln.bias"] = ops.layernorm_bwd(dy, p["head.ln.weight"], self.ln)
        dx = None
        if need_input_grad:
            dx = np.zeros((self.n_rows_total, dxr.shape[1]))
            dx[self.rows] = q(dxr)               # loss rows are distinct positions
        return g, dx


# ---- residual CNNs ------------------------------------------------------------------------------------

class _ConvAffine:
    """conv -> per-channel affine, shared by the CNN units.  Keeps the rounded pre-affine output for the scale gradient."""

    def __init__(self, name_conv, name_aff, kernel, stride, pad):
        self.w, self.scale, self.shift = name_conv + ".weight", name_aff + ".scale", name_aff + ".shift"
        self.kernel, self.stride, self.pad = kernel, stride, pad
        self.param_names = [self.w, self.scale, self.shift]

    def forward(self, x, p, q):
        self.x = x
        y = ops.conv_fwd(x, p[self.w], self.stride, self.pad)
        self.y = q(y)
        return ops.affine_fwd(y, p[self.scale], p[self.shift])          # not yet rounded: the caller adds and activates first

    def backward(self, dz, p, q, need_dx):
        """dz: gradient at the affine's output (already masked by the activation that followed)."""
        dy, dscale, dshift = ops.affine_bwd(dz, self.y, p[self.scale])
        dy = q(dy)
        g = {self.w: ops.conv_wgrad(self.x, dy, self.kernel, self.stride, self.pad), self.scale: dscale, self.shift: dshift}
        dx = ops.conv_dgrad(dy, p[self.w], self.x.shape[1:3], self.stride, self.pad) if need_dx else None
        return g, dx


class StemUnit:
    def __init__(self, lay):
        st = lay["stem"]
        self.conv = _ConvAffine("stem.conv", "stem.aff", st["kernel"], st["stride"], st["pad"])
        self.pool = st["pool"]
        self.param_names = self.conv.param_names

    def forward(self, x, p, q, batch):
        self.a = q(ops.relu_fwd(self.conv.forward(x, p, q)))
        if not self.pool:
            return self.a
        out, self.arg = ops.maxpool3x3s2_fwd(self.a)
        return out

    def backward(self, dout, p, q, need_input_grad):
        da = q(ops.maxpool3x3s2_bwd(dout, self.arg, self.a.shape[1:3])) if self.pool else dout
        g, _ = self.conv.backward(da * (self.a > 0), p, q, False)   # the stem is the lowest unit: no input gradient
        return g, None


class ResidualUnit:
    """Basic block (3x3, 3x3) or bottleneck (1x1, 3x3 carrying the stride, 1x1): out = relu(main(x) + shortcut(x))."""

    def __init__(self, blk, bottleneck):
        pre = f"block{blk['index']}."
        if bottleneck:
            spec = [(1, 1, 0), (3, blk["stride"], 1), (1, 1, 0)]
        else:
            spec = [(3, blk["stride"], 1), (3, 1, 1)]
        self.convs = [_ConvAffine(f"{pre}conv{j}", f"{pre}aff{j}", k, s, pd) for j, (k, s, pd) in enumerate(spec, start=1)]
        self.proj = _ConvAffine(pre + "proj", pre + "projaff", 1, blk["stride"], 0) if blk["proj"] else None
        self.param_names = [n for c in self.convs for n in c.param_names] + (self.proj.param_names if self.proj else [])

    def forward(self, x, p, q, batch):
        shortcut = q(self.proj.forward(x, p, q)) if self.proj else x
        h = x
        self.acts = []
        for conv in self.convs[:-1]:
            h = q(ops.relu_fwd(conv.forward(h, p, q)))
            self.acts.append(h)
        self.out = q(ops.relu_fwd(self.convs[-1].forward(h, p, q) + shortcut))
        return self.out

    def backward(self, dout, p, q, need_input_grad):
        g = {}
        dsum = dout * (self.out > 0)                  # flows into both branches of the add
        d = dsum
        for j in range(len(self.convs) - 1, -1, -1):
            first = j == 0
            gj, dx = self.convs[j].backward(d, p, q, need_dx=(not first) or need_input_grad)
            g.update(gj)
            if not first:
                d = q(dx) * (self.acts[j - 1] > 0)
        dx_main = dx
        if self.proj:
            gp, dx_sc = self.proj.backward(dsum, p, q, need_input_grad)
            g.update(gp)
            dx_sc = q(dx_sc) if need_input_grad else None
        else:
            dx_sc = dsum
        return g, (q(dx_main + dx_sc) if need_input_grad else None)


class PooledHeadUnit:
    param_names = ["head.fc.weight", "head.fc.bias"]

    def forward(self, x, p, q, batch):
        self.hw = x.shape[1:3]
        self.pooled = q(ops.avgpool_fwd(x))
        logits = ops.linear_fwd(self.pooled, p["head.fc.weight"], p["head.fc.bias"])
        self.loss_value, self.dz = ops.softmax_ce(logits, batch["labels"])
        return self.loss_value

    def backward(self, _dout, p, q, need_input_grad):
        dz = q(self.dz)
        dw, db, dp = ops.linear_bwd(dz, self.pooled, p["head.fc.weight"], need_input_grad)
        dx = q(ops.avgpool_bwd(q(dp), self.hw)) if need_input_grad else None
        return {"head.fc.weight": dw, "head.fc.bias": db}, dx
