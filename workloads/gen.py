"""Seeded tensor generators.

Every tensor is drawn from its own counter-based stream (numpy's Philox keyed
by the seed and a hash of the tensor's name), in float64, and rounded once to
the workload's storage type.  Consumers on both sides start from the rounded
values.
"""
from __future__ import annotations

import zlib

import numpy as np
import torch

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def _stream(seed: int, name: str) -> np.random.Generator:
    key = (int(seed) & 0xFFFFFFFF) | (zlib.crc32(name.encode()) << 32)
    return np.random.Generator(np.random.Philox(key=key))


def _normal(seed, name, shape, std):
    return _stream(seed, name).standard_normal(size=shape) * std


def _store(arr: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(arr)).to(_TORCH_DTYPE[dtype])


def tensor_specs(cfg: dict) -> list:
    """[(name, shape, unit, init)] in unit order, input end first.

    init: ("normal", std) | ("const", value)
    """
    fam = cfg["family"]
    specs = []
    if fam == "mlp":
        dims = cfg["dims"]
        for i in range(len(dims) - 1):
            fan_in = dims[i]
            specs.append((f"fc{i}.weight", (dims[i + 1], dims[i]), i, ("normal", (2.0 / fan_in) ** 0.5)))
            specs.append((f"fc{i}.bias", (dims[i + 1],), i, ("const", 0.0)))
        return specs
    if fam in ("resnet_basic", "resnet_bottleneck"):
        from .configs import resnet_layout
        lay = resnet_layout(cfg)

        def conv(name, unit, cout, k, cin):      # weights are [Cout, R, S, Cin]; He-normal with fan_in = Cin * R * S
            specs.append((name + ".weight", (cout, k, k, cin), unit, ("normal", (2.0 / (cin * k * k)) ** 0.5)))

        def affine(name, unit, c):               # the folded BatchNorm: trainable per-channel scale and shift
            specs.append((name + ".scale", (c,), unit, ("const", 1.0)))
            specs.append((name + ".shift", (c,), unit, ("const", 0.0)))

        st = lay["stem"]
        conv("stem.conv", 0, st["cout"], st["kernel"], st["cin"])
        affine("stem.aff", 0, st["cout"])
        for blk in lay["blocks"]:
            u, pre = blk["index"] + 1, f"block{blk['index']}."
            if lay["bottleneck"]:
                chain = [(1, blk["cin"], blk["mid"]), (3, blk["mid"], blk["mid"]), (1, blk["mid"], blk["cout"])]
            else:
                chain = [(3, blk["cin"], blk["cout"]), (3, blk["cout"], blk["cout"])]
            for j, (k, ci, co) in enumerate(chain, start=1):
                conv(f"{pre}conv{j}", u, co, k, ci)
                affine(f"{pre}aff{j}", u, co)
            if blk["proj"]:
                conv(pre + "proj", u, blk["cout"], 1, blk["cin"])
                affine(pre + "projaff", u, blk["cout"])
        u = len(lay["blocks"]) + 1
        specs.append(("head.fc.weight", (cfg["classes"], lay["features"]), u, ("normal", (2.0 / lay["features"]) ** 0.5)))
        specs.append(("head.fc.bias", (cfg["classes"],), u, ("const", 0.0)))
        return specs
    if fam == "encoder":
        h, f, v, seq = cfg["hidden"], cfg["ffn"], cfg["vocab"], cfg["seq"]
        std = 0.02
        specs.append(("embed.tok.weight", (v, h), 0, ("normal", std)))
        specs.append(("embed.pos.weight", (seq, h), 0, ("normal", std)))
        for i in range(cfg["layers"]):
            u, pre = i + 1, f"layer{i}."
            specs += [
                (pre + "ln1.weight", (h,), u, ("const", 1.0)), (pre + "ln1.bias", (h,), u, ("const", 0.0)),
                (pre + "attn.qkv.weight", (3 * h, h), u, ("normal", std)), (pre + "attn.qkv.bias", (3 * h,), u, ("const", 0.0)),
                (pre + "attn.out.weight", (h, h), u, ("normal", std)), (pre + "attn.out.bias", (h,), u, ("const", 0.0)),
                (pre + "ln2.weight", (h,), u, ("const", 1.0)), (pre + "ln2.bias", (h,), u, ("const", 0.0)),
                (pre + "ffn.w1.weight", (f, h), u, ("normal", std)), (pre + "ffn.w1.bias", (f,), u, ("const", 0.0)),
                (pre + "ffn.w2.weight", (h, f), u, ("normal", std)), (pre + "ffn.w2.bias", (h,), u, ("const", 0.0)),
            ]
        u = cfg["layers"] + 1
        specs += [("head.ln.weight", (h,), u, ("const", 1.0)), ("head.ln.bias", (h,), u, ("const", 0.0)),
                  ("head.vocab.weight", (v, h), u, ("normal", std)), ("head.vocab.bias", (v,), u, ("const", 0.0))]
        return specs
    raise NotImplementedError(fam)


def make_params(cfg: dict, seed: int = 0, perturbed: bool = False) -> dict:
    """name -> CPU tensor in the workload's storage type.

    perturbed=True replaces the constant initial values (zero biases and
    shifts, unit scales) by values with a N(0, 0.1^2) spread, so that a missing
    bias add or scale cannot hide behind a neutral element.
    """
    out = {}
    for name, shape, _unit, init in tensor_specs(cfg):
        if init[0] == "normal":
            arr = _normal(seed, name, shape, init[1])
        else:
            arr = np.full(shape, init[1], dtype=np.float64)
            if perturbed:
                arr = arr + _normal(seed, name + "/perturb", shape, 0.1)
        out[name] = _store(arr, cfg["dtype"])
    return out


def make_batch(cfg: dict, seed: int = 0) -> dict:
    fam = cfg["family"]
    if fam == "mlp":
        b, d, c = cfg["batch"], cfg["dims"][0], cfg["dims"][-1]
        x = _store(_normal(seed, "batch/x", (b, d), 1.0), cfg["dtype"])
        labels = _stream(seed, "batch/labels").integers(0, c, size=(b,), dtype=np.int32)
        return {"x": x, "labels": torch.from_numpy(labels)}
    if fam in ("resnet_basic", "resnet_bottleneck"):
        b, (h, w, c) = cfg["batch"], cfg["image"]
        x = _store(_normal(seed, "batch/x", (b, h, w, c), 1.0), cfg["dtype"])        # NHWC
        labels = _stream(seed, "batch/labels").integers(0, cfg["classes"], size=(b,), dtype=np.int32)
        return {"x": x, "labels": torch.from_numpy(labels)}
    if fam == "encoder":
        b, seq, v, rows = cfg["batch"], cfg["seq"], cfg["vocab"], cfg["loss_rows"]
        ids = _stream(seed, "batch/ids").integers(0, v, size=(b, seq), dtype=np.int32)
        # the positions that carry a loss: the first `rows` of a seeded permutation of all b * seq positions
        perm = _stream(seed, "batch/loss_rows").permutation(b * seq)[:rows].astype(np.int32)
        labels = _stream(seed, "batch/labels").integers(0, v, size=(rows,), dtype=np.int32)
        return {"x": torch.from_numpy(ids), "loss_rows": torch.from_numpy(perm), "labels": torch.from_numpy(labels)}
    raise NotImplementedError(fam)


def make_worker_grads(cfg: dict, seed: int, n_workers: int) -> list:
    """Stand-ins for the gradients of n_workers workers: one dict per worker, name -> float32 CPU tensor
    N(0, 0.01^2) of the parameter's shape, for every parameter (which of them a worker of a given depth actually
    sends is decided by whoever consumes them)."""
    return [{name: torch.from_numpy(_normal(seed, f"worker{j}/{name}", shape, 0.01).astype(np.float32))
             for name, shape, _unit, _init in tensor_specs(cfg)} for j in range(n_workers)]


def make_velocity(cfg: dict, seed: int) -> dict:
    """name -> float32 CPU tensor N(0, 0.01^2): the momentum buffers an optimizer would hold mid-training."""
    return {name: torch.from_numpy(_normal(seed, "velocity/" + name, shape, 0.01).astype(np.float32))
            for name, shape, _unit, _init in tensor_specs(cfg)}
