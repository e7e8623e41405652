"""Shape descriptors of the synthetic workloads.

The paper trains image classifiers (ResNet/VGG families on CIFAR-size images)
and text models (Sec. 4.1); it never prints layer shapes, so the descriptors
below are stand-ins of the same kind: two multilayer perceptrons, a basic-block
and a bottleneck residual CNN, and a pre-LayerNorm Transformer encoder.  Only
shapes live here.

A model is a list of *units*; the backward pass may stop only between units
(Sec. 1 and Sec. 2 speak of a fraction of the layers, counted from the end).
Depth k counts units from the output end.
"""
from __future__ import annotations

import copy

CONFIGS = {
    # Linear 784->256->256->256->10, ReLU between, softmax cross-entropy.
    "cfg1": dict(family="mlp", dtype="f32", batch=64,
                 dims=[784, 256, 256, 256, 10], depths=[2]),
    # 8 Linear layers of width 1024, 100 classes.
    "cfg2": dict(family="mlp", dtype="bf16", batch=256,
                 dims=[1024] * 8 + [100], depths=[1, 2, 3, 4, 5, 6, 7, 8]),
    # ResNet-18-style, CIFAR-size input; units = stem | 8 basic blocks | head.
    "cfg3": dict(family="resnet_basic", dtype="bf16", batch=128,
                 image=[32, 32, 3], stem=dict(kernel=3, stride=1, pad=1, pool=False, width=64),
                 stage_blocks=[2, 2, 2, 2], stage_widths=[64, 128, 256, 512],
                 classes=10, depths=[3, 5, 7, 9]),
    # ResNet-50-style; units = stem | 16 bottlenecks | head.
    "cfg4": dict(family="resnet_bottleneck", dtype="bf16", batch=64,
                 image=[224, 224, 3], stem=dict(kernel=7, stride=2, pad=3, pool=True, width=64),
                 stage_blocks=[3, 4, 6, 3], stage_widths=[256, 512, 1024, 2048],
                 classes=1000, depths=[4, 10, 14, 17]),
    # BERT-base-shaped pre-LN encoder; units = embedding | 12 layers | head.
    "cfg5": dict(family="encoder", dtype="bf16", batch=32, seq=128, layers=12,
                 hidden=768, heads=12, ffn=3072, vocab=30522, loss_rows=614,
                 depths=[4, 7, 13]),
    # ResNet-101-style stack on CIFAR-size images at batch 64 (the model and batch of Table 1); units = stem | 33
    # bottlenecks | head.  Depths are the table's percentages of the 35 units, rounded up.
    "resnet101_cifar": dict(family="resnet_bottleneck", dtype="bf16", batch=64,
                            image=[32, 32, 3], stem=dict(kernel=3, stride=1, pad=1, pool=False, width=64),
                            stage_blocks=[3, 4, 23, 3], stage_widths=[256, 512, 1024, 2048],
                            classes=10, depths=[2, 4, 7, 11, 14, 18, 21, 25, 28, 32, 35],
                            percents=[5, 10, 20, 30, 40, 50, 60, 70, 80, 90, 100]),
    # Small relatives used by the CPU tests and the small parity cases.
    "tiny_mlp_f32": dict(family="mlp", dtype="f32", batch=5,
                         dims=[12, 8, 8, 4], depths=[0, 1, 2, 3]),
    "ragged_mlp_f32": dict(family="mlp", dtype="f32", batch=37,
                           dims=[100, 72, 136, 52, 7], depths=[0, 1, 2, 3, 4]),
    "ragged_mlp_bf16": dict(family="mlp", dtype="bf16", batch=83,
                            dims=[136, 200, 72, 264, 13], depths=[0, 1, 2, 3, 4]),
    # a perceptron with the matrix shapes of a Transformer layer at 4096 rows: the products go through the large
    # tiles (256 x 192, 128 x 128 alone on a CU, 64 x 64 for the weight gradients) and are checked element by element
    "wide_mlp_bf16": dict(family="mlp", dtype="bf16", batch=4096, dims=[768, 3072, 2304, 768, 24], depths=[2, 4]),
    # 8192 x 4096 results over k = 512: 512 tiles of 256 x 256, several rounds over the CUs, forward and input gradient
    "big_tile_mlp_bf16": dict(family="mlp", dtype="bf16", batch=8192, dims=[512, 4096, 512, 16], depths=[2, 3]),
    # several thousand classes: the loss kernel that keeps a whole row of logits in the registers of one workgroup
    "many_class_mlp_bf16": dict(family="mlp", dtype="bf16", batch=37, dims=[72, 40, 4999], depths=[0, 1, 2]),
    "many_class_mlp_f32": dict(family="mlp", dtype="f32", batch=21, dims=[36, 2050], depths=[0, 1]),
    "tiny_encoder": dict(family="encoder", dtype="bf16", batch=2, seq=4, layers=2, hidden=8, heads=2, ffn=16,
                         vocab=11, loss_rows=3, depths=[0, 1, 2, 3, 4]),
    "small_encoder_bf16": dict(family="encoder", dtype="bf16", batch=3, seq=40, layers=2, hidden=64, heads=4,
                               ffn=136, vocab=203, loss_rows=17, depths=[0, 1, 2, 3, 4]),
    # heads of 64 features and sequences of at most 128 positions take the fused attention kernel
    "fused_attention_encoder_bf16": dict(family="encoder", dtype="bf16", batch=2, seq=128, layers=2, hidden=128, heads=2,
                                         ffn=256, vocab=97, loss_rows=31, depths=[0, 1, 2, 3, 4]),
    "fused_attention_short_bf16": dict(family="encoder", dtype="bf16", batch=3, seq=40, layers=1, hidden=64, heads=1,
                                       ffn=128, vocab=53, loss_rows=11, depths=[0, 1, 2, 3]),
    # widths of 512 and 1024: the LayerNorm backward variants with one and two 16-byte chunks per lane
    "wide_encoder_512_bf16": dict(family="encoder", dtype="bf16", batch=2, seq=24, layers=1, hidden=512, heads=8,
                                  ffn=192, vocab=61, loss_rows=13, depths=[0, 1, 2, 3]),
    "wide_encoder_1024_bf16": dict(family="encoder", dtype="bf16", batch=1, seq=40, layers=1, hidden=1024, heads=16,
                                   ffn=128, vocab=37, loss_rows=9, depths=[0, 1, 2, 3]),
    # a vocabulary large enough for the head's input gradient to be cut into k-slices and for the long-row loss kernel
    "big_vocab_encoder_bf16": dict(family="encoder", dtype="bf16", batch=2, seq=16, layers=1, hidden=64, heads=1,
                                   ffn=72, vocab=2311, loss_rows=9, depths=[0, 1, 2, 3]),
    "tiny_resnet_basic": dict(family="resnet_basic", dtype="bf16", batch=2, image=[6, 6, 3],
                              stem=dict(kernel=3, stride=1, pad=1, pool=False, width=4),
                              stage_blocks=[1, 1], stage_widths=[4, 6], classes=3, depths=[0, 1, 2, 3, 4]),
    "tiny_resnet_bottleneck": dict(family="resnet_bottleneck", dtype="bf16", batch=2, image=[9, 9, 3],
                                   stem=dict(kernel=7, stride=2, pad=3, pool=True, width=4),
                                   stage_blocks=[2, 1], stage_widths=[8, 12], classes=3, depths=[0, 1, 2, 3, 4, 5]),
    "small_resnet_basic_bf16": dict(family="resnet_basic", dtype="bf16", batch=3, image=[12, 12, 3],
                                    stem=dict(kernel=3, stride=1, pad=1, pool=False, width=16),
                                    stage_blocks=[1, 2], stage_widths=[16, 32], classes=7, depths=[0, 1, 2, 3, 4, 5]),
    "small_resnet_bottleneck_bf16": dict(family="resnet_bottleneck", dtype="bf16", batch=2, image=[20, 20, 3],
                                         stem=dict(kernel=7, stride=2, pad=3, pool=True, width=16),
                                         stage_blocks=[2, 1], stage_widths=[32, 64], classes=11, depths=[0, 1, 2, 3, 4, 5]),
    # one bottleneck stage 64 -> 256 on 56x56 images and a stride-2 block 128 -> 512 behind it, batch 8: products of
    # 25088 x 64..256 and 6272 x 128..512 rows, which take the 128-row and 256-row gathered tiles, the one-tap path
    # at 64 and 128 channels, a stride-2 input gradient and weight gradients cut into 64 and more k-slices; small
    # enough for the oracle to check every entry
    "mid_resnet_bottleneck_bf16": dict(family="resnet_bottleneck", dtype="bf16", batch=8, image=[56, 56, 3],
                                       stem=dict(kernel=3, stride=1, pad=1, pool=False, width=64),
                                       stage_blocks=[2, 1], stage_widths=[256, 512], classes=10, depths=[1, 2, 3, 4, 5]),
    # the 35-unit stack of resnet101_cifar at toy widths
    "small_resnet101_bf16": dict(family="resnet_bottleneck", dtype="bf16", batch=2, image=[8, 8, 3],
                                 stem=dict(kernel=3, stride=1, pad=1, pool=False, width=16),
                                 stage_blocks=[3, 4, 23, 3], stage_widths=[32, 64, 128, 256], classes=5,
                                 depths=[0, 2, 7, 18, 35]),
    "one_layer_bf16": dict(family="mlp", dtype="bf16", batch=16,
                           dims=[64, 10], depths=[0, 1]),
}


def get_config(name: str) -> dict:
    cfg = copy.deepcopy(CONFIGS[name])
    cfg["name"] = name
    return cfg


def unit_count(cfg: dict) -> int:
    fam = cfg["family"]
    if fam == "mlp":
        return len(cfg["dims"]) - 1
    if fam in ("resnet_basic", "resnet_bottleneck"):
        return 1 + sum(cfg["stage_blocks"]) + 1
    if fam == "encoder":
        return 1 + cfg["layers"] + 1
    raise ValueError(fam)


def depth_sweep(cfg: dict) -> list:
    return list(cfg["depths"])


def resnet_layout(cfg: dict) -> dict:
    """Shapes of a residual CNN: the stem, the list of blocks and the classifier input width.

    Stride 2 sits on the first block of every stage but the first (in a bottleneck, on its 3x3 convolution);
    a block whose input and output shapes differ gets a 1x1 projection shortcut with the same stride;
    a bottleneck's inner width is a quarter of its output width.
    """
    st = cfg["stem"]
    h = (cfg["image"][0] + 2 * st["pad"] - st["kernel"]) // st["stride"] + 1
    w = (cfg["image"][1] + 2 * st["pad"] - st["kernel"]) // st["stride"] + 1
    stem = dict(cin=cfg["image"][2], cout=st["width"], kernel=st["kernel"], stride=st["stride"], pad=st["pad"],
                pool=bool(st["pool"]), conv_hw=(h, w))
    if st["pool"]:
        h, w = (h + 2 - 3) // 2 + 1, (w + 2 - 3) // 2 + 1
    blocks, cin = [], st["width"]
    bottleneck = cfg["family"] == "resnet_bottleneck"
    for stage, (count, width) in enumerate(zip(cfg["stage_blocks"], cfg["stage_widths"])):
        for j in range(count):
            stride = 2 if (stage > 0 and j == 0) else 1
            blk = dict(index=len(blocks), cin=cin, cout=width, mid=width // 4 if bottleneck else width, stride=stride,
                       proj=(stride != 1 or cin != width), in_hw=(h, w))
            h, w = (h - 1) // stride + 1, (w - 1) // stride + 1
            blk["out_hw"] = (h, w)
            blocks.append(blk)
            cin = width
    return dict(stem=stem, blocks=blocks, bottleneck=bottleneck, features=cin, final_hw=(h, w))
