"""Seeded synthetic workloads: shapes, inputs and initial parameters.

Serves both the HIP path (through the binding) and the CPU oracle (through the
tests and the benchmark).  Holds none of the method's arithmetic: only shape
tables, random draws and the bf16 value rounding of generated inputs.

The images stand in for the paper's datasets (Section 4.1: CIFAR-10 and SVHN are
32x32x3, STL-10 is 96x96x3, all with 10 classes): shape and class count are kept,
pixels are N(0,1), labels uniform.  No item of those datasets is used.
"""
from __future__ import annotations

import numpy as np

# arch / input_kind / optimizer / precision codes are the ones of include/ppll.h
VIT, RESNET = 0, 1
IMAGE, ACTIVATION = 0, 1
SGD, ADAMW = 0, 1
FP32, BF16 = 0, 1

_VIT_STAGE = dict(arch=VIT, precision=BF16, input_kind=IMAGE, batch=128, num_classes=10,
                  img_h=32, img_w=32, img_c=3, patch=4, tokens=65, dim=384, heads=6,
                  mlp_dim=1536, depth=3, aux_depth=1, optimizer=ADAMW, weight_decay=0.01,
                  beta1=0.9, beta2=0.999, adam_eps=1e-8, ln_eps=1e-6, lr=1e-3)

WORKLOADS = {
    # the small fp32 case the CPU oracle finishes in seconds: tiny ViT block, one plain SGD step
    "vit_tiny_fp32": dict(arch=VIT, precision=FP32, input_kind=IMAGE, batch=8, num_classes=10,
                          img_h=32, img_w=32, img_c=3, patch=4, tokens=65, dim=64, heads=4,
                          mlp_dim=128, depth=2, aux_depth=0, optimizer=SGD, momentum=0.0,
                          nesterov=0, weight_decay=0.0, ln_eps=1e-6, lr=0.01),
    # the headline workload: one of 4 blocks of a 12-layer ViT
    "vit_stage_bf16": dict(_VIT_STAGE),
    # blocks 2..4 of the 4-block pipeline: same stage fed with token activations
    "vit_stage_act_bf16": dict(_VIT_STAGE, input_kind=ACTIVATION),
    # ResNet stage at batch 128 (Section 4.1 optimizer: Nesterov 0.9, L2 1e-4, lr 0.01)
    "resnet_stage_bf16": dict(arch=RESNET, precision=BF16, input_kind=ACTIVATION, batch=128,
                              num_classes=10, channels=32, height=16, width=16,
                              n_basic_blocks=5, aux_channels=64, optimizer=SGD, momentum=0.9,
                              nesterov=1, weight_decay=1e-4, bn_eps=1e-5, bn_momentum=0.1,
                              lr=0.01),
    # the paper's own ViT shape (Section 4.1: ViT-base-patch16 on 32x32 images, batch 128: 4 patches + class
    # token = 5 tokens of width 768, 12 heads, MLP 3072), one stage of 3 layers with a 1-layer auxiliary
    # network, trained with the paper's optimizer (SGD, Nesterov 0.9, L2 1e-4, lr 0.01)
    "vit_base_paper_bf16": dict(arch=VIT, precision=BF16, input_kind=IMAGE, batch=128, num_classes=10,
                                img_h=32, img_w=32, img_c=3, patch=16, tokens=5, dim=768, heads=12,
                                mlp_dim=3072, depth=3, aux_depth=1, optimizer=SGD, momentum=0.9, nesterov=1,
                                weight_decay=1e-4, ln_eps=1e-6, lr=0.01),
    # the same model at the input resolution Section 4.3 states for the speed measurements (224 x 224: 196 patches + class
    # token = 197 tokens), one stage of 3 layers with a 1-layer auxiliary network, batch 128
    "vit_base_224_bf16": dict(arch=VIT, precision=BF16, input_kind=IMAGE, batch=128, num_classes=10,
                              img_h=224, img_w=224, img_c=3, patch=16, tokens=197, dim=768, heads=12,
                              mlp_dim=3072, depth=3, aux_depth=1, optimizer=SGD, momentum=0.9, nesterov=1,
                              weight_decay=1e-4, ln_eps=1e-6, lr=0.01),
    # second stage of ResNet-32 at the paper's CIFAR batch (Section 4.1: batch 1024; Section 4.3 names its
    # 1024 x 32 x 16 x 16 activations): the basic block that halves the 32 x 32 x 16 input and doubles its
    # channels, then four shape-keeping blocks
    "resnet32_stage2_bf16": dict(arch=RESNET, precision=BF16, input_kind=ACTIVATION, batch=1024,
                                 num_classes=10, channels=32, height=16, width=16, transition_block=1,
                                 n_basic_blocks=5, aux_channels=64, optimizer=SGD, momentum=0.9,
                                 nesterov=1, weight_decay=1e-4, bn_eps=1e-5, bn_momentum=0.1, lr=0.01),
    # first stage of the same network: the stem on the image and the five 16-channel blocks on 32 x 32 maps
    "resnet32_stage1_bf16": dict(arch=RESNET, precision=BF16, input_kind=IMAGE, img_h=32, img_w=32, img_c=3,
                                 batch=1024, num_classes=10, channels=16, height=32, width=32, transition_block=0,
                                 n_basic_blocks=5, aux_channels=64, optimizer=SGD, momentum=0.9,
                                 nesterov=1, weight_decay=1e-4, bn_eps=1e-5, bn_momentum=0.1, lr=0.01),
    # third stage: the block that halves the 16 x 16 x 32 input to 8 x 8 x 64, then four 64-channel blocks
    "resnet32_stage3_bf16": dict(arch=RESNET, precision=BF16, input_kind=ACTIVATION, batch=1024,
                                 num_classes=10, channels=64, height=8, width=8, transition_block=1,
                                 n_basic_blocks=5, aux_channels=64, optimizer=SGD, momentum=0.9,
                                 nesterov=1, weight_decay=1e-4, bn_eps=1e-5, bn_momentum=0.1, lr=0.01),
    # STL-10-shaped ViT stage (96 x 96 images)
    "vit_large_image_bf16": dict(_VIT_STAGE, batch=64, img_h=96, img_w=96, patch=8, tokens=145),
}


def workload(name: str, **overrides) -> dict:
    wl = dict(WORKLOADS[name])
    wl.update(overrides)
    return wl


def resnet32_modules(k: int, **overrides) -> list:
    """ResNet-32 for 32 x 32 images (Section 4.1) cut into k local modules: the stem (conv3x3 3 -> 16, BN,
    ReLU) and 15 basic blocks, 5 each at 16 channels on 32 x 32, 32 on 16 x 16 and 64 on 8 x 8 maps, the
    first block of the second and third group halving the map and doubling the channels.  The basic
    blocks are dealt to the modules as evenly as possible, earlier modules taking the extra ones; the stem
    belongs to module 0.  A module here holds at least one basic block, so k <= 15.  Every module carries
    the conv-BN-ReLU-pool-Linear auxiliary head of the ResNet stage workload; the network's own classifier
    (global average, Linear) is not part of any module."""
    if not 1 <= k <= 15:
        raise ValueError("k must be in 1..15")
    base = dict(WORKLOADS["resnet32_stage2_bf16"], transition_block=0)
    sizes = [15 // k + (1 if i < 15 % k else 0) for i in range(k)]
    out, first = [], 0
    for i, n in enumerate(sizes):
        last = first + n - 1
        group = last // 5                      # group of the module's output
        wl = dict(base, n_basic_blocks=n, channels=16 << group, height=32 >> group, width=32 >> group)
        for t in (5, 10):                      # the downsampling blocks of the network
            if first <= t <= last:
                wl["transition_block"] = t - first + 1
        if (first <= 5 <= last) and (first <= 10 <= last):
            raise ValueError("a module may hold one downsampling block: use k >= 2")
        if i == 0:
            wl.update(input_kind=IMAGE, img_h=32, img_w=32, img_c=3)
        wl.update(overrides)
        out.append(wl)
        first += n
    return out


def cosine_lr(step: int, total_steps: int, lr0: float = 0.01) -> float:
    """Learning rate of call `step` (0-based) under cosine annealing from lr0 to 0 over total_steps calls
    (Section 4.1: initial rate 0.01, cosine schedule).  The library takes the rate per call; the schedule
    lives on the host."""
    import math
    return 0.5 * lr0 * (1.0 + math.cos(math.pi * step / total_steps))


def aux_depth_schedule(d_max: int, n_blocks: int = 12, n: int = 3) -> list:
    """Depth of the auxiliary network of local block l (0-based) of a ViT cut into n_blocks local
    blocks: N_l = d' - floor(l / n) with n = 3 (Section 4.2, the auxiliary-depth heuristic), d' the
    maximum depth (2, 3 or 4 in the paper).  The formula goes negative for d' < 4 and l >= 3 d';
    a block cannot have fewer than zero auxiliary layers, so it is floored at 0 (head only)."""
    return [max(0, d_max - l // n) for l in range(n_blocks)]


def lpp_workloads(d_max: int, n_blocks: int = 12, **overrides) -> list:
    """The finest partition of Section 4.2 ("largest pipeline parallelism"): every encoder layer of
    the ViT is a local block of its own, with the auxiliary depth of aux_depth_schedule().  Block 0
    takes images, the others the token activations of their predecessor."""
    out = []
    for l, a in enumerate(aux_depth_schedule(d_max, n_blocks)):
        wl = workload("vit_stage_bf16" if l == 0 else "vit_stage_act_bf16", depth=1, aux_depth=a)
        wl.update(overrides)
        if l > 0:
            wl["input_kind"] = ACTIVATION
        out.append(wl)
    return out


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16-representable value (ties to even),
    returned as fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def input_shape(wl: dict) -> tuple:
    if wl["arch"] == VIT:
        if wl["input_kind"] == IMAGE:
            return (wl["batch"], wl["img_h"], wl["img_w"], wl["img_c"])
        return (wl["batch"], wl["tokens"], wl["dim"])
    if wl["input_kind"] == IMAGE:     # the stem reads the image
        return (wl["batch"], wl["img_h"], wl["img_w"], wl["img_c"])
    if wl.get("transition_block", 0) > 0:   # a basic block of the stage halves the map and doubles the channels
        return (wl["batch"], 2 * wl["height"], 2 * wl["width"], wl["channels"] // 2)
    return (wl["batch"], wl["height"], wl["width"], wl["channels"])


def output_shape(wl: dict) -> tuple:
    if wl["arch"] == VIT:
        return (wl["batch"], wl["tokens"], wl["dim"])
    return (wl["batch"], wl["height"], wl["width"], wl["channels"])


def make_batch(wl: dict, seed: int = 0, index: int = 0):
    """(x, labels): x ~ N(0,1) fp32 (bf16-representable on the bf16 path),
    labels uniform int32.  `index` selects the batch within the seeded stream."""
    rng = np.random.default_rng([seed, index])
    x = rng.standard_normal(input_shape(wl), dtype=np.float32)
    if wl["precision"] == BF16:
        x = round_to_bf16(x)
    y = rng.integers(0, wl["num_classes"], size=wl["batch"], dtype=np.int32)
    return x, y


def make_params(spec, seed: int = 0, jitter: bool = False) -> np.ndarray:
    """Flat fp32 parameter blob for an ordered (name, shape) table.

    Linear, patch-embed, cls and pos ~ N(0, 0.02^2); 3x3 convolutions
    ~ N(0, 2/(9 Cin)); biases 0 and norm scales 1 / shifts 0 unless `jitter`,
    which perturbs them (bias ~ N(0, 0.02^2), scale ~ 1 + N(0, 0.1^2), shift
    ~ N(0, 0.1^2)) so that parity runs exercise every tensor."""
    rng = np.random.default_rng([seed, 12345])
    parts = []
    for name, shape in spec:
        n = int(np.prod(shape))
        leaf = name.split(".")[-1]
        is_norm = ".ln" in name or ".bn" in name
        if len(shape) == 4:
            v = rng.standard_normal(n) * np.sqrt(2.0 / (9.0 * shape[2]))
        elif is_norm and leaf == "g":
            v = 1.0 + (rng.standard_normal(n) * 0.1 if jitter else np.zeros(n))
        elif is_norm and leaf == "b":
            v = rng.standard_normal(n) * 0.1 if jitter else np.zeros(n)
        elif leaf == "b":
            v = rng.standard_normal(n) * 0.02 if jitter else np.zeros(n)
        else:
            v = rng.standard_normal(n) * 0.02
        parts.append(v.astype(np.float32))
    return np.concatenate(parts)
