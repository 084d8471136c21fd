"""Partition descriptions and seeded synthetic inputs.

This module describes WHAT is run (which residual blocks a partition holds,
tensor shapes, the canonical flat parameter order) and draws the seeded random
tensors that are handed, unchanged, both to the CPU oracle and to the HIP
library.  It contains none of the method's arithmetic and imports neither of
them.

The workloads are the model partitions of HyPar-Flow-style model-parallel
training (paper Section "Designing Distributed Model Representation" and the
ResNet experiments of "Model-Parallelism on a Single Node"): a deep
pre-activation ResNet is cut into contiguous partitions at residual-block
boundaries, each batch is cut into micro-batches ("pipeline stages", Section
"Exploiting Pipeline Stages within Each Minibatch"), and one partition's share
of the work is run with seeded tensors standing in for what the neighbouring
partitions would send.  Images have the 32x32x3 and 224x224x3 shapes of the
CIFAR-10 / ImageNet-style inputs the paper's models take; the values are
N(0,1) noise, not dataset items.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np

BASIC = 0
BOTTLENECK = 1
POSTACT = 2      # ResNet-v1 basic block: conv3x3(stride) - bn - relu - conv3x3 - bn, + shortcut, relu
CONV_RELU = 3    # plain (VGG) unit: conv3x3 + bias + relu, followed by a 2x2 max-pool iff stride == 2
DENSE = 4        # flatten - fully connected + bias, relu iff c_mid != 0
BN_RELU = 5      # BatchNorm + relu on its own (the stem of ResNet-v1 is conv - bn - relu)
BIAS_RELU = 6    # bias + relu on its own (VGG's first convolution is the stem, its bias and relu this unit)

SEED_BASE = 191105146


@dataclass(frozen=True)
class Block:
    """One pre-activation residual block.

    kind BASIC:      bn-relu-conv3x3(stride) - bn-relu-conv3x3, c_mid == c_out
    kind BOTTLENECK: bn-relu-conv1x1(stride) - bn-relu-conv3x3 - bn-relu-conv1x1
    A 1x1 projection shortcut (same stride) exists iff stride != 1 or c_in != c_out.

    The units of the paper's other two models (Section "Model-Parallelism on a Single Node": ResNet-110-v1,
    VGG-16), which are not pre-activation residual blocks:
    kind POSTACT:    y = relu(bn2(conv3x3(relu(bn1(conv3x3_stride(x))))) + shortcut), c_mid == c_out; shortcut = x, or
                     a 1x1 convolution (same stride, no BatchNorm) of x iff stride != 1 or c_in != c_out
    kind CONV_RELU:  relu(conv3x3(x) + bias) with padding 1, then a 2x2 max-pool of stride 2 iff stride == 2
    kind DENSE:      flatten(x) * W + bias, relu iff c_mid != 0; the output is 1 x 1 x c_out
    kind BN_RELU:    relu(bn(x)), c_in == c_out
    kind BIAS_RELU:  relu(x + bias), c_in == c_out
    """
    kind: int
    c_in: int
    c_mid: int
    c_out: int
    stride: int

    @property
    def has_proj(self) -> bool:
        return self.kind in (BASIC, BOTTLENECK, POSTACT) and (self.stride != 1 or self.c_in != self.c_out)

    @property
    def residual(self) -> bool:
        """A pre-activation residual block (the only kinds that can be cut at layer granularity)."""
        return self.kind in (BASIC, BOTTLENECK)


@dataclass(frozen=True)
class PartitionSpec:
    name: str
    in_h: int
    in_w: int
    in_c: int
    blocks: Tuple[Block, ...]
    has_stem: bool = False
    stem_c_out: int = 0
    has_head: bool = False
    num_classes: int = 0
    head_bn: bool = True           # the head starts with BatchNorm + relu (pre-activation models); False: pool - FC only
    microbatch: int = 1
    num_microbatches: int = 1
    loss_divisor: int = 0          # full batch B; 0 -> microbatch * num_microbatches
    bn_eps: float = 1e-5
    bn_mode: int = 0               # 0: statistics of the micro-batch, 1: frozen mean 0 / var 1
    seed: int = SEED_BASE
    # Cuts at layer granularity: the partition holds convolutions [first_from, n) of its first block and
    # [0, last_to) of its last block (0 = the whole block).  A BatchNorm+ReLU belongs to the convolution it
    # feeds, the projection to convolution 0, the residual add to the last convolution.  With first_from > 0,
    # (in_h, in_w, in_c) is the output of convolution first_from-1 (block-output size, c_mid channels).
    first_from: int = 0
    last_to: int = 0

    @property
    def batch(self) -> int:
        return self.microbatch * self.num_microbatches

    @property
    def divisor(self) -> int:
        return self.loss_divisor if self.loss_divisor > 0 else self.batch

    def conv_range(self, i: int) -> Tuple[int, int]:
        """[j0, j1): the convolutions of block i that this partition holds."""
        if not self.blocks[i].residual:
            return 0, {POSTACT: 2, CONV_RELU: 1, DENSE: 1, BN_RELU: 0, BIAS_RELU: 0}[self.blocks[i].kind]
        n = 2 if self.blocks[i].kind == BASIC else 3
        j0 = self.first_from if i == 0 else 0
        j1 = self.last_to if (i == len(self.blocks) - 1 and self.last_to > 0) else n
        return j0, j1

    def out_shape(self) -> Tuple[int, int, int]:
        """(H, W, C) of the tensor leaving the partition's last layer (before the head)."""
        h, w = self.in_h, self.in_w
        c = self.stem_c_out if self.has_stem else self.in_c
        for i, b in enumerate(self.blocks):
            if not b.residual:
                assert b.c_in == c, (self.name, b, c)
                if b.kind == DENSE:
                    h, w = 1, 1
                else:
                    h, w = h // b.stride, w // b.stride
                c = b.c_out
                continue
            j0, j1 = self.conv_range(i)
            n = 2 if b.kind == BASIC else 3
            if j0 == 0:
                assert b.c_in == c, (self.name, b, c)
                h, w = h // b.stride, w // b.stride
            else:
                assert b.c_mid == c, (self.name, b, c)
            c = b.c_out if j1 == n else b.c_mid
        return h, w, c

    @property
    def has_skip_in(self) -> bool:
        """The first block starts after its convolution 0 and ends here: its shortcut value comes from the
        partition that holds its start."""
        return self.first_from > 0 and self.conv_range(0)[1] == (2 if self.blocks[0].kind == BASIC else 3)

    @property
    def has_skip_out(self) -> bool:
        """The last block starts here and ends in a later partition: its shortcut value leaves directly."""
        return self.last_to > 0 and self.conv_range(len(self.blocks) - 1)[0] == 0

    def skip_in_shape(self) -> Tuple[int, int, int]:
        return self.in_h, self.in_w, self.blocks[0].c_out

    def skip_out_shape(self) -> Tuple[int, int, int]:
        h, w, _ = self.out_shape()
        return h, w, self.blocks[-1].c_out


# ----------------------------------------------------------------------------
# model families
# ----------------------------------------------------------------------------
def basic_resnet_blocks(n_per_stage: int, widths=(16, 32, 64)) -> List[Block]:
    blocks, c = [], widths[0]
    for s, wdt in enumerate(widths):
        for i in range(n_per_stage):
            stride = 2 if (s > 0 and i == 0) else 1
            blocks.append(Block(BASIC, c, wdt, wdt, stride))
            c = wdt
    return blocks


def bottleneck_resnet_blocks(n_per_stage, mids, outs, c0, first_stride=1) -> List[Block]:
    blocks, c = [], c0
    if isinstance(n_per_stage, int):
        n_per_stage = [n_per_stage] * len(mids)
    for s, (n, mid, out) in enumerate(zip(n_per_stage, mids, outs)):
        for i in range(n):
            stride = 1
            if i == 0:
                stride = first_stride if s == 0 else 2
            blocks.append(Block(BOTTLENECK, c, mid, out, stride))
            c = out
    return blocks


def split_range(n_blocks: int, n_parts: int, p: int) -> Tuple[int, int]:
    """Even split of blocks over partitions: partition p holds [lo, hi)."""
    return (p * n_blocks) // n_parts, ((p + 1) * n_blocks) // n_parts


def partition_of(name, all_blocks, n_parts, p, in_hw, in_c0, stem_c, classes,
                 microbatch, num_microbatches, seed, in_c_img=3) -> PartitionSpec:
    """Partition p (0-based) of n_parts of a stem + blocks + head model."""
    lo, hi = split_range(len(all_blocks), n_parts, p)
    h = w = in_hw
    for b in all_blocks[:lo]:
        h, w = h // b.stride, w // b.stride
    first, last = (p == 0), (p == n_parts - 1)
    return PartitionSpec(
        name=name, in_h=h, in_w=w,
        in_c=in_c_img if first else all_blocks[lo].c_in,
        blocks=tuple(all_blocks[lo:hi]),
        has_stem=first, stem_c_out=stem_c if first else 0,
        has_head=last, num_classes=classes if last else 0,
        microbatch=microbatch, num_microbatches=num_microbatches, seed=seed)


def resnet20(microbatch=4, num_microbatches=2, seed=SEED_BASE + 1) -> PartitionSpec:
    return partition_of("resnet20-whole", basic_resnet_blocks(3), 1, 0, 32, 16, 16, 10,
                        microbatch, num_microbatches, seed)


def resnet110_partition(p=2, n_parts=4, microbatch=16, num_microbatches=8,
                        seed=SEED_BASE + 2) -> PartitionSpec:
    return partition_of(f"resnet110-part{p}of{n_parts}", basic_resnet_blocks(18), n_parts, p,
                        32, 16, 16, 10, microbatch, num_microbatches, seed)


def resnet1001_blocks() -> List[Block]:
    return bottleneck_resnet_blocks(111, (16, 32, 64), (64, 128, 256), 16)


def resnet1001_partition(p=7, n_parts=16, microbatch=32, num_microbatches=8,
                         seed=SEED_BASE + 3) -> PartitionSpec:
    return partition_of(f"resnet1001-part{p}of{n_parts}", resnet1001_blocks(), n_parts, p,
                        32, 16, 16, 10, microbatch, num_microbatches, seed)


def resnet1001_whole(microbatch=8, num_microbatches=8, seed=SEED_BASE + 4) -> PartitionSpec:
    return partition_of("resnet1001-whole", resnet1001_blocks(), 1, 0, 32, 16, 16, 10,
                        microbatch, num_microbatches, seed)


def resnet152_stage3(n_blocks=36, microbatch=16, num_microbatches=4,
                     seed=SEED_BASE + 5) -> PartitionSpec:
    blocks = [Block(BOTTLENECK, 512, 256, 1024, 2)]
    blocks += [Block(BOTTLENECK, 1024, 256, 1024, 1)] * (n_blocks - 1)
    return PartitionSpec(name=f"resnet152v2-stage3-{n_blocks}blocks", in_h=28, in_w=28, in_c=512,
                         blocks=tuple(blocks), microbatch=microbatch,
                         num_microbatches=num_microbatches, seed=seed)


def resnet1001_wide_blocks() -> List[Block]:
    """The wider ResNet-1001-v2 with about 30 M parameters (the size the paper quotes for its ResNet-1001):
    333 bottleneck blocks whose inner width is the width of the stage's input, i.e. 16 -> 64 in stage 1,
    64 -> 128 in stage 2 and 128 -> 256 in stage 3 (inner widths 16 / 64 / 128)."""
    blocks, c = [], 16
    for s, (mid, out) in enumerate(((16, 64), (64, 128), (128, 256))):
        for i in range(111):
            blocks.append(Block(BOTTLENECK, c, mid, out, 2 if (s > 0 and i == 0) else 1))
            c = out
    return blocks


def resnet1001_wide_partition(p=7, n_parts=16, microbatch=32, num_microbatches=8,
                              seed=SEED_BASE + 6) -> PartitionSpec:
    """Partition 7 of 16 of the 30 M-parameter variant: 21 identity blocks 128-64-64-128 at 16x16."""
    return partition_of(f"resnet1001wide-part{p}of{n_parts}", resnet1001_wide_blocks(), n_parts, p,
                        32, 16, 16, 10, microbatch, num_microbatches, seed)


def resnet_v1_blocks(n_per_stage: int, widths=(16, 32, 64)) -> List[Block]:
    """ResNet-v1 for 32x32 images (6n+2 layers: n = 18 gives the ResNet-110 the paper trains): after the stem
    (conv3x3 - BatchNorm - relu) three stages of n post-activation basic blocks; the first block of stages 2 and 3
    halves the resolution and doubles the width, its shortcut is a 1x1 convolution of stride 2."""
    blocks, c = [Block(BN_RELU, widths[0], widths[0], widths[0], 1)], widths[0]
    for s, wdt in enumerate(widths):
        for i in range(n_per_stage):
            blocks.append(Block(POSTACT, c, wdt, wdt, 2 if (s > 0 and i == 0) else 1))
            c = wdt
    return blocks


def resnet110_v1(n_parts=1, p=0, microbatch=16, num_microbatches=8, seed=SEED_BASE + 7, n_per_stage=18) -> PartitionSpec:
    """Partition p of n_parts of ResNet-110-v1 (paper Section "Model-Parallelism on a Single Node"): units = the stem's
    BatchNorm-relu and 54 post-activation blocks; the head is global average pool - FC (no BatchNorm)."""
    spec = partition_of(f"resnet{6 * n_per_stage + 2}v1-part{p}of{n_parts}", resnet_v1_blocks(n_per_stage), n_parts, p,
                        32, 16, 16, 10, microbatch, num_microbatches, seed)
    return replace(spec, head_bn=False)


def vgg16_blocks(in_hw=32, widths=(64, 128, 256, 512, 512), convs=(2, 2, 3, 3, 3), dense=(4096, 4096), in_c=3) -> List[Block]:
    """VGG-16 (configuration D of the VGG paper: 13 convolutions 3x3 in five groups, each group followed by a 2x2
    max-pool, then fully connected layers), the paper's third model; on 32x32 images the last pool leaves 1 x 1 x 512.
    The last fully connected layer (-> classes) with the softmax is the partition's head."""
    blocks, c = [Block(BIAS_RELU, widths[0], widths[0], widths[0], 1)], widths[0]   # after the stem convolution
    for g, (wdt, n) in enumerate(zip(widths, convs)):
        for i in range(1 if g == 0 else 0, n):
            blocks.append(Block(CONV_RELU, c, wdt, wdt, 2 if i == n - 1 else 1))
            c = wdt
    for d in dense:
        blocks.append(Block(DENSE, c, 1, d, 1))
        c = d
    return blocks


def vgg16(n_parts=1, p=0, microbatch=16, num_microbatches=8, seed=SEED_BASE + 8, **kw) -> PartitionSpec:
    """Partition p of n_parts of VGG-16 on 32x32x3 images, cut at unit boundaries (the paper runs it in up to 8
    partitions).  The first convolution (3 -> 64 channels, on the fp32 image) is the partition's stem; its bias and
    relu are the first unit."""
    blocks = vgg16_blocks(**kw)
    lo, hi = split_range(len(blocks), n_parts, p)
    h = w = kw.get("in_hw", 32)
    c = blocks[0].c_in
    for b in blocks[:lo]:
        h, w = (1, 1) if b.kind == DENSE else (h // b.stride, w // b.stride)
        c = b.c_out
    first, last = p == 0, p == n_parts - 1
    return PartitionSpec(name=f"vgg16-part{p}of{n_parts}", in_h=h, in_w=w, in_c=kw.get("in_c", 3) if first else c,
                         blocks=tuple(blocks[lo:hi]), has_stem=first, stem_c_out=blocks[0].c_in if first else 0,
                         has_head=last, num_classes=10 if last else 0, head_bn=False, microbatch=microbatch,
                         num_microbatches=num_microbatches, seed=seed)


def config(index: int) -> PartitionSpec:
    """The five benchmark configurations, numbered 1..5; 6: the same cut of the wider ResNet-1001; 7 and 8: the
    paper's two other models whole, ResNet-110-v1 and VGG-16 on 32x32 images (8 micro-batches of 16 images)."""
    return {1: resnet20, 2: resnet110_partition, 3: resnet1001_partition,
            4: resnet1001_whole, 5: resnet152_stage3, 6: resnet1001_wide_partition,
            7: resnet110_v1, 8: vgg16}[index]()


def with_microbatching(spec: PartitionSpec, microbatch: int, num_microbatches: int,
                       **kw) -> PartitionSpec:
    kw.setdefault("loss_divisor", 0)
    return replace(spec, microbatch=microbatch, num_microbatches=num_microbatches, **kw)


# ----------------------------------------------------------------------------
# canonical flat parameter order
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class ParamEntry:
    name: str
    shape: Tuple[int, ...]
    kind: str          # "conv" (HWIO), "gamma", "beta", "fc" ([C][classes]), "bias"
    offset: int

    @property
    def size(self) -> int:
        return int(np.prod(self.shape))


def param_layout(spec: PartitionSpec) -> List[ParamEntry]:
    """Units in model order; stem W; per block bn1.g, bn1.b, W1, bn2.g, bn2.b, W2,
    [bn3.g, bn3.b, W3], [Wproj]; head bn.g, bn.b, Wfc, bfc.  Conv weights are
    [R][S][Cin][Cout]."""
    out: List[ParamEntry] = []
    off = 0

    def add(name, shape, kind):
        nonlocal off
        e = ParamEntry(name, tuple(shape), kind, off)
        out.append(e)
        off += e.size

    if spec.has_stem:
        add("stem.W", (3, 3, spec.in_c, spec.stem_c_out), "conv")
    h, w = spec.in_h, spec.in_w
    for i, b in enumerate(spec.blocks):
        p = f"block{i}."
        if not b.residual:
            if b.kind == POSTACT:
                add(p + "W1", (3, 3, b.c_in, b.c_mid), "conv")
                add(p + "bn1.gamma", (b.c_mid,), "gamma")
                add(p + "bn1.beta", (b.c_mid,), "beta")
                add(p + "W2", (3, 3, b.c_mid, b.c_out), "conv")
                add(p + "bn2.gamma", (b.c_out,), "gamma")
                add(p + "bn2.beta", (b.c_out,), "beta")
                if b.has_proj:
                    add(p + "Wproj", (1, 1, b.c_in, b.c_out), "conv")
                h, w = h // b.stride, w // b.stride
            elif b.kind == CONV_RELU:
                add(p + "W", (3, 3, b.c_in, b.c_out), "conv")
                add(p + "bias", (b.c_out,), "bias")
                h, w = h // b.stride, w // b.stride
            elif b.kind == DENSE:
                add(p + "W", (h * w * b.c_in, b.c_out), "fc")
                add(p + "bias", (b.c_out,), "bias")
                h, w = 1, 1
            elif b.kind == BN_RELU:
                add(p + "bn.gamma", (b.c_in,), "gamma")
                add(p + "bn.beta", (b.c_in,), "beta")
            else:
                add(p + "bias", (b.c_in,), "bias")
            continue
        h, w = h // b.stride, w // b.stride
        j0, j1 = spec.conv_range(i)
        cin = (b.c_in, b.c_mid, b.c_mid)
        cout = (b.c_mid, b.c_out, None) if b.kind == BASIC else (b.c_mid, b.c_mid, b.c_out)
        R = (3, 3, None) if b.kind == BASIC else (1, 3, 1)
        for j in range(j0, j1):        # only the layers held here, in canonical order
            add(p + f"bn{j + 1}.gamma", (cin[j],), "gamma")
            add(p + f"bn{j + 1}.beta", (cin[j],), "beta")
            add(p + f"W{j + 1}", (R[j], R[j], cin[j], cout[j]), "conv")
        if b.has_proj and j0 == 0:
            add(p + "Wproj", (1, 1, b.c_in, b.c_out), "conv")
    if spec.has_head:
        c = spec.out_shape()[2]
        if spec.head_bn:
            add("head.bn.gamma", (c,), "gamma")
            add("head.bn.beta", (c,), "beta")
        add("head.Wfc", (c, spec.num_classes), "fc")
        add("head.bfc", (spec.num_classes,), "bias")
    return out


def n_params(spec: PartitionSpec) -> int:
    lay = param_layout(spec)
    return lay[-1].offset + lay[-1].size if lay else 0


# ----------------------------------------------------------------------------
# seeded tensors
# ----------------------------------------------------------------------------
@dataclass
class StepInputs:
    params: np.ndarray                       # [P] float32, canonical order
    act_in: List[np.ndarray]                 # per micro-batch [b,H,W,C] float32
    labels: Optional[List[np.ndarray]]       # per micro-batch [b] int32 (head only)
    err_in: Optional[List[np.ndarray]]       # per micro-batch [b,H',W',C'] float32 (no head)
    skip_in: Optional[List[np.ndarray]] = None       # shortcut value for a first block cut after its start
    skip_err_in: Optional[List[np.ndarray]] = None   # gradient w.r.t. skip_out of a last block cut before its end


def make_params(spec: PartitionSpec, rng: np.random.Generator,
                randomize_affine: bool = False) -> np.ndarray:
    """He-normal conv/FC weights N(0, 2/fan_in), gamma=1, beta=0, bias=0.
    randomize_affine draws gamma ~ U(0.5,1.5), beta, bias ~ N(0,0.1) instead
    (used by tests so that no term is hidden by a neutral value)."""
    flat = np.empty(n_params(spec), dtype=np.float32)
    for e in param_layout(spec):
        sl = slice(e.offset, e.offset + e.size)
        if e.kind in ("conv", "fc"):
            fan_in = int(np.prod(e.shape[:-1]))
            flat[sl] = rng.normal(0.0, np.sqrt(2.0 / fan_in), e.size).astype(np.float32)
        elif e.kind == "gamma":
            flat[sl] = rng.uniform(0.5, 1.5, e.size) if randomize_affine else 1.0
        else:
            flat[sl] = rng.normal(0.0, 0.1, e.size) if randomize_affine else 0.0
    return flat


def make_inputs(spec: PartitionSpec, randomize_affine: bool = False) -> StepInputs:
    """Draw order: parameters in canonical order, then per micro-batch in index
    order: act_in ~ N(0,1); labels uniform in [0, classes) if the partition has
    the head, else err_in ~ N(0, variance 1e-2) with the shape of act_out."""
    rng = np.random.default_rng(spec.seed)
    params = make_params(spec, rng, randomize_affine)
    b = spec.microbatch
    oh, ow, oc = spec.out_shape()
    act_in, labels, err_in, skip_in, skip_err_in = [], [], [], [], []
    for _ in range(spec.num_microbatches):
        act_in.append(rng.standard_normal((b, spec.in_h, spec.in_w, spec.in_c), dtype=np.float32))
        if spec.has_head:
            labels.append(rng.integers(0, spec.num_classes, size=b, dtype=np.int32))
        else:
            err_in.append((0.1 * rng.standard_normal((b, oh, ow, oc), dtype=np.float32)))
        if spec.has_skip_in:
            skip_in.append(rng.standard_normal((b,) + spec.skip_in_shape(), dtype=np.float32))
        if spec.has_skip_out:
            skip_err_in.append(0.1 * rng.standard_normal((b,) + spec.skip_out_shape(), dtype=np.float32))
    return StepInputs(params, act_in, labels if spec.has_head else None,
                      None if spec.has_head else err_in, skip_in or None, skip_err_in or None)
