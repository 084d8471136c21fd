"""GPU parity, layer by layer and block by block, at full size: every tensor the device keeps for
back-propagation, for every block and micro-batch of the benchmark configurations, against the plain CPU oracle
(float64, nothing rounded) fed the device's own layer inputs / block inputs (tests/teacher.py).  Element-wise,
2e-2 (bf16 operands) / 1e-4 (fp32 check mode), in the launch configuration bench.py times (all micro-batches of
the batch in one group call per direction)."""
import time

import numpy as np
import pytest

from paper_1911_05146_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: these tests need a real MI355X")
    from paper_1911_05146_amd import hpf
    return hpf


def layerwise(oracle, spec, mode, grouped=True, fusion=2, randomize_affine=True, blockwise=True):
    from parity import run_gpu_step
    from teacher import blockwise_check, layerwise_check
    print(f"\n[case] layer-wise {spec.name} b={spec.microbatch} m={spec.num_microbatches} mode={mode} grouped={grouped} "
          f"fusion={fusion} seed={spec.seed}", flush=True)
    inp = W.make_inputs(spec, randomize_affine=randomize_affine)
    t0 = time.time()
    seen, res = run_gpu_step(spec, inp, mode, grouped=grouped, fusion=fusion, keep=True)
    part = res.pop("part")
    try:
        rep = layerwise_check(oracle, part, spec, seen, res, mode)
        print(f"[layer-wise] {spec.name} {mode}: {rep.summary()} ({time.time() - t0:.0f} s)", flush=True)
        if blockwise:
            t0 = time.time()
            rb = blockwise_check(oracle, part, spec, seen, res, mode)
            print(f"[block-wise] {spec.name} {mode}: {rb.summary()}; {rb.extra} ({time.time() - t0:.0f} s)", flush=True)
    finally:
        part.close()
    return rep


@pytest.mark.parametrize("mode", ["bf16", "f32"])
def test_single_blocks_layerwise(gpu, oracle, mode):
    """Every block kind at its full micro-batch, first seed, no retries."""
    cases = {
        "bottleneck-identity-r1001-stage2": (W.Block(W.BOTTLENECK, 128, 32, 128, 1), 16, 32),
        "bottleneck-entry-stride2-proj": (W.Block(W.BOTTLENECK, 64, 32, 128, 2), 16, 8),
        "bottleneck-widen-proj-stride1": (W.Block(W.BOTTLENECK, 16, 16, 64, 1), 32, 8),
        "bottleneck-wide-identity": (W.Block(W.BOTTLENECK, 128, 64, 128, 1), 16, 8),
        "basic-identity": (W.Block(W.BASIC, 32, 32, 32, 1), 16, 16),
        "basic-identity-64": (W.Block(W.BASIC, 64, 64, 64, 1), 8, 16),
        "basic-entry-stride2-proj": (W.Block(W.BASIC, 32, 64, 64, 2), 16, 16),
        "bottleneck-r152-stage3": (W.Block(W.BOTTLENECK, 1024, 256, 1024, 1), 14, 4),
        "bottleneck-r152-entry": (W.Block(W.BOTTLENECK, 512, 256, 1024, 2), 28, 2),
    }
    for name, (blk, hw, b) in cases.items():
        spec = W.PartitionSpec(name=name, in_h=hw, in_w=hw, in_c=blk.c_in, blocks=(blk,), microbatch=b,
                               num_microbatches=2, seed=21)
        layerwise(oracle, spec, mode)


def test_row_band_runs_layerwise(gpu, oracle):
    """Runs of 64-16-16-64 bottlenecks at 32x32 (the first stage of ResNet-1001): each image is cut into four bands of
    eight rows, one work-group each, and the rows next to a band travel with the BatchNorm records.  Three blocks, so
    that every exchange of the loop runs; an odd number of images; one and several micro-batches per launch."""
    blocks = tuple(W.Block(W.BOTTLENECK, 64, 16, 64, 1) for _ in range(3))
    for b, m, grouped in ((8, 2, True), (3, 2, True), (5, 3, False)):
        spec = W.PartitionSpec(name=f"bands-3x(64-16-64)@32x32-b{b}", in_h=32, in_w=32, in_c=64, blocks=blocks, microbatch=b,
                               num_microbatches=m, seed=23)
        layerwise(oracle, spec, "bf16", grouped=grouped)
    spec = W.PartitionSpec(name="bands-3x(64-16-64)@32x32-level1", in_h=32, in_w=32, in_c=64, blocks=blocks, microbatch=4,
                           num_microbatches=2, seed=23)
    layerwise(oracle, spec, "bf16", fusion=1)


def test_runs_with_weights_through_lds_layerwise(gpu, oracle):
    """Resident runs whose weight matrices the work-group stages through LDS: 128-64 bottlenecks at 16x16 (through the
    tile that is idle at the time, conv2 in three rounds), 128-32 at 16x16, 32-channel basic and post-activation blocks,
    16-channel basic and post-activation blocks at 32x32.
    Three blocks, so that the staging of the first block, of a following block and of the last one all run; an odd
    number of images; one call per micro-batch and one for all."""
    runs = {
        "wide-3x(128-64-128)@16x16": (tuple(W.Block(W.BOTTLENECK, 128, 64, 128, 1) for _ in range(3)), 16, 128, True),
        "3x(128-32-128)@16x16": (tuple(W.Block(W.BOTTLENECK, 128, 32, 128, 1) for _ in range(3)), 16, 128, True),
        "3x basic32@16x16": (tuple(W.Block(W.BASIC, 32, 32, 32, 1) for _ in range(3)), 16, 32, True),
        "3x basic16@32x32": (tuple(W.Block(W.BASIC, 16, 16, 16, 1) for _ in range(3)), 32, 16, True),
        "3x postact32@16x16": (tuple(W.Block(W.POSTACT, 32, 32, 32, 1) for _ in range(3)), 16, 32, False),
        "3x postact16@32x32": (tuple(W.Block(W.POSTACT, 16, 16, 16, 1) for _ in range(3)), 32, 16, False),
    }
    # 40 images per micro-batch: the gathered 128-channel records then reach into the tile that also takes a weight matrix
    spec = W.PartitionSpec(name="wide-3x(128-64-128)@16x16-b40", in_h=16, in_w=16, in_c=128, blocks=runs["wide-3x(128-64-128)@16x16"][0],
                           microbatch=40, num_microbatches=2, seed=37)
    layerwise(oracle, spec, "bf16", blockwise=False)
    spec = W.PartitionSpec(name="3x(128-32-128)@16x16-b40", in_h=16, in_w=16, in_c=128, blocks=runs["3x(128-32-128)@16x16"][0],
                           microbatch=40, num_microbatches=2, seed=37)   # the records fill both narrow tiles
    layerwise(oracle, spec, "bf16", blockwise=False)
    # 100 images per micro-batch: the records no longer fit a tile and are gathered in an area of their own, behind
    # which the staged matrix then lies
    for name, blocks, hw, c in (("3x basic32@16x16-b100", runs["3x basic32@16x16"][0], 16, 32),
                                ("3x basic64@8x8-b100", tuple(W.Block(W.BASIC, 64, 64, 64, 1) for _ in range(3)), 8, 64),
                                ("3x postact32@16x16-b100", runs["3x postact32@16x16"][0], 16, 32)):
        spec = W.PartitionSpec(name=name, in_h=hw, in_w=hw, in_c=c, blocks=blocks, microbatch=100, num_microbatches=2, seed=37)
        layerwise(oracle, spec, "bf16", blockwise=False)
    for name, (blocks, hw, c, blockwise) in runs.items():
        for b, m, grouped in ((3, 2, True), (4, 3, False)):
            spec = W.PartitionSpec(name=f"{name}-b{b}", in_h=hw, in_w=hw, in_c=c, blocks=blocks, microbatch=b,
                                   num_microbatches=m, seed=37)
            layerwise(oracle, spec, "bf16", grouped=grouped, blockwise=blockwise)


def test_convolutions_with_split_reductions_layerwise(gpu, oracle):
    """Plain 3x3 convolution units with long reductions into few output tiles (VGG-16's last two groups: 512 channels on
    4x4 and 2x2 pixels) run with every reduction split over two to four work-groups whose fp32 partial sums a second
    launch adds up, in both directions.  Group sizes 1 and several (the split count depends on it), a ragged last
    tile (48 pixel rows), 9 x 256 and 9 x 512 reduction elements (36 and 72 steps: splits of unequal length)."""
    cases = (("512@4x4", 512, 512, 4, 16, 2, True), ("512@4x4-single-calls", 512, 512, 4, 16, 2, False),
             ("512@2x2-ragged", 512, 512, 2, 12, 3, True), ("256-512@4x4", 256, 512, 4, 8, 2, True))
    for name, cin, cout, hw, b, m, grouped in cases:
        blocks = (W.Block(W.CONV_RELU, cin, cout, cout, 1), W.Block(W.CONV_RELU, cout, cout, cout, 1))
        spec = W.PartitionSpec(name=f"splitk-{name}-b{b}", in_h=hw, in_w=hw, in_c=cin, blocks=blocks, microbatch=b,
                               num_microbatches=m, seed=41)
        layerwise(oracle, spec, "bf16", grouped=grouped, blockwise=False)
    layerwise(oracle, spec, "bf16", fusion=0, blockwise=False)   # every step a kernel of its own: the same convolution launches


def test_whole_image_weight_gradient_of_16_channel_convolutions_layerwise(gpu, oracle):
    """3x3 convolutions between 16 and 16 channels on 1024-pixel images take the weight-gradient kernel that forms all
    nine taps from one staging of an image.  Square images (32 pixels per row: one image row per MFMA step) and the
    two other row lengths it accepts (16 and 8 pixels: two and four image rows per step, other border lanes); image
    counts that do not divide into equal work items; one image; pre- and post-activation operands (with and without
    the BatchNorm recomputed while staging); one call per micro-batch and one for all."""
    basic = tuple(W.Block(W.BASIC, 16, 16, 16, 1) for _ in range(2))
    for (h, w), b, m, grouped in (((32, 32), 5, 3, True), ((32, 32), 1, 2, False), ((64, 16), 3, 2, True), ((128, 8), 2, 2, True)):
        spec = W.PartitionSpec(name=f"t9-basic16@{h}x{w}-b{b}", in_h=h, in_w=w, in_c=16, blocks=basic, microbatch=b,
                               num_microbatches=m, seed=29)
        layerwise(oracle, spec, "bf16", grouped=grouped)
    # many convolutions of the class in one partition: the work items then take several images each (here 3, 3, ..., 2)
    many = tuple(W.Block(W.BASIC, 16, 16, 16, 1) for _ in range(40))
    spec = W.PartitionSpec(name="t9-40xbasic16@32x32-b32", in_h=32, in_w=32, in_c=16, blocks=many, microbatch=32,
                           num_microbatches=2, seed=29)
    layerwise(oracle, spec, "bf16", blockwise=False)
    post = tuple(W.Block(W.POSTACT, 16, 16, 16, 1) for _ in range(2))
    for fusion in (2, 1, 0):
        spec = W.PartitionSpec(name=f"t9-postact16@32x32-level{fusion}", in_h=32, in_w=32, in_c=16, blocks=post, microbatch=6,
                               num_microbatches=2, seed=31)
        layerwise(oracle, spec, "bf16", fusion=fusion, blockwise=False)   # the block-wise harness covers pre-activation blocks


def test_config1_resnet20_layerwise(gpu, oracle):
    for mode in ("bf16", "f32"):
        layerwise(oracle, W.config(1), mode, grouped=False)
        layerwise(oracle, W.config(1), mode, grouped=True)


def test_config2_resnet110_partition_full_size_layerwise(gpu, oracle):
    """Full size in the launch configuration bench.py times; the other fusion level and the fp32 mode on two of the eight
    micro-batches (same micro-batch size, same kernels)."""
    layerwise(oracle, W.config(2), "bf16")
    small = W.with_microbatching(W.config(2), 16, 2, loss_divisor=128)
    layerwise(oracle, small, "bf16", fusion=1)
    layerwise(oracle, small, "f32")


def test_config3_resnet1001_partition_full_size_layerwise(gpu, oracle):
    """The benchmark configuration: 21 blocks x 8 micro-batches x 32 images through the image-resident kernels."""
    layerwise(oracle, W.config(3), "bf16")


def test_config3_other_schedules_layerwise(gpu, oracle):
    spec = W.with_microbatching(W.config(3), 32, 2, loss_divisor=256)
    layerwise(oracle, spec, "bf16", fusion=1, blockwise=False)
    layerwise(oracle, spec, "bf16", fusion=0, blockwise=False)
    layerwise(oracle, spec, "bf16", grouped=False)
    layerwise(oracle, W.with_microbatching(W.config(3), 8, 2, loss_divisor=256), "f32")


def test_config6_wide_resnet1001_partition_full_size_layerwise(gpu, oracle):
    """Layer by layer at full size; block by block on two of the eight micro-batches."""
    layerwise(oracle, W.config(6), "bf16", blockwise=False)
    layerwise(oracle, W.with_microbatching(W.config(6), 32, 2, loss_divisor=256), "bf16")


def test_config4_resnet1001_whole_full_size_layerwise(gpu, oracle):
    """333 blocks + stem + head, 8 micro-batches of 8 images."""
    layerwise(oracle, W.config(4), "bf16", blockwise=False)


def test_config5_resnet152_stage3_full_size_layerwise(gpu, oracle):
    """36 blocks at 14x14x1024, 4 micro-batches of 16 images (3 TFLOP per oracle pass)."""
    layerwise(oracle, W.config(5), "bf16", blockwise=False)
