"""GPU parity: the HIP library against the CPU oracle, element by element, on the same seeded
inputs, through the C ABI.  Tolerances (max|gpu-ref| / max|ref| per tensor): 2e-2 with bf16
operands, 1e-4 in the fp32 check mode."""
from dataclasses import replace

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


def to64(inp):
    return W.StepInputs(inp.params.astype(np.float64), [a.astype(np.float64) for a in inp.act_in], inp.labels,
                        [e.astype(np.float64) for e in inp.err_in] if inp.err_in else None)


def check(oracle, spec, mode, multi_stream=False, sgd=None, randomize_affine=True, strict=False, beta_shift=0.0,
          grouped=False, fusion=2):
    """GPU batch vs the oracle in the same precision reading (criterion A), falling back -- unless
    strict -- to the sensitivity-limited criterion B against the oracle in double (see parity.compare)."""
    return check_once(oracle, spec, mode, multi_stream, sgd, randomize_affine, strict, beta_shift, grouped, fusion)


def check_block(oracle, spec, mode, grouped=False, fusion=2):
    """Shallow bf16 cases with ReLUs in play: every layer, and the block end to end, against the plain oracle with
    the differing ReLU decisions found explicitly (tests/teacher.py); first seed, no retries."""
    from teacher import run_and_check
    print(f"\n[case] {spec.name} b={spec.microbatch} m={spec.num_microbatches} mode={mode} grouped={grouped} "
          f"fusion={int(fusion)} seed={spec.seed} (layer-wise and block-wise)", flush=True)
    return run_and_check(oracle, spec, mode, grouped=grouped, fusion=int(fusion))


def check_once(oracle, spec, mode, multi_stream, sgd, randomize_affine, strict, beta_shift, grouped=False, fusion=2):
    from parity import compare, fmt, needs_layerwise, run_gpu_step
    print(f"\n[case] {spec.name} b={spec.microbatch} m={spec.num_microbatches} mode={mode} streams={multi_stream} "
          f"grouped={grouped} fusion={int(fusion)} seed={spec.seed}", flush=True)
    inp = W.make_inputs(spec, randomize_affine=randomize_affine)
    if beta_shift:
        for e in W.param_layout(spec):
            if e.kind == "beta":
                inp.params[e.offset:e.offset + e.size] += beta_shift
    seen, res = run_gpu_step(spec, inp, mode, multi_stream=multi_stream, sgd=sgd, grouped=grouped, fusion=fusion, keep=True)
    part = res.pop("part")
    try:
        yard = oracle.run_step(spec, seen, np.float32, sgd=sgd, storage="bf16" if mode == "bf16" else "none")
        rep = compare(spec, res, yard, mode, ref64=lambda: oracle.run_step(spec, to64(seen), np.float64, sgd=sgd), strict=strict,
                      insensitive="skip")
        print(f"[parity] {spec.name} {mode}: " + fmt(rep), flush=True)
        if needs_layerwise(rep) and spec.first_from == 0 and spec.last_to == 0:
            # end to end some tensors passed only statistically, or could not be judged at all: every layer on its own
            from teacher import layerwise_check
            lw = layerwise_check(oracle, part, spec, seen, res, mode)
            print(f"[layer-wise] {spec.name} {mode}: {lw.summary()}", flush=True)
    finally:
        part.close()
    return rep


# ---- shallow partitions: element-wise parity is required (criterion A only) -----------------------
@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_single_blocks_of_every_kind(gpu, oracle, mode):
    cases = {
        "bottleneck-identity-r1001-stage2": (W.Block(W.BOTTLENECK, 128, 32, 128, 1), 16, 32),
        "bottleneck-entry-stride2-proj": (W.Block(W.BOTTLENECK, 64, 32, 128, 2), 16, 8),
        "bottleneck-widen-proj-stride1": (W.Block(W.BOTTLENECK, 16, 16, 64, 1), 32, 8),
        "basic-identity": (W.Block(W.BASIC, 32, 32, 32, 1), 16, 16),
        "basic-entry-stride2-proj": (W.Block(W.BASIC, 32, 64, 64, 2), 16, 16),
        "bottleneck-r152-stage3": (W.Block(W.BOTTLENECK, 1024, 256, 1024, 1), 14, 3),
    }
    for name, (blk, hw, b) in cases.items():
        spec = W.PartitionSpec(name=name, in_h=hw, in_w=hw, in_c=blk.c_in, blocks=(blk,), microbatch=b,
                               num_microbatches=2, seed=21)
        if mode == "bf16":
            check_block(oracle, spec, mode)
        else:
            check(oracle, spec, mode, strict=True)


def test_separate_bn_reduction_kernels_bf16(gpu, oracle):
    """bf16 mode with the BatchNorm reductions as separate kernels (fusion off): same criteria."""
    check(oracle, W.resnet20(), "bf16", strict=True, beta_shift=6.0, sgd=(0.1, 0.9), fusion=False)
    check(oracle, W.config(1), "bf16", sgd=(0.1, 0.9), fusion=False)
    check(oracle, W.with_microbatching(W.config(2), 16, 2, loss_divisor=128), "bf16", fusion=False, grouped=True)
    blk = W.Block(W.BOTTLENECK, 64, 32, 128, 2)
    spec = W.PartitionSpec(name="entry-unfused", in_h=16, in_w=16, in_c=64, blocks=(blk,), microbatch=2, num_microbatches=2, seed=21)
    check_block(oracle, spec, "bf16", fusion=0)


def _bottleneck_run(name, c, mid, hw, n, b, m, seed=31, **kw):
    blk = W.Block(W.BOTTLENECK, c, mid, c, 1)
    return W.PartitionSpec(name=name, in_h=hw, in_w=hw, in_c=c, blocks=(blk,) * n, microbatch=b, num_microbatches=m, seed=seed, **kw)


def test_image_resident_runs_small(gpu, oracle):
    """Runs of identity bottleneck blocks in the image-resident kernels (fusion level 2), in every shape class
    the path covers.  With every pre-activation above 0 (beta + 6) no ReLU decision can differ and the run must
    agree element by element; with ReLUs in play one block is checked layer by layer and end to end with the
    differing ReLU decisions found explicitly (check_block), longer runs fall under the same criteria as every
    other partition."""
    cases = [
        (_bottleneck_run("resident-128x32-16x16", 128, 32, 16, 2, 2, 2), False),
        (_bottleneck_run("resident-128x32-8x8", 128, 32, 8, 2, 3, 2), False),
        (_bottleneck_run("resident-128x32-8x8-grouped", 128, 32, 8, 3, 2, 3, seed=33), True),
        (_bottleneck_run("resident-256x64-8x8", 256, 64, 8, 2, 2, 2), False),
        (replace(_bottleneck_run("resident-128x32-8x16", 128, 32, 16, 2, 2, 2, seed=35), in_h=8), True),
    ]
    for spec, grouped in cases:
        check(oracle, spec, "bf16", strict=True, beta_shift=6.0, grouped=grouped)
        check_block(oracle, replace(spec, blocks=spec.blocks[:1]), "bf16", grouped=grouped)
        check(oracle, spec, "bf16", grouped=grouped)


def test_image_resident_runs_of_wide_bottlenecks(gpu, oracle):
    """128-64-64-128 blocks (the 30 M-parameter ResNet-1001): at 256 pixels the backward kernel reads c1 / c2 at the
    accumulator positions instead of staging them as tiles."""
    cases = [
        (_bottleneck_run("resident-128x64-16x16", 128, 64, 16, 2, 2, 2, seed=51), False),
        (_bottleneck_run("resident-128x64-8x8-grouped", 128, 64, 8, 3, 3, 2, seed=52), True),
        (replace(_bottleneck_run("resident-128x64-8x16", 128, 64, 16, 2, 2, 3, seed=53), in_h=8), True),
    ]
    for spec, grouped in cases:
        check(oracle, spec, "bf16", strict=True, beta_shift=6.0, grouped=grouped)
        check_block(oracle, replace(spec, blocks=spec.blocks[:1]), "bf16", grouped=grouped)
        check(oracle, spec, "bf16", grouped=grouped)
    check(oracle, _bottleneck_run("resident-128x64-deep-active", 128, 64, 16, 21, 8, 2, seed=54), "bf16", beta_shift=6.0, grouped=True)
    check(oracle, _bottleneck_run("resident-128x64-deep", 128, 64, 16, 21, 8, 2, seed=55), "bf16", grouped=True)


def test_image_resident_runs_of_basic_blocks(gpu, oracle):
    """The ResNet-20 / ResNet-110 family: runs of basic blocks (two 3x3 convolutions) in the image-resident kernels."""
    def basic_run(name, c, hw, n, b, m, seed=43):
        blk = W.Block(W.BASIC, c, c, c, 1)
        return W.PartitionSpec(name=name, in_h=hw, in_w=hw, in_c=c, blocks=(blk,) * n, microbatch=b, num_microbatches=m, seed=seed)
    for spec, grouped in ((basic_run("resident-basic-32x16x16", 32, 16, 2, 2, 2), False),
                          (basic_run("resident-basic-64x8x8", 64, 8, 3, 3, 2), True),
                          (replace(basic_run("resident-basic-32x8x16", 32, 16, 2, 2, 3, seed=45), in_h=8), True)):
        check(oracle, spec, "bf16", strict=True, beta_shift=6.0, grouped=grouped)
        check_block(oracle, replace(spec, blocks=spec.blocks[:1]), "bf16", grouped=grouped)
        check(oracle, spec, "bf16", grouped=grouped)
    check(oracle, basic_run("resident-basic-deep", 32, 16, 9, 16, 2), "bf16", grouped=True)
    check(oracle, basic_run("resident-basic-deep-active", 32, 16, 9, 16, 2), "bf16", beta_shift=6.0, grouped=True)


def test_image_resident_runs_deep_and_mixed(gpu, oracle):
    """Deep runs (ReLU always active: element-wise; otherwise the sensitivity-limited criterion), runs between
    other units (stem, projection blocks, head), runs split by a shape change, and groups of micro-batches."""
    check(oracle, _bottleneck_run("resident-deep-active", 128, 32, 16, 21, 8, 2), "bf16", beta_shift=6.0, grouped=True)
    check(oracle, _bottleneck_run("resident-deep", 128, 32, 16, 21, 8, 3), "bf16", grouped=True)
    blocks = (W.Block(W.BOTTLENECK, 64, 32, 128, 2),) + (W.Block(W.BOTTLENECK, 128, 32, 128, 1),) * 3 + \
             (W.Block(W.BOTTLENECK, 128, 64, 256, 2),) + (W.Block(W.BOTTLENECK, 256, 64, 256, 1),) * 2
    mixed = W.PartitionSpec(name="resident-mixed-stem-head", in_h=32, in_w=32, in_c=3, has_stem=True, stem_c_out=64, blocks=blocks,
                            has_head=True, num_classes=10, microbatch=4, num_microbatches=3, seed=37)
    check(oracle, mixed, "bf16", sgd=(0.1, 0.9))
    check(oracle, mixed, "bf16", grouped=True)
    check(oracle, replace(mixed, name="resident-mixed-level1"), "bf16", fusion=1)


def test_image_resident_runs_edge_cases(gpu, oracle):
    """One image per micro-batch (the all-gather has a single member), an odd micro-batch (weight-gradient groups of
    one image), more images than CUs (the run falls back to the per-layer kernels), and the level switch between
    batches of one handle."""
    from parity import run_gpu_step, rel_err
    check(oracle, _bottleneck_run("resident-single-image", 128, 32, 16, 2, 1, 3), "bf16", strict=True, beta_shift=6.0, grouped=True)
    check(oracle, _bottleneck_run("resident-odd-microbatch", 128, 32, 8, 2, 5, 2), "bf16", strict=True, beta_shift=6.0)
    check(oracle, _bottleneck_run("resident-more-images-than-cus", 128, 32, 8, 1, 260, 1), "bf16", strict=True, beta_shift=6.0)
    # 7 micro-batches of 48 images in one group call: at most 5 fit the chip at once, so the call runs as launches of
    # 5 and 2 micro-batches; weight-gradient groups of 8 images
    check(oracle, _bottleneck_run("resident-chunked-group-call", 128, 32, 8, 2, 48, 7, seed=47), "bf16", strict=True, beta_shift=6.0,
          grouped=True)
    # 12 images per micro-batch: weight-gradient groups of 4 images, 3 members per channel subset in the merges
    check(oracle, _bottleneck_run("resident-microbatch-12", 128, 64, 8, 2, 12, 3, seed=48), "bf16", strict=True, beta_shift=6.0,
          grouped=True)
    spec = _bottleneck_run("resident-level-switch", 128, 32, 8, 2, 4, 2, seed=41)
    inp = W.make_inputs(spec, randomize_affine=True)
    _, r2 = run_gpu_step(spec, inp, "bf16", keep=True, fusion=2)
    part = r2["part"]
    part.grad_accum_zero()
    part.set_fusion(1)
    _, r1 = run_gpu_step(spec, inp, "bf16", part=part)
    part.grad_accum_zero()
    part.set_fusion(2)
    _, r2b = run_gpu_step(spec, inp, "bf16", part=part)
    part.close()
    for x, y in zip(r2["act_out"] + r2["err_out"], r2b["act_out"] + r2b["err_out"]):
        assert np.array_equal(x, y)                       # the same schedule twice: identical tensors
    assert rel_err(r2b["grad"], r2["grad"]) < 1e-5         # fp32 atomics in another order
    assert rel_err(r1["act_out"][0], r2["act_out"][0]) < 2e-2   # the other schedule: another bf16 evaluation


def test_fusion_levels_agree_on_the_benchmark_partition(gpu, oracle):
    """The three kernel schedules are three bf16 evaluations of the same batch."""
    spec = W.with_microbatching(W.config(3), 32, 2, loss_divisor=256)
    for level in (0, 1, 2):
        check(oracle, spec, "bf16", fusion=level, grouped=(level == 2))


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_head_only_and_stem_only_partitions(gpu, oracle, mode):
    head = W.PartitionSpec(name="head-only", in_h=8, in_w=8, in_c=64, blocks=(), has_head=True, num_classes=10,
                           microbatch=4, num_microbatches=2, seed=9)
    check(oracle, head, mode, strict=True)
    stem = W.PartitionSpec(name="stem-only", in_h=16, in_w=16, in_c=3, blocks=(), has_stem=True, stem_c_out=16,
                           microbatch=2, num_microbatches=2, seed=10)
    check(oracle, stem, mode, strict=True)
    wide = W.PartitionSpec(name="head-1000-classes", in_h=7, in_w=7, in_c=256, blocks=(), has_head=True,
                           num_classes=1000, microbatch=3, num_microbatches=1, seed=12)
    check(oracle, wide, mode, strict=True)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_deep_partitions_with_relu_always_active(gpu, oracle, mode):
    """beta shifted by +6 puts every pre-activation above 0: no ReLU decision can differ, so the deep
    backward pass (indexing, accumulation, shortcut gradients) must agree element by element."""
    strict = mode == "f32"   # bf16: rounding of 60 stored tensors in a row alone passes 2e-2 (no ReLU involved)
    check(oracle, W.with_microbatching(W.config(2), 8, 2, loss_divisor=128), mode, strict=strict, beta_shift=6.0)
    check(oracle, W.with_microbatching(W.config(3), 8, 2, loss_divisor=256), mode, strict=strict, beta_shift=6.0)
    check(oracle, W.resnet20(), mode, strict=True, beta_shift=6.0, sgd=(0.1, 0.9))


def test_fp32_check_mode_is_elementwise_on_medium_partitions(gpu, oracle):
    """Up to a few million stored elements the check mode (fp32 tensors, double sums) and the oracle
    agree to rounding of the last bit, ReLU decisions included."""
    check(oracle, W.config(1), "f32", sgd=(0.1, 0.9), strict=True)
    check(oracle, W.config(1), "f32", randomize_affine=False, strict=True)
    for p in (0, 1, 2, 3):
        check(oracle, W.resnet110_partition(p=p, microbatch=4, num_microbatches=2), "f32", strict=True)
    check(oracle, W.resnet152_stage3(n_blocks=3, microbatch=2, num_microbatches=2), "f32", strict=True)
    check(oracle, W.with_microbatching(W.config(3), 4, 2, loss_divisor=256), "f32", strict=True)


# ---- the benchmark partitions: A where it holds, B where ReLU sensitivity limits it ----------------
@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_resnet20_whole_model_with_sgd(gpu, oracle, mode):
    check(oracle, W.config(1), mode, sgd=(0.1, 0.9))
    check(oracle, W.config(1), mode, randomize_affine=False)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_resnet110_partitions(gpu, oracle, mode):
    check(oracle, W.with_microbatching(W.config(2), 16, 2, loss_divisor=128), mode)
    for p in (0, 1, 3):
        check(oracle, W.resnet110_partition(p=p, microbatch=4, num_microbatches=2), mode)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_resnet1001_partition_two_microbatches(gpu, oracle, mode):
    check(oracle, W.with_microbatching(W.config(3), 32, 2, loss_divisor=256), mode)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_resnet1001_wide_partition_two_microbatches(gpu, oracle, mode):
    """The 30 M-parameter variant (inner widths 16 / 64 / 128): 21 blocks 128-64-64-128 at 16x16."""
    check(oracle, W.with_microbatching(W.config(6), 8, 2, loss_divisor=64), mode)


def test_resnet1001_partition_full_batch_on_streams(gpu, oracle):
    """8 micro-batches of 32, one stream each."""
    check(oracle, W.config(3), "bf16", multi_stream=True, randomize_affine=False)


def test_resnet1001_partition_full_batch_grouped(gpu, oracle):
    """The benchmark's launch configuration: the 8 micro-batches of 32 issued as one group."""
    check(oracle, W.config(3), "bf16", grouped=True, randomize_affine=False)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_grouped_calls_equal_single_calls(gpu, oracle, mode):
    """A group call is the same work as single calls: bit-identical activations and errors."""
    from parity import rel_err, run_gpu_step
    for spec in (W.resnet20(microbatch=4, num_microbatches=3), W.resnet110_partition(p=2, microbatch=4, num_microbatches=8),
                 W.resnet110_partition(p=1, microbatch=2, num_microbatches=11)):     # 11 > 8: two groups
        inp = W.make_inputs(spec, randomize_affine=True)
        _, a = run_gpu_step(spec, inp, mode)
        _, b = run_gpu_step(spec, inp, mode, grouped=True)
        for x, y in zip(a["act_out"] + a["err_out"], b["act_out"] + b["err_out"]):
            assert (x is None and y is None) or np.array_equal(x, y)
        assert abs(a["loss"] - b["loss"]) <= 1e-6 * abs(a["loss"]) + 1e-12
        assert rel_err(b["grad"], a["grad"]) < 1e-5
    check(oracle, W.resnet20(microbatch=4, num_microbatches=2), mode, grouped=True, sgd=(0.1, 0.9), strict=(mode == "f32"))


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_resnet1001_whole_model_small_batch(gpu, oracle, mode):
    """333 blocks at 2 micro-batches of 2 images: end to end the backward pass of this network says nothing (two
    evaluations of the oracle itself, float and double, differ by a third in G), so every layer is checked on its
    own; the full-size configuration is in test_gpu_teacher.py."""
    from teacher import run_and_check
    spec = W.resnet1001_whole(microbatch=2, num_microbatches=2)
    print(f"\n[case] {spec.name} b=2 m=2 mode={mode} (layer-wise)", flush=True)
    run_and_check(oracle, spec, mode, randomize_affine=False, blockwise=False)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_resnet152_stage3_first_blocks(gpu, oracle, mode):
    check(oracle, W.resnet152_stage3(n_blocks=3, microbatch=2, num_microbatches=2), mode)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_ragged_tiles_and_single_image(gpu, oracle, mode):
    # 14x14 images, b = 3: 588 rows -- not a multiple of any tile; b = 1 with stride 2
    blocks = (W.Block(W.BOTTLENECK, 64, 32, 128, 2), W.Block(W.BOTTLENECK, 128, 32, 128, 1),
              W.Block(W.BASIC, 128, 48 if mode == "f32" else 64, 48 if mode == "f32" else 64, 1))
    spec = W.PartitionSpec(name="ragged", in_h=28, in_w=28, in_c=64, blocks=blocks, microbatch=3, num_microbatches=2, seed=5)
    check(oracle, spec, mode)
    check(oracle, replace(spec, name="single-image", microbatch=1, num_microbatches=3), mode)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_frozen_batchnorm_mode(gpu, oracle, mode):
    check(oracle, replace(W.resnet110_partition(p=2, microbatch=4, num_microbatches=2), bn_mode=1), mode)


def test_streams_give_the_same_result_as_one_stream(gpu, oracle):
    from parity import run_gpu_step, rel_err
    spec = W.with_microbatching(W.config(2), 16, 4, loss_divisor=128)
    inp = W.make_inputs(spec)
    _, a = run_gpu_step(spec, inp, "bf16", multi_stream=False)
    _, b = run_gpu_step(spec, inp, "bf16", multi_stream=True)
    for x, y in zip(a["act_out"] + a["err_out"], b["act_out"] + b["err_out"]):
        assert np.array_equal(x, y)                      # activations and errors: no atomics involved
    assert rel_err(b["grad"], a["grad"]) < 1e-5          # gradient sums: fp32 atomics, order may differ


def test_directions_on_different_streams_wait_for_each_other(gpu, oracle):
    """Forward group on one stream, backward group on a second, the clearing of the gradient buffer on a third:
    the library's events order them (waits are only skipped between calls on one and the same stream)."""
    import torch
    from parity import device_inputs, run_gpu_step, rel_err
    from paper_1911_05146_amd import hpf
    spec = W.with_microbatching(W.config(3), 8, 4, loss_divisor=32)
    inp = W.make_inputs(spec)
    _, ref = run_gpu_step(spec, inp, "bf16", grouped=True)
    _, t = device_inputs(spec, inp, "bf16")
    part = hpf.Partition(spec, inp.params, hpf.HPF_BF16)
    sa, sb, sc = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(3):                                   # several batches: events are re-recorded on changing streams
        part.grad_accum_zero(stream=sc)
        outs = part.forward_microbatches(0, t["act_in"], None, stream=sa)
        errs = part.backward_microbatches(0, 4, t["err_in"], stream=sb)
        sa, sb, sc = sb, sc, sa
    grad = part.grad_accum_read()
    torch.cuda.synchronize()
    for x, y in zip(outs + errs, ref["act_out"] + ref["err_out"]):
        assert np.array_equal(x.float().cpu().numpy(), y)
    assert rel_err(grad, ref["grad"]) < 1e-5             # one batch's sums: the buffer was cleared before each
    part.close()


def test_two_batches_accumulate_zero_and_step(gpu, oracle):
    """Gradient buffer life cycle over consecutive batches on one handle."""
    from parity import run_gpu_step, rel_err
    spec = W.resnet110_partition(p=3, microbatch=4, num_microbatches=2)
    inp = W.make_inputs(spec, randomize_affine=True)
    seen, r1 = run_gpu_step(spec, inp, "f32", keep=True)
    part = r1["part"]
    part.grad_accum_zero()
    _, r2 = run_gpu_step(spec, inp, "f32", part=part)          # same batch again after zeroing
    assert rel_err(r2["grad"], r1["grad"]) < 1e-5
    part.sgd_step(0.1, 0.9)
    w1 = part.params_read()
    assert rel_err(w1, inp.params - 0.1 * r2["grad"]) < 1e-6
    _, r3 = run_gpu_step(spec, inp, "f32", part=part)          # next batch: buffer was cleared by the step
    ref = oracle.OraclePartition(spec, w1)
    for i in range(2):
        ref.forward(i, seen.act_in[i], seen.labels[i])
    for i in range(2):
        ref.backward(i, None, want_err_out=False)
    assert rel_err(r3["grad"], ref.grad()) < 1e-4
    part.sgd_step(0.1, 0.9)
    assert rel_err(part.params_read(), w1 - 0.1 * (0.9 * r2["grad"] + r3["grad"])) < 1e-5
    part.close()


def test_call_order_and_arguments_are_enforced(gpu):
    import torch
    hpf = gpu
    spec = W.resnet110_partition(p=2, microbatch=2, num_microbatches=2)
    inp = W.make_inputs(spec)
    part = hpf.Partition(spec, inp.params)
    x = torch.zeros(part.in_shape, dtype=torch.bfloat16, device="cuda:0")
    e = torch.zeros(part.out_shape, dtype=torch.bfloat16, device="cuda:0")

    def status(fn, *a, **k):
        with pytest.raises(hpf.HpfError) as ei:
            fn(*a, **k)
        return ei.value.status

    assert status(part.backward_microbatch, 0, e) == hpf.HPF_ESTATE
    assert status(part.forward_microbatch, 2, x) == hpf.HPF_EINVAL
    part.forward_microbatch(0, x)
    assert status(part.forward_microbatch, 0, x) == hpf.HPF_ESTATE
    assert status(part.grad_accum_read) == hpf.HPF_ESTATE
    assert status(part.sgd_step, 0.1, 0.9) == hpf.HPF_ESTATE
    assert status(part.grad_accum_zero) == hpf.HPF_ESTATE
    part.backward_microbatch(0, e)
    assert status(part.backward_microbatch, 0, e) == hpf.HPF_ESTATE
    assert status(hpf.hpf_backward_microbatch, part.handle, 1, 0, 0) == hpf.HPF_EINVAL
    part.forward_microbatch(1, x)
    part.backward_microbatch(1, e)
    part.grad_accum_read()
    part.sgd_step(0.1, 0.9)
    part.forward_microbatch(0, x)                          # next batch may start
    torch.cuda.synchronize()
    part.close()


@pytest.mark.parametrize("fusion", [False, True])
def test_partition_chain_on_device_equals_unsplit_model(gpu, fusion):
    """The paper's premise on the GPU: ResNet-20 as 3 chained partitions == one partition.
    With the separate BN reduction kernels both runs add in the same order and agree to fp32 atomics;
    with the reductions fused into the conv epilogues the first BatchNorm of a partition (its input
    comes from the caller) sums in another order than inside the unsplit model, so the two runs are
    two bf16 evaluations of the same function (loss within 2e-3; see the parity criteria)."""
    import torch
    from parity import rel_err, run_gpu_step
    hpf = gpu
    whole = W.resnet20(microbatch=4, num_microbatches=2)
    inp = W.make_inputs(whole, randomize_affine=True)
    _, ref = run_gpu_step(whole, inp, "bf16", fusion=fusion)
    blocks = W.basic_resnet_blocks(3)
    specs = [W.partition_of(f"p{p}", blocks, 3, p, 32, 16, 16, 10, 4, 2, whole.seed) for p in range(3)]
    parts, off = [], 0
    for s in specs:
        n = W.n_params(s)
        parts.append(hpf.Partition(s, inp.params[off:off + n]))
        parts[-1].set_fusion(fusion)
        off += n
    dev = torch.device("cuda:0")
    keep = []            # act_in of every partition is read again by its backward call: keep it alive
    for i in range(2):
        x = torch.from_numpy(inp.act_in[i]).to(dev)
        lab = torch.from_numpy(inp.labels[i]).to(dev)
        for p, part in enumerate(parts):
            keep.append(x)
            x = part.forward_microbatch(i, x, lab if specs[p].has_head else None)
    for i in range(2):
        e = None
        for p in reversed(range(3)):
            e = parts[p].backward_microbatch(i, e)
    G = np.concatenate([p.grad_accum_read() for p in parts])
    torch.cuda.synchronize()
    if fusion:
        assert abs(parts[-1].loss.item() - ref["loss"]) <= 2e-3 * abs(ref["loss"])
    else:
        assert abs(parts[-1].loss.item() - ref["loss"]) <= 1e-6 * abs(ref["loss"])
        assert rel_err(G, ref["grad"]) < 1e-5
    for p in parts:
        p.close()
