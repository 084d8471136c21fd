"""GPU parity for the paper's two other models (Section "Model-Parallelism on a Single Node"): the post-activation
ResNet-110-v1 and VGG-16, as single partitions and as pipelines of partitions on one GPU (VGG-16 in 8 partitions is
the paper's best split).  fp32 check mode: element-wise 1e-4 against the plain oracle; bf16: 2e-2 where the
arithmetic allows it, else the sensitivity-limited criterion of parity.compare."""
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


def check(oracle, spec, mode, strict=False, sgd=None, grouped=False):
    from parity import compare, fmt, run_gpu_step
    print(f"\n[case] {spec.name} b={spec.microbatch} m={spec.num_microbatches} mode={mode} grouped={grouped}", flush=True)
    inp = W.make_inputs(spec, randomize_affine=True)
    seen, res = run_gpu_step(spec, inp, mode, sgd=sgd, grouped=grouped)
    yard = oracle.run_step(spec, seen, np.float32, sgd=sgd, storage="bf16" if mode == "bf16" else "none")
    rep = compare(spec, res, yard, mode, ref64=lambda: oracle.run_step(spec, to64(seen), np.float64, sgd=sgd), strict=strict,
                  insensitive="skip")
    print(f"[parity] {spec.name} {mode}: " + fmt(rep), flush=True)
    return rep


def unit(name, blocks, hw, c, b=4, m=2, seed=61, **kw):
    return W.PartitionSpec(name=name, in_h=hw, in_w=hw, in_c=c, blocks=tuple(blocks), microbatch=b, num_microbatches=m, seed=seed, **kw)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_units_of_both_models(gpu, oracle, mode):
    cases = [
        unit("postact-identity", [W.Block(W.POSTACT, 32, 32, 32, 1)], 16, 32),
        unit("postact-stride2-proj", [W.Block(W.POSTACT, 16, 32, 32, 2)], 32, 16),
        unit("postact-pair", [W.Block(W.POSTACT, 32, 64, 64, 2), W.Block(W.POSTACT, 64, 64, 64, 1)], 16, 32),
        unit("conv-relu", [W.Block(W.CONV_RELU, 64, 64, 64, 1)], 16, 64),
        unit("conv-relu-pool", [W.Block(W.CONV_RELU, 64, 128, 128, 2)], 16, 64),
        unit("conv-relu-pool-2x2-image", [W.Block(W.CONV_RELU, 512, 512, 512, 2)], 2, 512, b=16),
        unit("dense-relu-dense", [W.Block(W.DENSE, 512, 1, 256, 1), W.Block(W.DENSE, 256, 0, 64, 1)], 1, 512, b=16),
        unit("dense-on-2x2", [W.Block(W.DENSE, 64, 1, 128, 1)], 2, 64, b=5),
        unit("bn-relu-unit", [W.Block(W.BN_RELU, 16, 16, 16, 1)], 32, 16),
        unit("bias-relu-unit", [W.Block(W.BIAS_RELU, 64, 64, 64, 1)], 32, 64),
        unit("plain-head", [W.Block(W.DENSE, 512, 1, 128, 1)], 1, 512, b=16, has_head=True, num_classes=10, head_bn=False),
    ]
    for spec in cases:
        check(oracle, spec, mode, strict=(mode == "f32"))
        check(oracle, spec, mode, strict=(mode == "f32"), grouped=True)
        layerwise(oracle, spec, mode)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_small_models_with_sgd(gpu, oracle, mode):
    check(oracle, W.resnet110_v1(microbatch=4, num_microbatches=2, n_per_stage=2), mode, strict=(mode == "f32"), sgd=(0.1, 0.9))
    check(oracle, W.vgg16(microbatch=4, num_microbatches=2, widths=(16, 32, 32, 64, 64), dense=(128, 128)), mode,
          strict=(mode == "f32"), sgd=(0.1, 0.9))


def layerwise(oracle, spec, mode, grouped=True):
    """Every layer on its own from the device's stored input of that layer (tests/teacher.py): element-wise."""
    from teacher import run_and_check
    print(f"\n[case] layer-wise {spec.name} b={spec.microbatch} m={spec.num_microbatches} mode={mode} grouped={grouped}", flush=True)
    return run_and_check(oracle, spec, mode, grouped=grouped, blockwise=False)


def test_resnet110_v1_full_size(gpu, oracle):
    """54 post-activation blocks, 8 micro-batches of 16 images of 32x32x3: end to end (the deep backward pass is
    sensitivity-limited in bf16) and layer by layer (element-wise)."""
    check(oracle, W.resnet110_v1(), "bf16", grouped=True)
    layerwise(oracle, W.resnet110_v1(), "bf16")
    check(oracle, W.resnet110_v1(microbatch=4, num_microbatches=2), "f32", strict=True)
    layerwise(oracle, W.resnet110_v1(microbatch=4, num_microbatches=2), "f32", grouped=False)


def test_vgg16_full_size(gpu, oracle):
    """13 convolutions, 5 max-pools, two dense layers of 4096 and the classifier; 8 micro-batches of 16 images."""
    check(oracle, W.vgg16(), "bf16", grouped=True)
    layerwise(oracle, W.vgg16(), "bf16")
    check(oracle, W.vgg16(microbatch=4, num_microbatches=2), "f32", strict=True)
    layerwise(oracle, W.vgg16(microbatch=4, num_microbatches=2), "f32", grouped=False)


def test_micro_batches_on_their_own_streams_plain_units(gpu, oracle):
    """Calls for different micro-batches may overlap on different streams: everything they write besides their own
    regions must be either per micro-batch (the partial sums of the split reductions) or added atomically (the weight
    gradients).  Eight micro-batches of plain 512-channel units on 4x4 pixels, several batches in a row."""
    from parity import rel_err, run_gpu_step
    blocks = tuple(W.Block(W.CONV_RELU, 512, 512, 512, 1) for _ in range(3))
    spec = W.PartitionSpec(name="plain-512@4x4-streams", in_h=4, in_w=4, in_c=512, blocks=blocks, microbatch=8,
                           num_microbatches=8, seed=67)
    inp = W.make_inputs(spec)
    _, a = run_gpu_step(spec, inp, "bf16", multi_stream=False)
    for _ in range(3):
        _, b = run_gpu_step(spec, inp, "bf16", multi_stream=True)
        for x, y in zip(a["act_out"] + a["err_out"], b["act_out"] + b["err_out"]):
            assert np.array_equal(x, y)                  # activations and errors: fixed summation order, no atomics
        assert rel_err(b["grad"], a["grad"]) < 1e-5      # gradient sums: fp32 atomics, order may differ


@pytest.mark.parametrize("model,n_parts", [("vgg16", 8), ("resnet110v1", 4)])
def test_pipelines_of_partitions_equal_the_unsplit_model(gpu, oracle, model, n_parts):
    """The paper's premise on the GPU for both models: cut into partitions (VGG-16 in 8: the paper's best split),
    each on its own stream, micro-batches flowing through, against the UNSPLIT oracle; fp32 check mode,
    element-wise."""
    import torch
    from parity import compare, fmt
    from paper_1911_05146_amd import hpf
    from paper_1911_05146_amd.pipeline import Pipeline
    b, m = 4, 4
    mk = (lambda n, p: W.vgg16(n, p, microbatch=b, num_microbatches=m)) if model == "vgg16" else \
         (lambda n, p: W.resnet110_v1(n, p, microbatch=b, num_microbatches=m, n_per_stage=6))
    whole, specs = mk(1, 0), [mk(n_parts, p) for p in range(n_parts)]
    assert sum(W.n_params(s) for s in specs) == W.n_params(whole)
    inp = W.make_inputs(whole, randomize_affine=True)
    dev = torch.device("cuda:0")
    x = [torch.from_numpy(a).to(dev) for a in inp.act_in]
    lab = [torch.from_numpy(l).to(dev) for l in inp.labels]
    for mode in ("f32", "bf16"):
        print(f"\n[case] pipeline {whole.name}: {n_parts} partitions, b={b} m={m} mode={mode}", flush=True)
        pipe = Pipeline(specs, inp.params, hpf.HPF_F32 if mode == "f32" else hpf.HPF_BF16, group=1)
        pipe.run_batch(x, lab)
        res = {"act_out": [], "err_out": [], "grad": pipe.grad_accum_read(), "loss": float(pipe.loss.item())}
        pipe.sgd_step(0.1, 0.9)
        res["params"] = pipe.params_read()
        pipe.close()
        yard = oracle.run_step(whole, inp, np.float32, sgd=(0.1, 0.9), storage="bf16" if mode == "bf16" else "none")
        rep = compare(whole, res, yard, mode, ref64=lambda: oracle.run_step(whole, to64(inp), np.float64, sgd=(0.1, 0.9)),
                      strict=(mode == "f32"), insensitive="skip")
        print(f"[parity] pipeline {whole.name} {mode}: " + fmt(rep), flush=True)
