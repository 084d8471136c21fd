"""The paper's pipelined model parallelism on one GPU: a model cut into partitions, each on its own stream,
micro-batches flowing through them, must give the loss and the gradients of the unsplit model (paper Section
"Verifying the Correctness of HyPar-Flow" states this premise for the sequential vs the model-parallel run)."""
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


def _run(oracle, name, blocks, n_parts, in_hw, stem_c, b, m, seed, group, fusion=None, sgd=None, mode="bf16", strict=False):
    import torch
    from parity import compare, fmt
    from paper_1911_05146_amd.pipeline import Pipeline, split_model
    from test_gpu_parity import to64
    whole = W.partition_of(name, list(blocks), 1, 0, in_hw, blocks[0].c_in, stem_c, 10, b, m, seed)
    specs = split_model(name, blocks, n_parts, in_hw, stem_c, 10, b, m, seed)
    assert sum(W.n_params(s) for s in specs) == W.n_params(whole)
    inp = W.make_inputs(whole, randomize_affine=True)
    print(f"\n[case] pipeline {name}: {n_parts} partitions, b={b} m={m} group={group} fusion={fusion}", flush=True)
    dev = torch.device("cuda:0")
    x = [torch.from_numpy(a).to(dev) for a in inp.act_in]
    lab = [torch.from_numpy(l).to(dev) for l in inp.labels]
    from paper_1911_05146_amd import hpf
    pipe = Pipeline(specs, inp.params, hpf.HPF_BF16 if mode == "bf16" else hpf.HPF_F32, group=group, fusion=fusion)
    pipe.run_batch(x, lab)
    res = {"act_out": [], "err_out": [], "grad": pipe.grad_accum_read(), "loss": float(pipe.loss.item())}
    if sgd:
        pipe.sgd_step(*sgd)
        res["params"] = pipe.params_read()
    pipe.close()
    yard = oracle.run_step(whole, inp, np.float32, sgd=sgd, storage="bf16" if mode == "bf16" else "none")
    rep = compare(whole, res, yard, mode, ref64=lambda: oracle.run_step(whole, to64(inp), np.float64, sgd=sgd), strict=strict, insensitive="skip")
    print(f"[parity] pipeline {name}: " + fmt(rep), flush=True)
    return res


def test_resnet20_in_three_partitions(gpu, oracle):
    blocks = W.basic_resnet_blocks(3)
    a = _run(oracle, "resnet20", blocks, 3, 32, 16, 4, 4, 77, group=1, sgd=(0.1, 0.9))
    b = _run(oracle, "resnet20", blocks, 3, 32, 16, 4, 4, 77, group=2)
    # the grouping of the calls changes launches, not arithmetic
    assert abs(a["loss"] - b["loss"]) <= 1e-5 * abs(a["loss"])
    # fp32 check mode: the pipelined, partitioned run equals the unsplit oracle element by element
    _run(oracle, "resnet20", blocks, 3, 32, 16, 4, 4, 77, group=1, sgd=(0.1, 0.9), mode="f32", strict=True)


def test_bottleneck_model_in_two_and_four_partitions(gpu, oracle):
    """Stem, a 128-channel stage at 16x16 and a 256-channel stage at 8x8 (both with image-resident runs),
    head: every cut position lands inside or between runs."""
    blocks = W.bottleneck_resnet_blocks(4, (32, 64), (128, 256), 64)
    for n_parts, group in ((2, 1), (4, 2), (3, 4)):
        _run(oracle, "bottleneck-2stage", blocks, n_parts, 16, 64, 4, 4, 78, group=group)
    _run(oracle, "bottleneck-2stage-level1", blocks, 2, 16, 64, 4, 4, 78, group=1, fusion=1)
