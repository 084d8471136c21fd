"""GPU parity of partitions cut at layer granularity (paper Section "Special Handling for Non-consecutive
Models"): single cut partitions against the oracle on the same seeded inputs, and a whole model cut inside
its residual blocks, chained on the device through the rank-sorted message lists, against the unsplit oracle."""
import numpy as np
import pytest

import parity
from paper_1911_05146_amd import layer_cuts as LC
from paper_1911_05146_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: these tests need a real MI355X")
    from paper_1911_05146_amd import hpf
    return hpf


def run_gpu_cut_step(spec, inp, mode):
    import torch
    from paper_1911_05146_amd import hpf
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if mode == "bf16" else torch.float32
    rnd = parity.bf16_round if mode == "bf16" else (lambda a: a)
    seen = W.StepInputs(inp.params, [rnd(a) for a in inp.act_in], None, [rnd(e) for e in inp.err_in],
                        [rnd(a) for a in inp.skip_in] if inp.skip_in else None,
                        [rnd(a) for a in inp.skip_err_in] if inp.skip_err_in else None)
    up = lambda lst: [torch.from_numpy(a).to(dev, tdt) for a in lst] if lst else None
    act, err, sk, ske = up(seen.act_in), up(seen.err_in), up(seen.skip_in), up(seen.skip_err_in)
    part = hpf.Partition(spec, inp.params, hpf.HPF_BF16 if mode == "bf16" else hpf.HPF_F32)
    m = spec.num_microbatches
    outs, skips, errs, skerrs = [], [], [], []
    for i in range(m):
        o, so = part.forward_microbatch_cut(i, act[i], sk[i] if sk else None)
        outs.append(o); skips.append(so)
    for i in range(m):
        e, se = part.backward_microbatch_cut(i, err[i], ske[i] if ske else None)
        errs.append(e); skerrs.append(se)
    grad = part.grad_accum_read()
    torch.cuda.synchronize()
    host = lambda lst: [t.float().cpu().numpy() for t in lst if t is not None]
    res = {"act_out": host(outs), "err_out": host(errs), "loss": 0.0, "grad": grad}
    if spec.has_skip_out:
        res["skip_out"] = host(skips)
    if spec.has_skip_in:
        res["skip_err_out"] = host(skerrs)
    part.close()
    return seen, res


CUT_PARTITIONS = {
    # (blocks, in_hw, in_c, first_from, last_to)
    "tail_then_head_bottleneck": ((W.Block(W.BOTTLENECK, 64, 32, 128, 2), W.Block(W.BOTTLENECK, 128, 32, 128, 1)), 8, 32, 2, 2),
    "middle_piece_3x3": ((W.Block(W.BOTTLENECK, 128, 32, 128, 1),), 16, 32, 1, 2),
    "head_with_projection": ((W.Block(W.BOTTLENECK, 64, 32, 128, 2),), 16, 64, 0, 1),
    "head_identity_two_convs": ((W.Block(W.BOTTLENECK, 128, 32, 128, 1),), 16, 128, 0, 2),
    "tail_basic_then_whole_blocks": ((W.Block(W.BASIC, 16, 32, 32, 2), W.Block(W.BASIC, 32, 32, 32, 1), W.Block(W.BASIC, 32, 32, 32, 1)), 8, 32, 1, 0),
    "whole_blocks_then_head_basic": ((W.Block(W.BASIC, 32, 32, 32, 1), W.Block(W.BASIC, 32, 64, 64, 2)), 16, 32, 0, 1),
    "wide_tail_then_head": ((W.Block(W.BOTTLENECK, 256, 128, 512, 2), W.Block(W.BOTTLENECK, 512, 128, 512, 1)), 7, 128, 1, 2),
}


@pytest.mark.parametrize("mode", ["f32", "bf16"])
@pytest.mark.parametrize("case", sorted(CUT_PARTITIONS))
def test_cut_partition_against_oracle(gpu, oracle, case, mode):
    blocks, hw, in_c, ff, lt = CUT_PARTITIONS[case]
    spec = W.PartitionSpec(name=case, in_h=hw, in_w=hw, in_c=in_c, blocks=blocks, microbatch=3, num_microbatches=2,
                           seed=41, first_from=ff, last_to=lt)
    inp = W.make_inputs(spec, randomize_affine=True)
    print(f"[case] {case} {mode}", flush=True)
    seen, res = run_gpu_cut_step(spec, inp, mode)
    yard = oracle.run_step(spec, seen, np.float32, storage="bf16" if mode == "bf16" else "none")
    ref64 = lambda: oracle.run_step(spec, seen, np.float64)
    rep = parity.compare(spec, res, yard, mode, ref64=ref64, insensitive="skip")
    assert set(rep) >= {"act_out", "err_out", "grad"} | ({"skip_out"} if spec.has_skip_out else set()) | \
        ({"skip_err_out"} if spec.has_skip_in else set())
    print("[parity]", parity.fmt(rep), flush=True)


def test_cut_partitions_reject_the_plain_entry_points(gpu):
    import torch
    from paper_1911_05146_amd import hpf
    blocks, hw, in_c, ff, lt = CUT_PARTITIONS["tail_then_head_bottleneck"]
    spec = W.PartitionSpec(name="x", in_h=hw, in_w=hw, in_c=in_c, blocks=blocks, microbatch=2, num_microbatches=1,
                           first_from=ff, last_to=lt)
    part = hpf.Partition(spec, W.make_inputs(spec).params, hpf.HPF_BF16)
    x = torch.zeros(part.in_shape, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(hpf.HpfError) as e:
        part.forward_microbatch(0, x)
    assert e.value.status == hpf.HPF_EINVAL
    with pytest.raises(hpf.HpfError):       # skip_in missing
        hpf.hpf_forward_microbatch_cut(part.handle, 0, x.data_ptr(), 0, 0, x.data_ptr(), x.data_ptr(), 0, 0)
    part.close()


def small_model():
    return (W.bottleneck_resnet_blocks([2, 2], (16, 32), (64, 128), 16) +
            [W.Block(W.BASIC, 128, 128, 128, 1), W.Block(W.BASIC, 128, 64, 64, 2)])


@pytest.mark.parametrize("cuts", [[1, 2], list(range(1, 16)), [2, 4, 8, 13], [13, 15]], ids=["middle_piece", "every_layer", "tail_and_head", "basic_cut"])
def test_layer_cut_pipeline_on_device_equals_unsplit_model(gpu, oracle, cuts):
    """fp32 check mode: the chained, layer-cut model against the unsplit oracle, element by element."""
    import torch
    from paper_1911_05146_amd import hpf
    from paper_1911_05146_amd.pipeline import Pipeline
    cm = LC.split_at_layers("cutnet", small_model(), cuts, 16, 16, 10, 4, 3, 77)
    inp = W.make_inputs(cm.whole, randomize_affine=True)
    ref = oracle.run_step(cm.whole, inp, np.float32)
    dev = torch.device("cuda:0")
    pipe = Pipeline(cm.specs, inp.params, hpf.HPF_F32, cut_model=cm)
    act = [torch.from_numpy(a).to(dev) for a in inp.act_in]
    lab = [torch.from_numpy(l).to(dev) for l in inp.labels]
    pipe.run_batch(act, lab)
    G = pipe.grad_accum_read()
    loss = float(pipe.loss.item())
    pipe.close()
    assert abs(loss - ref["loss"]) <= 1e-4 * abs(ref["loss"])
    e = parity.rel_err(G, ref["grad"])
    print(f"[parity] layer-cut pipeline {len(cm.specs)} partitions: loss {loss:.6f} vs {ref['loss']:.6f}, grad max-norm {e:.2e}", flush=True)
    assert e <= 1e-4


def test_layer_cut_pipeline_bf16(gpu, oracle):
    import torch
    from paper_1911_05146_amd import hpf
    from paper_1911_05146_amd.pipeline import Pipeline
    cm = LC.split_at_layers("cutnet", small_model(), [1, 2, 5, 7, 10, 13], 16, 16, 10, 4, 2, 78)
    inp = W.make_inputs(cm.whole, randomize_affine=True)
    yard = oracle.run_step(cm.whole, inp, np.float32, storage="bf16")
    dev = torch.device("cuda:0")
    pipe = Pipeline(cm.specs, inp.params, hpf.HPF_BF16, cut_model=cm)
    act = [torch.from_numpy(a).to(dev) for a in inp.act_in]
    lab = [torch.from_numpy(l).to(dev) for l in inp.labels]
    pipe.run_batch(act, lab)
    res = {"grad": pipe.grad_accum_read(), "loss": float(pipe.loss.item())}
    pipe.close()
    rep = parity.compare(cm.whole, res, yard, "bf16", ref64=lambda: oracle.run_step(cm.whole, inp, np.float64), insensitive="skip")
    print("[parity]", parity.fmt(rep), flush=True)
