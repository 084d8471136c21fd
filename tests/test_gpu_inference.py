"""GPU parity of the BatchNorm running statistics and the inference forward against the oracle (the paper
reports test accuracy of the trained models -- Section "Verifying the Correctness of HyPar-Flow" -- which needs
BatchNorm's inference form; reading: moving averages of the micro-batch statistics, biased variance)."""
import numpy as np
import pytest

import parity
from paper_1911_05146_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: these tests need a real MI355X")
    from paper_1911_05146_amd import hpf
    return hpf


def small_specs():
    r20 = W.resnet20(microbatch=4, num_microbatches=2)                                    # stem, basic runs, head
    bott = W.PartitionSpec(name="bott", in_h=16, in_w=16, in_c=64,                          # projection + resident run
                           blocks=(W.Block(W.BOTTLENECK, 64, 32, 128, 1),) + (W.Block(W.BOTTLENECK, 128, 32, 128, 1),) * 3,
                           microbatch=4, num_microbatches=2, seed=9)
    cut = W.PartitionSpec(name="cut", in_h=8, in_w=8, in_c=32,                              # tail of one block, head of the next
                          blocks=(W.Block(W.BOTTLENECK, 64, 32, 128, 2), W.Block(W.BOTTLENECK, 128, 32, 128, 1)),
                          microbatch=3, num_microbatches=2, seed=10, first_from=2, last_to=2)
    wide = W.PartitionSpec(name="wide", in_h=16, in_w=16, in_c=128,                        # resident runs of the two other shapes
                           blocks=(W.Block(W.BOTTLENECK, 128, 64, 128, 1),) * 2 + (W.Block(W.BOTTLENECK, 128, 64, 256, 2),) +
                                  (W.Block(W.BOTTLENECK, 256, 64, 256, 1),) * 2,
                           microbatch=3, num_microbatches=2, seed=11)
    return {"resnet20": r20, "bottleneck_run": bott, "cut_partition": cut, "wide_runs": wide}


def train_batch(part, spec, t, grouped):
    m = spec.num_microbatches
    if grouped and not (spec.has_skip_in or spec.has_skip_out):
        part.forward_microbatches(0, t["act_in"], t["labels"])
        part.backward_microbatches(0, m, t["err_in"])
    else:
        for i in range(m):
            part.forward_microbatch_cut(i, t["act_in"][i], t["skip_in"][i] if t["skip_in"] else None,
                                        t["labels"][i] if t["labels"] else None)
        for i in range(m):
            part.backward_microbatch_cut(i, t["err_in"][i] if t["err_in"] else None,
                                         t["skip_err_in"][i] if t["skip_err_in"] else None)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
@pytest.mark.parametrize("grouped", [False, True])
@pytest.mark.parametrize("name", ["resnet20", "bottleneck_run", "cut_partition", "wide_runs"])
def test_running_statistics_and_inference_against_oracle(gpu, oracle, name, grouped, mode):
    import torch
    hpf = gpu
    spec = small_specs()[name]
    inp = W.make_inputs(spec, randomize_affine=True)
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if mode == "bf16" else torch.float32
    rnd = parity.bf16_round if mode == "bf16" else (lambda a: a)
    act = [a if spec.has_stem else rnd(a) for a in inp.act_in]
    err = [rnd(e) for e in inp.err_in] if inp.err_in else None
    sk = [rnd(a) for a in inp.skip_in] if inp.skip_in else None
    ske = [rnd(a) for a in inp.skip_err_in] if inp.skip_err_in else None
    up = lambda lst, dt=tdt: [torch.from_numpy(a).to(dev, dt) for a in lst] if lst else None
    t = {"act_in": up(act, torch.float32 if spec.has_stem else tdt), "labels": up(inp.labels, torch.int32),
         "err_in": up(err), "skip_in": up(sk), "skip_err_in": up(ske)}
    print(f"[case] {name} grouped={grouped} {mode}", flush=True)

    part = hpf.Partition(spec, inp.params, hpf.HPF_BF16 if mode == "bf16" else hpf.HPF_F32)
    opart = oracle.OraclePartition(spec, inp.params, np.float32, storage="bf16" if mode == "bf16" else "none")
    mom = 0.8
    part.set_bn_momentum(mom)
    opart.set_bn_momentum(mom)
    for _ in range(2):                                        # two batches of training forwards move the statistics
        train_batch(part, spec, t, grouped)
        part.grad_accum_zero()
        for i in range(spec.num_microbatches):
            opart.forward(i, act[i], inp.labels[i] if inp.labels else None, skip_in=sk[i] if sk else None)
        for i in range(spec.num_microbatches):
            opart.backward(i, err[i] if err else None, want_err_out=not spec.has_stem, skip_err_in=ske[i] if ske else None)
        opart.zero_grad()
    r_gpu, r_ref = part.bn_running_read().astype(np.float64), opart.bn_running()
    assert r_gpu.size == r_ref.size == int(part.sizes.n_bn_running) > 0
    e = parity.rel_err(r_gpu, r_ref)
    tol = 2e-2 if mode == "bf16" else 1e-4
    assert e <= tol, f"running statistics: {e:.2e}"

    # inference with the oracle's running statistics on both sides
    part.bn_running_write(r_ref)
    x = t["act_in"][1]
    got = part.forward_inference(x, t["skip_in"][1] if t["skip_in"] else None)
    ref = opart.infer(act[1], sk[1] if sk else None)
    torch.cuda.synchronize()
    gl = got if isinstance(got, tuple) else (got,)
    rl = ref if isinstance(ref, tuple) else (ref,)
    errs = [parity.rel_err(g.float().cpu().numpy(), r) for g, r in zip(gl, rl)]
    print(f"[parity] running statistics {e:.2e}; inference outputs {['%.2e' % v for v in errs]}", flush=True)
    assert len(gl) == len(rl) and max(errs) <= tol
    # the group call gives what the single calls give (twice: the second call replays the captured launches)
    outs = None
    for _ in range(2):
        grp = part.forward_inference_group(t["act_in"], t["skip_in"], out=outs)
        outs = [g[0] if isinstance(g, tuple) else g for g in grp]
        torch.cuda.synchronize()
        g1 = grp[1][0] if isinstance(grp[1], tuple) else grp[1]
        assert torch.equal(g1, gl[0])
    part.close()
    opart.close()


def test_inference_between_batches_leaves_training_untouched(gpu):
    import torch
    hpf = gpu
    spec = small_specs()["resnet20"]
    inp = W.make_inputs(spec, randomize_affine=True)
    dev = torch.device("cuda:0")
    x = [torch.from_numpy(a).to(dev) for a in inp.act_in]
    lab = [torch.from_numpy(l).to(dev) for l in inp.labels]
    grads = []
    for with_inference in (False, True):
        part = hpf.Partition(spec, inp.params, hpf.HPF_F32)
        part.forward_microbatches(0, x, lab)
        part.backward_microbatches(0, spec.num_microbatches)
        part.sgd_step(0.1, 0.9)
        if with_inference:
            logits = part.forward_inference(x[0])
            assert tuple(logits.shape) == (spec.microbatch, spec.num_classes) and torch.isfinite(logits).all()
        part.forward_microbatches(0, x, lab)
        if with_inference:                                     # a micro-batch is between forward and backward
            with pytest.raises(hpf.HpfError) as e:
                part.forward_inference(x[0])
            assert e.value.status == hpf.HPF_ESTATE
        part.backward_microbatches(0, spec.num_microbatches)
        grads.append(part.grad_accum_read())
        part.close()
    # equal up to the order of the fp32 atomic adds into the gradient buffer
    assert parity.rel_err(grads[1], grads[0]) <= 1e-5


def test_momentum_one_and_frozen_mode_never_touch_the_running_statistics(gpu):
    import torch
    hpf = gpu
    for kw, mom in ((dict(), 1.0), (dict(bn_mode=1), 0.5)):
        spec = W.resnet20(microbatch=2, num_microbatches=2)
        spec = W.with_microbatching(spec, 2, 2, **kw)
        inp = W.make_inputs(spec)
        part = hpf.Partition(spec, inp.params, hpf.HPF_BF16)
        part.set_bn_momentum(mom)
        r0 = part.bn_running_read()
        x = [torch.from_numpy(a).to("cuda:0") for a in inp.act_in]
        lab = [torch.from_numpy(l).to("cuda:0") for l in inp.labels]
        part.forward_microbatches(0, x, lab)
        part.backward_microbatches(0, 2)
        assert np.array_equal(part.bn_running_read(), r0)
        with pytest.raises(hpf.HpfError):
            part.set_bn_momentum(1.5)
        with pytest.raises(hpf.HpfError):
            part.bn_running_write(-np.ones_like(r0))
        part.close()


def test_running_statistics_with_one_stream_per_microbatch(gpu, oracle):
    """Forward calls on different streams are chained by the library while they move the running statistics:
    the result is that of the calls in call order."""
    import torch
    hpf = gpu
    spec = small_specs()["bottleneck_run"]
    inp = W.make_inputs(spec, randomize_affine=True)
    dev = torch.device("cuda:0")
    act = [parity.bf16_round(a) for a in inp.act_in]
    x = [torch.from_numpy(a).to(dev, torch.bfloat16) for a in act]
    e = [torch.from_numpy(parity.bf16_round(a)).to(dev, torch.bfloat16) for a in inp.err_in]
    part = hpf.Partition(spec, inp.params, hpf.HPF_BF16)
    opart = oracle.OraclePartition(spec, inp.params, np.float32, storage="bf16")
    part.set_bn_momentum(0.5)
    opart.set_bn_momentum(0.5)
    streams = [torch.cuda.Stream() for _ in x]
    torch.cuda.synchronize()
    for i, s in enumerate(streams):
        part.forward_microbatch(i, x[i], stream=s)
    for i, s in enumerate(streams):
        part.backward_microbatch(i, e[i], stream=s)
    for i in range(spec.num_microbatches):
        opart.forward(i, act[i])
    err = parity.rel_err(part.bn_running_read().astype(np.float64), opart.bn_running())
    print(f"[parity] running statistics over streams {err:.2e}", flush=True)
    assert err <= 2e-2
    part.close()
    opart.close()


def test_inference_group_larger_than_the_chip(gpu, oracle):
    """8 micro-batches of 48 images in one inference call: 384 work-groups of the image-resident kernel on 256
    CUs.  The images are independent at inference, so the work-groups simply queue (a training launch of that size
    is split); the group call equals the single calls, and one micro-batch is checked against the oracle."""
    import torch
    hpf = gpu
    blk = W.Block(W.BOTTLENECK, 128, 32, 128, 1)
    spec = W.PartitionSpec(name="infer-large-group", in_h=8, in_w=8, in_c=128, blocks=(blk,) * 3, microbatch=48,
                           num_microbatches=8, seed=12)
    inp = W.make_inputs(spec, randomize_affine=True)
    dev = torch.device("cuda:0")
    act = [parity.bf16_round(a) for a in inp.act_in]
    xs = [torch.from_numpy(a).to(dev, torch.bfloat16) for a in act]
    part = hpf.Partition(spec, inp.params, hpf.HPF_BF16)
    opart = oracle.OraclePartition(spec, inp.params, np.float32, storage="bf16")
    rng = np.random.default_rng(5)
    run = rng.uniform(0.5, 1.5, opart.bn_running().size)                             # means and variances in [0.5, 1.5]
    opart.set_bn_running(run)
    part.bn_running_write(run)
    grp = part.forward_inference_group(xs, None)
    torch.cuda.synchronize()
    for i in (0, 5, 7):
        single = part.forward_inference(xs[i], None)
        torch.cuda.synchronize()
        assert torch.equal(single, grp[i])
    ref = opart.infer(act[5], None)
    e = parity.rel_err(grp[5].float().cpu().numpy(), ref)
    print(f"[parity] inference output {e:.2e}", flush=True)
    assert e <= 2e-2
    part.close()
    opart.close()
