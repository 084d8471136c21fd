"""The error path of the image-resident launches, forced from the host: the "results invalid" flag that a launch
sets when it gives up waiting for its partner work-groups is written by a plain copy (no kernel times out), and
every blocking call must then report HPF_EDEVICE while the optimizer step leaves the parameters alone.  Also:
forward / backward calls on a stream the caller is capturing are refused at fusion level 2."""
import numpy as np
import pytest

from paper_1911_05146_amd import workloads as W

pytestmark = pytest.mark.gpu


def _part():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: these tests need a real MI355X")
    from paper_1911_05146_amd import hpf
    blk = W.Block(W.BOTTLENECK, 128, 32, 128, 1)
    spec = W.PartitionSpec(name="flag", in_h=8, in_w=8, in_c=128, blocks=(blk, blk), microbatch=4, num_microbatches=2, seed=3)
    inp = W.make_inputs(spec, randomize_affine=True)
    return hpf, spec, inp, hpf.Partition(spec, inp.params)


def _status(hpf, fn, *a, **k):
    with pytest.raises(hpf.HpfError) as ei:
        fn(*a, **k)
    return ei.value.status


def test_invalid_flag_is_reported_and_stops_the_step():
    import torch
    hpf, spec, inp, part = _part()
    x = [torch.from_numpy(a).to("cuda:0", torch.bfloat16) for a in inp.act_in]
    e = [torch.from_numpy(a).to("cuda:0", torch.bfloat16) for a in inp.err_in]
    part.forward_microbatches(0, x)
    part.backward_microbatches(0, 2, e)
    g0 = part.grad_accum_read()
    part.check()                                            # a healthy handle
    assert np.abs(g0).max() > 0
    hpf.hpf_debug_set_invalid(part.handle, 1)
    assert _status(hpf, part.check) == hpf.HPF_EDEVICE
    assert _status(hpf, part.grad_accum_read) == hpf.HPF_EDEVICE
    assert _status(hpf, part.params_read) == hpf.HPF_EDEVICE
    assert _status(hpf, part.bn_running_read) == hpf.HPF_EDEVICE
    assert _status(hpf, part.stash_read, 0, 0, hpf.HPF_T_C1) == hpf.HPF_EDEVICE
    part.sgd_step(0.1, 0.9)                                 # enqueues only; on the device it must change nothing
    assert _status(hpf, part.check) == hpf.HPF_EDEVICE      # sticky
    hpf.hpf_debug_set_invalid(part.handle, 0)
    part.check()
    assert np.array_equal(part.params_read(), inp.params)   # the step was skipped
    part.forward_microbatches(0, x)                         # the step still started the next batch on the host side
    part.backward_microbatches(0, 2, e)
    g1 = part.grad_accum_read()
    assert np.allclose(g1, 2 * g0, rtol=1e-4, atol=1e-6 * np.abs(g0).max())   # ... and had not cleared the gradients
    part.close()


def test_calls_on_a_capturing_stream_are_refused_at_level_2():
    import torch
    hpf, spec, inp, part = _part()
    x = [torch.from_numpy(a).to("cuda:0", torch.bfloat16) for a in inp.act_in]
    out = [torch.empty(part.out_shape, dtype=torch.bfloat16, device="cuda:0") for _ in x]
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        g.capture_begin()
        try:
            st = _status(hpf, part.forward_microbatches, 0, x, None, out, stream=s)
        finally:
            g.capture_end()
    assert st == hpf.HPF_EUNSUPPORTED
    torch.cuda.synchronize()
    part.forward_microbatches(0, x, None, out, stream=s)    # outside a capture the same call runs
    part.check()
    part.close()
