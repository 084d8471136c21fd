"""The BN+ReLU forward entry point that allocates nothing (its reduction partials live in an array built into
the library) against the workspace-taking entry point it is a variant of: same kernels, so the outputs must be
identical bit for bit (a fortiori within 2e-2 / 1e-4), on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["bf16", "f32"])
def test_no_alloc_bn_relu_forward_matches_the_workspace_entry_point(mode):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: this test needs a real MI355X")
    from paper_1911_05146_amd import hpf
    dev = torch.device("cuda:0")
    dt = hpf.HPF_BF16 if mode == "bf16" else hpf.HPF_F32
    tdt = torch.bfloat16 if mode == "bf16" else torch.float32
    sdt = torch.float32 if mode == "bf16" else torch.float64
    ops = hpf.Ops(dt)
    rng = np.random.default_rng(191105146 + 77)
    s = torch.cuda.current_stream(dev).cuda_stream
    for M, Cc in ((12544, 1024), (8192, 128), (333, 32), (7, 16)):   # large first: later calls find the array dirty
        x = torch.from_numpy(rng.standard_normal((M, Cc), dtype=np.float32) * 1.7 + 0.3).to(dev, tdt)
        gamma = torch.from_numpy(rng.uniform(0.5, 1.5, Cc).astype(np.float32)).to(dev)
        beta = torch.from_numpy(rng.normal(0, 0.3, Cc).astype(np.float32)).to(dev)
        a_ref, st_ref = ops.bn_relu_forward(x, gamma, beta)
        a = torch.full_like(x, float("nan"))
        st = torch.full((2 * Cc,), float("nan"), device=dev, dtype=sdt)
        hpf.hpf_op_bn_relu_forward_noalloc(dt, x.data_ptr(), gamma.data_ptr(), beta.data_ptr(), 1e-5, a.data_ptr(),
                                           st.data_ptr(), M, Cc, s)
        torch.cuda.synchronize()
        assert torch.equal(st, st_ref), (M, Cc)
        assert torch.equal(a, a_ref), (M, Cc)
        den = float(a_ref.float().abs().max())
        assert float((a.float() - a_ref.float()).abs().max()) <= (2e-2 if mode == "bf16" else 1e-4) * den
    # beyond the array's size: a clear error, nothing launched
    x = torch.zeros((4, 2048), device=dev, dtype=tdt)
    g = torch.ones(2048, device=dev)
    with pytest.raises(hpf.HpfError) as ei:
        hpf.hpf_op_bn_relu_forward_noalloc(dt, x.data_ptr(), g.data_ptr(), g.data_ptr(), 1e-5, x.data_ptr(), g.data_ptr(), 4, 2048, s)
    assert ei.value.status == hpf.HPF_EUNSUPPORTED and "1024" in str(ei.value)
