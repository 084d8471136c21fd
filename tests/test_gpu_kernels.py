"""GPU parity of the single kernels (through the C ABI's hpf_op_* entry points) against the CPU
oracle's single operations, on seeded inputs: shapes of the benchmark partitions plus ragged and
strided cases.  Both sides get the same bf16-rounded inputs in bf16 mode."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "f32": 1e-4}


@pytest.fixture(scope="module")
def env():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: these tests need a real MI355X")
    from paper_1911_05146_amd import hpf
    return hpf, torch


def ops_for(hpf, mode):
    return hpf.Ops(hpf.HPF_BF16 if mode == "bf16" else hpf.HPF_F32)


def to_dev(torch, a, mode):
    t = torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()
    return t.to(torch.bfloat16) if mode == "bf16" else t


def seen(torch, a, mode):
    """The values the device tensor holds, as float32 numpy."""
    return to_dev(torch, a, mode).float().cpu().numpy()


def rel(got, ref):
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / np.abs(ref).max())


CONV_SHAPES = [
    # b, h, w, cin, cout, R, stride
    (4, 16, 16, 128, 32, 1, 1),      # ResNet-1001 stage-2 bottleneck conv1
    (4, 16, 16, 32, 32, 3, 1),       # conv2
    (4, 16, 16, 32, 128, 1, 1),      # conv3
    (2, 32, 32, 16, 16, 3, 1),       # stage 1, 16 channels
    (2, 32, 32, 64, 16, 1, 1),
    (2, 32, 32, 16, 64, 1, 1),
    (3, 16, 16, 32, 64, 3, 2),       # ResNet-110 stage entry, stride 2
    (3, 16, 16, 32, 64, 1, 2),       # its projection
    (2, 28, 28, 512, 256, 1, 2),     # ResNet-152 stage-3 entry
    (3, 14, 14, 256, 256, 3, 1),     # 588 rows: ragged tile
    (1, 14, 14, 256, 1024, 1, 1),    # wide channel tile
    (1, 8, 8, 64, 64, 3, 1),
    # wide tensors (8-wave 128x128x64 kernels): step counts 16, 18, 9, 7, 11 exercise every tail of the unrolled loop
    (2, 14, 14, 1024, 256, 1, 1),    # ResNet-152 stage-3 conv1: 16 steps; data gradient 4 steps into 1024 channels
    (1, 28, 28, 128, 128, 3, 2),     # 3x3 stride 2 on the wide kernel: 18 steps, stride holes in the data gradient
    (5, 7, 7, 64, 128, 3, 1),        # 9 steps, 245 rows (ragged second tile)
    (1, 8, 8, 448, 128, 1, 1),       # 7 steps
    (1, 8, 8, 704, 128, 1, 1),       # 11 steps
]


@pytest.mark.parametrize("mode", ["f32", "bf16"])
@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_forward_dgrad_wgrad(env, oracle, mode, shape):
    hpf, torch = env
    b, h, w, cin, cout, R, stride = shape
    print(f"\n[case] conv {shape} {mode}", flush=True)
    rng = np.random.default_rng(hash(shape) % (2 ** 31))
    x = rng.standard_normal((b, h, w, cin), dtype=np.float32)
    wt = (rng.standard_normal((R, R, cin, cout), dtype=np.float32) * np.sqrt(2.0 / (R * R * cin))).astype(np.float32)
    dy = 0.1 * rng.standard_normal((b, h // stride, w // stride, cout), dtype=np.float32)
    res = rng.standard_normal(dy.shape, dtype=np.float32)
    ops = ops_for(hpf, mode)
    xd, dyd, resd = to_dev(torch, x, mode), to_dev(torch, dy, mode), to_dev(torch, res, mode)
    wd = torch.from_numpy(wt).cuda()
    xs, dys, ress = seen(torch, x, mode), seen(torch, dy, mode), seen(torch, res, mode)
    ws = seen(torch, wt, mode)                       # the MFMA path rounds the weights to bf16
    tol = TOL[mode]

    y = ops.conv_forward(xd, wd, stride).float().cpu().numpy()
    e = rel(y, oracle.conv_fwd(xs, ws, stride).astype(np.float64))
    y2 = ops.conv_forward(xd, wd, stride, add=resd).float().cpu().numpy()
    e2 = rel(y2, oracle.conv_fwd(xs, ws, stride).astype(np.float64) + ress)
    dx = ops.conv_dgrad(dyd, wd, (h, w), stride).float().cpu().numpy()
    e3 = rel(dx, oracle.conv_dgrad(dys, ws, (h, w), stride).astype(np.float64))
    dw = ops.conv_wgrad(xd, dyd, R, stride)
    dw = ops.conv_wgrad(xd, dyd, R, stride, out=dw).cpu().numpy()     # second call accumulates
    e4 = rel(dw, 2 * oracle.conv_wgrad(xs, dys, R, stride))
    print(f"[parity] fwd {e:.2e} fwd+add {e2:.2e} dgrad {e3:.2e} wgrad {e4:.2e}", flush=True)
    assert max(e, e2, e3) <= tol and e4 <= (1e-5 if mode == "f32" else 1e-3)


BN_SHAPES = [(8192, 128), (8192, 32), (1024, 64), (588, 256), (3136, 1024), (12544, 512), (100, 48), (7, 16)]


@pytest.mark.parametrize("mode", ["f32", "bf16"])
@pytest.mark.parametrize("shape", BN_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_bn_relu_forward_backward(env, oracle, mode, shape):
    hpf, torch = env
    M, C = shape
    print(f"\n[case] bn {shape} {mode}", flush=True)
    rng = np.random.default_rng(M * 131 + C)
    x = (rng.standard_normal((M, C), dtype=np.float32) * rng.uniform(0.5, 3.0, C).astype(np.float32)
         + rng.uniform(-4, 4, C).astype(np.float32))           # per-channel scale and a large offset
    gamma = rng.uniform(0.5, 1.5, C).astype(np.float32)
    beta = (0.3 * rng.standard_normal(C)).astype(np.float32)
    da = rng.standard_normal((M, C), dtype=np.float32)
    skip = rng.standard_normal((M, C), dtype=np.float32)
    ops = ops_for(hpf, mode)
    xd, dad, skd = to_dev(torch, x, mode), to_dev(torch, da, mode), to_dev(torch, skip, mode)
    gd, bd = torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
    xs, das, sks = seen(torch, x, mode), seen(torch, da, mode), seen(torch, skip, mode)
    a, stats = ops.bn_relu_forward(xd, gd, bd)
    ra, rmean, rinv = oracle.bn_relu_fwd(xs, gamma, beta)
    stats_dev = stats
    stats = stats.cpu().numpy().astype(np.float64)
    e_mean = np.abs(stats[:C] - rmean).max() / np.abs(rmean).max()
    e_inv = np.abs(stats[C:] / rinv - 1).max()
    e_a = rel(a.float().cpu().numpy(), ra.astype(np.float64))
    dx, dg, db = ops.bn_relu_backward(xd, dad, gd, bd, stats_dev, skip=skd)
    rdx, rdg, rdb = oracle.bn_relu_bwd(xs, das, gamma, beta, rmean, rinv)
    # The ReLU decision z > 0 is taken in fp32 on the device and in double in the reference: where
    # |z| is within fp32 rounding of 0 the two may differ.  Those elements are left out of the
    # element-wise comparison and bound the slack allowed on the two reductions.
    z = gamma * ((xs.astype(np.float64) - rmean) * rinv) + beta
    tie = np.abs(z) < 1e-5
    slack = (np.abs(das) * tie).sum(0).max()
    gdx = dx.float().cpu().numpy().astype(np.float64)
    rfull = rdx.astype(np.float64) + sks
    e_dx = float(np.abs((gdx - rfull) * ~tie).max() / np.abs(rfull).max())
    e_dg = float((np.abs(dg.cpu().numpy() - rdg).max() - 4 * slack) / np.abs(rdg).max())
    e_db = float((np.abs(db.cpu().numpy() - rdb).max() - slack) / np.abs(rdb).max())
    print(f"[parity] mean {e_mean:.2e} invstd {e_inv:.2e} a {e_a:.2e} dx {e_dx:.2e} dgamma {e_dg:.2e} dbeta {e_db:.2e}", flush=True)
    assert e_mean < 1e-5 and e_inv < 1e-5
    tol = TOL[mode]
    assert e_a <= tol and e_dx <= tol and e_dg <= tol and e_db <= tol


# ---------------------------------------------------------------------------------------------
# the two measurement aids: results are checked, rates are bench.py's business
# ---------------------------------------------------------------------------------------------
def test_probe_copy_copies_and_rejects_overlap(env):
    hpf, torch = env
    n = (1 << 20) + 13                                   # ragged tail behind the 16-byte units
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n + 16, dtype=torch.uint8, device="cuda")
    hpf.hpf_probe_copy(dst.data_ptr(), src.data_ptr(), n)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and int(dst[n:].sum()) == 0
    with pytest.raises(hpf.HpfError):
        hpf.hpf_probe_copy(src.data_ptr() + 16, src.data_ptr(), 64)


@pytest.mark.parametrize("wide", [False, True], ids=["16x16x32", "32x32x16"])
def test_probe_mfma_loop_computes_the_product_it_claims(env, wide):
    """The register-only MFMA loops: every lane's result against the product of the operands the kernel builds.
    16x16x32: lane l feeds row / column l%16 with k = 8*(l/16)..+7 and holds rows 4*(l/16)..+3 of column l%16;
    32x32x16: lane l feeds row / column l%32 with k = 8*(l/32)..+7 and holds rows 8g + 4*(l/32) + v (g, v < 4)."""
    hpf, torch = env
    wgs, iters = 3, 3
    sink = torch.full((wgs * 256,), float("nan"), dtype=torch.float32, device="cuda")
    flops = hpf.hpf_probe_mfma_bf16(sink.data_ptr(), wgs, iters, wide)
    torch.cuda.synchronize()
    assert flops == wgs * 4 * iters * 131072

    def bf16_pairs(words):                               # uint32 words -> the bf16 values they pack, low half first
        w = np.asarray(words, np.uint32)
        lo = (w << np.uint32(16)).view(np.float32)
        hi = (w & np.uint32(0xffff0000)).view(np.float32)
        return np.stack([lo, hi], -1).reshape(-1)

    n = 32 if wide else 16
    A = np.zeros((n, 512 // n)); B = np.zeros((512 // n, n))
    for lane in range(64):
        seed = np.uint32(0x3f803f80 + ((lane & 7) << 16))
        a = bf16_pairs([seed, seed ^ np.uint32(0x00010000), seed, seed ^ np.uint32(0x00000001)])
        b = bf16_pairs([seed ^ np.uint32(0x80000000), seed, seed ^ np.uint32(0x00008000), seed])
        k0 = (lane // n) * 8
        A[lane % n, k0:k0 + 8] = a
        B[k0:k0 + 8, lane % n] = b
    D = A @ B
    if wide:
        rows = lambda l: [8 * g + 4 * (l // 32) + v for g in range(4) for v in range(4)]
        tiles = 4
    else:
        rows = lambda l: [4 * (l // 16) + v for v in range(4)]
        tiles = 8
    want = np.array([tiles * iters * D[rows(l), l % n].sum() for l in range(64)])
    got = sink.cpu().numpy().reshape(wgs * 4, 64)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= 1e-6 * np.abs(want).max()
    with pytest.raises(hpf.HpfError):
        hpf.hpf_probe_mfma_bf16(sink.data_ptr(), 0, 1)
