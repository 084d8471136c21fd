"""No-GPU checks of the boundary: the C-ABI library loads, exports every symbol include/hpf.h
declares, and validates descriptions on the host."""
import ctypes as C
import dataclasses
import os
import re

import pytest

from paper_1911_05146_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hpf():
    from paper_1911_05146_amd import hpf as h
    return h


def test_library_exports_every_declared_symbol(hpf):
    header = open(os.path.join(ROOT, "include", "hpf.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(hpf_[a-z0-9_]+)\s*\(", header))
    assert {"hpf_partition_create", "hpf_forward_microbatch", "hpf_backward_microbatch", "hpf_grad_accum_read",
            "hpf_sgd_step"} <= declared
    lib = C.CDLL(hpf.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in hpf.h but not exported"
    assert declared == set(hpf.EXPORTS), declared ^ set(hpf.EXPORTS)


def test_sizes_of_the_benchmark_partitions(hpf):
    expect = {1: 272282, 2: 446528, 3: 373632, 4: 10327706, 5: 40610816}
    for i, n in expect.items():
        spec = W.config(i)
        z = hpf.hpf_partition_sizes(hpf.make_desc(spec)[0])
        assert z.n_params == n == W.n_params(spec)
        b = spec.microbatch
        assert z.act_in_elems == b * spec.in_h * spec.in_w * spec.in_c
        oh, ow, oc = spec.out_shape()
        assert z.act_out_elems == (0 if spec.has_head else b * oh * ow * oc)
        assert z.arena_bytes > z.stash_bytes > 0 and z.arena_bytes % 256 == 0
    for i in (6, 7, 8):   # the wider ResNet-1001 partition, ResNet-110-v1 and VGG-16: the plan of their other unit kinds
        spec = W.config(i)
        z = hpf.hpf_partition_sizes(hpf.make_desc(spec)[0])
        assert z.n_params == W.n_params(spec)
        assert z.arena_bytes > z.stash_bytes > 0 and z.arena_bytes % 256 == 0


def status_of(hpf, spec, dtype=None):
    try:
        hpf.hpf_partition_sizes(hpf.make_desc(spec, hpf.HPF_BF16 if dtype is None else dtype)[0])
        return hpf.HPF_OK
    except hpf.HpfError as e:
        assert str(e)
        return e.status


def test_invalid_and_unsupported_descriptions(hpf):
    good = W.config(3)
    assert status_of(hpf, good) == hpf.HPF_OK
    r = dataclasses.replace
    assert status_of(hpf, r(good, microbatch=0)) == hpf.HPF_EINVAL
    assert status_of(hpf, r(good, num_microbatches=-1)) == hpf.HPF_EINVAL
    assert status_of(hpf, r(good, in_h=0)) == hpf.HPF_EINVAL
    assert status_of(hpf, r(good, bn_mode=2)) == hpf.HPF_EINVAL
    assert status_of(hpf, r(good, bn_eps=0.0)) == hpf.HPF_EINVAL
    assert status_of(hpf, r(good, in_c=64)) == hpf.HPF_EINVAL                      # chain broken at block 0
    assert status_of(hpf, r(good, blocks=())) == hpf.HPF_EINVAL                    # no unit: partitions <= layers
    odd = r(good, in_h=15, blocks=(W.Block(W.BOTTLENECK, 128, 32, 128, 2),))
    assert status_of(hpf, odd) == hpf.HPF_EINVAL                                    # 15 rows, stride 2
    bad_kind = r(good, blocks=(W.Block(7, 128, 32, 128, 1),))
    assert status_of(hpf, bad_kind) == hpf.HPF_EINVAL
    basic_mismatch = r(good, blocks=(W.Block(W.BASIC, 128, 32, 128, 1),))
    assert status_of(hpf, basic_mismatch) == hpf.HPF_EINVAL
    narrow = r(good, in_c=24, blocks=(W.Block(W.BOTTLENECK, 24, 8, 24, 1),))
    assert status_of(hpf, narrow) == hpf.HPF_EUNSUPPORTED                           # not multiples of 16 in bf16
    assert status_of(hpf, narrow, hpf.HPF_F32) == hpf.HPF_OK
    d, _ = hpf.make_desc(good)
    d.abi_version = 99
    with pytest.raises(hpf.HpfError):
        hpf.hpf_partition_sizes(d)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_layer_cut_descriptions_sizes_and_validation(hpf):
    """Partitions cut inside residual blocks (paper Section "Special Handling for Non-consecutive Models"): the
    library and the host-side splitter agree on parameter counts and tensor sizes; bad cuts are rejected."""
    from paper_1911_05146_amd import layer_cuts as LC
    blocks = W.bottleneck_resnet_blocks([2, 2], (16, 32), (64, 128), 16) + [W.Block(W.BASIC, 128, 128, 128, 1)]
    cm = LC.split_at_layers("m", blocks, [1, 2, 4, 8, 13], 16, 16, 10, 4, 2, 3)
    total = 0
    for spec in cm.specs:
        z = hpf.hpf_partition_sizes(hpf.make_desc(spec)[0])
        assert z.n_params == W.n_params(spec)
        total += z.n_params
        b = spec.microbatch
        oh, ow, oc = spec.out_shape()
        assert z.act_in_elems == b * spec.in_h * spec.in_w * spec.in_c
        assert z.act_out_elems == (0 if spec.has_head else b * oh * ow * oc)
        assert z.skip_in_elems == (b * int(__import__("numpy").prod(spec.skip_in_shape())) if spec.has_skip_in else 0)
        assert z.skip_out_elems == (b * int(__import__("numpy").prod(spec.skip_out_shape())) if spec.has_skip_out else 0)
    assert total == W.n_params(cm.whole)
    r = dataclasses.replace
    tail = cm.specs[2]                       # starts after the first two convolutions of block 0
    assert tail.first_from == 2 and status_of(hpf, tail) == hpf.HPF_OK
    assert status_of(hpf, r(tail, first_from=3)) == hpf.HPF_EINVAL           # a bottleneck has three convolutions
    assert status_of(hpf, r(tail, first_from=-1)) == hpf.HPF_EINVAL
    assert status_of(hpf, r(tail, in_c=64)) == hpf.HPF_EINVAL                # the input must have c_mid channels
    assert status_of(hpf, r(tail, has_stem=True, stem_c_out=16)) == hpf.HPF_EINVAL
    head = cm.specs[0]
    assert head.last_to == 1 and head.has_stem
    assert status_of(hpf, r(head, last_to=3)) == hpf.HPF_EINVAL              # the whole block is last_to = 0
    assert status_of(hpf, r(head, has_head=True, num_classes=10)) == hpf.HPF_EINVAL
    one = r(tail, blocks=tail.blocks[:1], first_from=1, last_to=1)
    assert status_of(hpf, one) == hpf.HPF_EINVAL                             # empty range of convolutions
