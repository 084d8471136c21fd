"""MI355X-native partition engine: one model partition's forward and backward
propagation over pipelined micro-batches with gradient accumulation and an SGD
step (HyPar-Flow-style model-parallel training, one GPU's share).

`paper_1911_05146_amd.hpf` is the ctypes binding to the HIP library; it is
imported lazily so that `paper_1911_05146_amd.workloads` (shapes and seeded
inputs only) can be used without it.
"""

__all__ = ["workloads", "hpf"]
