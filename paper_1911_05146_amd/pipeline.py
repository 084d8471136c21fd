"""Several partitions of one model chained on ONE GPU, scheduled the way the paper pipelines a batch
(Section "Exploiting Pipeline Stages within Each Minibatch"): the batch is cut into micro-batches, every
partition forwards micro-batch i as soon as the partition before it has, the partial errors flow back the
same way, and every partition accumulates its weight gradients over the micro-batches before the one
update of the batch.  Here the "ranks" are HIP streams: one per partition, with events standing in for
the send/recv pairs, so partition p works on micro-batch i while partition p+1 still works on i-1.

Host logic only: every tensor operation is a call into the C-ABI library through `hpf.Partition`.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

from . import hpf
from . import layer_cuts
from . import workloads as W


def split_model(name: str, blocks: Sequence[W.Block], n_parts: int, in_hw: int, stem_c: int, classes: int,
                microbatch: int, num_microbatches: int, seed: int) -> List[W.PartitionSpec]:
    """A stem + blocks + head model cut into n_parts contiguous partitions at block boundaries."""
    return [W.partition_of(f"{name}-part{p}of{n_parts}", list(blocks), n_parts, p, in_hw, blocks[0].c_in, stem_c, classes,
                           microbatch, num_microbatches, seed) for p in range(n_parts)]


class Pipeline:
    """specs: the partitions in model order (the first holds the stem, the last the head); params: the flat
    parameter vector of the whole model (canonical order = concatenation of the partitions' vectors).
    group: micro-batches per library call (1: finest pipelining; more: fewer, larger launches per partition)."""

    def __init__(self, specs: Sequence[W.PartitionSpec], params, compute_dtype=hpf.HPF_BF16, device="cuda:0", group: int = 1,
                 fusion: Optional[int] = None, cut_model: Optional[layer_cuts.CutModel] = None):
        """cut_model: the partitions come from layer_cuts.split_at_layers (cuts inside residual blocks, shortcut
        values exchanged between the two partitions that hold a block's ends); `specs` must be cut_model.specs and
        `params` the whole model's vector.  Such a pipeline runs one micro-batch per call (group 1)."""
        import torch
        self.torch = torch
        self.specs = list(specs)
        self.cut = cut_model
        assert self.specs[0].has_stem and self.specs[-1].has_head, "first partition holds the stem, last the head"
        self.m = self.specs[0].num_microbatches
        assert all(s.num_microbatches == self.m and s.microbatch == self.specs[0].microbatch for s in self.specs)
        assert group >= 1 and self.m % group == 0, "group must divide the number of micro-batches"
        assert cut_model is None or group == 1, "partitions cut at layer granularity run one micro-batch per call"
        self.group = group
        self.device = torch.device(device)
        self.parts: List[hpf.Partition] = []
        if cut_model is not None:
            assert len(cut_model.specs) == len(self.specs)
            pieces = cut_model.split_params(params)
            self.lists = layer_cuts.dependency_lists(cut_model)
        else:
            pieces, off = [], 0
            for s in self.specs:
                n = W.n_params(s)
                pieces.append(params[off:off + n])
                off += n
            assert off == len(params), "parameter vector does not match the partitions"
        for s, piece in zip(self.specs, pieces):
            self.parts.append(hpf.Partition(s, piece, compute_dtype, device))
            if fusion is not None:
                self.parts[-1].set_fusion(fusion)
        self.streams = [torch.cuda.Stream(self.device) for _ in self.parts]
        self._keep = []

    @property
    def loss(self):
        return self.parts[-1].loss

    def run_batch(self, act_in, labels):
        """Forward and backward of one batch: act_in / labels are lists of m device tensors.  Returns when all work
        is queued; the gradients are complete after `synchronize()` / `grad_accum_read()`."""
        if self.cut is not None:
            return self._run_batch_cut(act_in, labels)
        torch, P, g = self.torch, len(self.parts), self.group
        units = [list(range(u, u + g)) for u in range(0, self.m, g)]
        with torch.cuda.stream(self.streams[-1]):     # in the order of the head's own work; no drain of the device
            self.parts[-1].loss.zero_()
        fwd_done = [[torch.cuda.Event() for _ in units] for _ in range(P)]
        bwd_done = [[torch.cuda.Event() for _ in units] for _ in range(P)]
        acts = [[None] * self.m for _ in range(P)]   # acts[p][i]: output of partition p (input of p+1)
        errs = [[None] * self.m for _ in range(P)]   # errs[p][i]: partial error leaving partition p (into p-1)
        # ---- fill and drain, forward: unit u reaches partition p after it left p-1
        for ui, unit in enumerate(units):
            for p, part in enumerate(self.parts):
                s = self.streams[p]
                if p > 0:
                    s.wait_event(fwd_done[p - 1][ui])
                x = [act_in[i] for i in unit] if p == 0 else [acts[p - 1][i] for i in unit]
                lab = [labels[i] for i in unit] if part.spec.has_head else None
                if g == 1:
                    out = [part.forward_microbatch(unit[0], x[0], lab[0] if lab else None, stream=s)]
                else:
                    out = part.forward_microbatches(unit[0], x, lab, stream=s) or [None] * g
                for i, o in zip(unit, out):
                    acts[p][i] = o
                fwd_done[p][ui].record(s)
        # ---- backward: the partial errors travel from the head to the stem
        for ui, unit in enumerate(units):
            for p in reversed(range(P)):
                part, s = self.parts[p], self.streams[p]
                if p < P - 1:
                    s.wait_event(bwd_done[p + 1][ui])
                e_in = None if part.spec.has_head else [errs[p + 1][i] for i in unit]
                if g == 1:
                    out = [part.backward_microbatch(unit[0], e_in[0] if e_in else None, stream=s)]
                else:
                    out = part.backward_microbatches(unit[0], g, e_in, stream=s) or [None] * g
                for i, o in zip(unit, out):
                    errs[p][i] = o
                bwd_done[p][ui].record(s)
        # the boundary tensors must outlive the queued work: those of the batch before are let go only now that this
        # batch is queued behind it on the same streams
        self._keep = [self._keep[-4:] if self._keep else None, acts, errs, act_in, labels]

    def _run_batch_cut(self, act_in, labels):
        """The same schedule for partitions cut at layer granularity.  Every rank walks its Forward list (receives
        ordered by source rank, then sends ordered by destination rank) and, in the backward pass, its Backward
        list; a receive is a wait on the sender's event plus the use of its buffer, a send is the record of the
        rank's own event (all tensors of one call are complete together)."""
        torch, P = self.torch, len(self.parts)
        with torch.cuda.stream(self.streams[-1]):
            self.parts[-1].loss.zero_()
        fwd_done = [[torch.cuda.Event() for _ in range(self.m)] for _ in range(P)]
        bwd_done = [[torch.cuda.Event() for _ in range(self.m)] for _ in range(P)]
        sent = [[{} for _ in range(self.m)] for _ in range(P)]       # sent[p][i][tensor]: forward outputs of rank p
        grads = [[{} for _ in range(self.m)] for _ in range(P)]      # grads[p][i][tensor]: gradients rank p returns for what it received
        for i in range(self.m):
            for p, part in enumerate(self.parts):
                s, L = self.streams[p], self.lists[p]
                got = {"act": act_in[i] if p == 0 else None, "skip": None}
                for msg in L.forward_recv:
                    s.wait_event(fwd_done[msg.src][i])
                    got[msg.tensor] = sent[msg.src][i][msg.tensor]
                out, skip_out = part.forward_microbatch_cut(i, got["act"], got["skip"],
                                                            labels[i] if part.spec.has_head else None, stream=s)
                sent[p][i] = {"act": out, "skip": skip_out}
                fwd_done[p][i].record(s)
        for i in range(self.m):
            for p in reversed(range(P)):
                part, s, L = self.parts[p], self.streams[p], self.lists[p]
                got = {"act": None, "skip": None}
                for msg in L.backward_recv:                         # gradients of what this rank sent
                    s.wait_event(bwd_done[msg.dst][i])
                    got[msg.tensor] = grads[msg.dst][i][msg.tensor]
                err_out, skip_err_out = part.backward_microbatch_cut(i, got["act"], got["skip"], stream=s)
                grads[p][i] = {"act": err_out, "skip": skip_err_out}
                bwd_done[p][i].record(s)
        self._keep = [self._keep[-4:] if self._keep else None, sent, grads, act_in, labels]

    def synchronize(self):
        self.torch.cuda.synchronize(self.device)
        self._keep = []

    def grad_accum_read(self):
        """The accumulated gradients of all partitions in whole-model order (numpy)."""
        import numpy as np
        per = [p.grad_accum_read() for p in self.parts]
        out = self.cut.merge(per) if self.cut is not None else np.concatenate(per)
        self.synchronize()
        return out

    def sgd_step(self, lr, momentum):
        for p, s in zip(self.parts, self.streams):
            p.sgd_step(lr, momentum, stream=s)

    def params_read(self):
        import numpy as np
        per = [p.params_read() for p in self.parts]
        return self.cut.merge(per) if self.cut is not None else np.concatenate(per)

    def close(self):
        self.synchronize()
        for p in self.parts:
            p.close()
        self.parts = []
