"""Cutting a model into partitions at LAYER granularity, with skip connections that cross partitions.

Paper Section "Special Handling for Non-consecutive Models": a partition is a range of layers, so a cut may
fall inside a residual block; the skip connection of such a block then runs between two partitions that need
not be neighbours, next to the boundary tensor that runs between neighbours.  Every partition keeps a Forward
list (where the outputs of its layers go) and a Backward list (where their inputs come from), and the messages
are ordered by rank so that no cycle of blocking sends and receives can form.

This module is host logic only (no arithmetic of the method, no GPU): it turns a list of cut positions into
partition descriptions, says which slice of the whole model's parameter vector each partition owns, builds the
two lists per partition, and can replay them under blocking send / receive semantics to show whether an
ordering completes.  The unit of a cut is a convolution together with the BatchNorm+ReLU that feeds it; the
projection shortcut goes with a block's first convolution and the residual add with its last.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import workloads as W


def n_convs(block: W.Block) -> int:
    return 2 if block.kind == W.BASIC else 3


def conv_layers(blocks: Sequence[W.Block]) -> List[Tuple[int, int]]:
    """(block index, convolution index within the block) of every convolution layer, in model order."""
    return [(i, j) for i, b in enumerate(blocks) for j in range(n_convs(b))]


def even_layer_cuts(blocks: Sequence[W.Block], n_parts: int) -> List[int]:
    """Cut positions (global convolution indices at which partitions 1.. begin) of an even split."""
    n = len(conv_layers(blocks))
    assert 1 <= n_parts <= n, "at most one partition per layer"
    return [(p * n) // n_parts for p in range(1, n_parts)]


@dataclass(frozen=True)
class Message:
    """One tensor that crosses partitions in the forward pass; the backward pass returns its gradient."""
    tensor: str          # "act": boundary tensor between neighbours; "skip": shortcut value of a cut block
    src: int             # rank (partition index) that produces it
    dst: int             # rank that consumes it


@dataclass
class CutModel:
    specs: List[W.PartitionSpec]
    whole: W.PartitionSpec
    param_index: List[np.ndarray]                      # partition p owns whole-model parameters param_index[p]
    messages: List[Message] = field(default_factory=list)

    @property
    def n_parts(self) -> int:
        return len(self.specs)

    def skip_src(self, p: int) -> Optional[int]:
        """Rank that sends partition p its skip_in (None: p needs none)."""
        for m in self.messages:
            if m.tensor == "skip" and m.dst == p:
                return m.src
        return None

    def skip_dst(self, p: int) -> Optional[int]:
        """Rank that takes partition p's skip_out."""
        for m in self.messages:
            if m.tensor == "skip" and m.src == p:
                return m.dst
        return None

    def split_params(self, params: np.ndarray) -> List[np.ndarray]:
        return [np.ascontiguousarray(params[ix]) for ix in self.param_index]

    def merge(self, per_partition: Sequence[np.ndarray]) -> np.ndarray:
        """Per-partition flat vectors (parameters or gradients) back into whole-model order."""
        out = np.empty(W.n_params(self.whole), dtype=per_partition[0].dtype)
        for ix, v in zip(self.param_index, per_partition):
            out[ix] = v
        return out


def split_at_layers(name: str, blocks: Sequence[W.Block], cuts: Sequence[int], in_hw: int, stem_c: int, classes: int,
                    microbatch: int, num_microbatches: int, seed: int, in_c_img: int = 3) -> CutModel:
    """A stem + blocks + head model cut where the convolutions with global indices `cuts` begin (strictly
    increasing, 0 < cut < number of convolutions).  Partition 0 holds the stem, the last one the head."""
    blocks = list(blocks)
    layers = conv_layers(blocks)
    cuts = list(cuts)
    assert all(0 < c < len(layers) for c in cuts) and all(a < b for a, b in zip(cuts, cuts[1:])), "bad cut positions"
    bounds = [0] + cuts + [len(layers)]
    n_parts = len(bounds) - 1
    whole = W.PartitionSpec(name=name, in_h=in_hw, in_w=in_hw, in_c=in_c_img, blocks=tuple(blocks), has_stem=True,
                            stem_c_out=stem_c, has_head=True, num_classes=classes, microbatch=microbatch,
                            num_microbatches=num_microbatches, seed=seed)
    whole_off = {e.name: e for e in W.param_layout(whole)}
    hw_before = [in_hw]                                 # spatial size entering block i
    for b in blocks:
        hw_before.append(hw_before[-1] // b.stride)

    specs, param_index, messages = [], [], []
    open_skip: Dict[int, int] = {}                      # block index -> rank holding its start, while the block is cut open
    for p in range(n_parts):
        (b_lo, j_lo), (b_hi, j_hi) = layers[bounds[p]], layers[bounds[p + 1] - 1]
        first, last = p == 0, p == n_parts - 1
        ends_inside = j_hi + 1 < n_convs(blocks[b_hi])
        if j_lo == 0:
            h, c = hw_before[b_lo], blocks[b_lo].c_in
        else:
            h, c = hw_before[b_lo + 1], blocks[b_lo].c_mid
        spec = W.PartitionSpec(
            name=f"{name}-layers{bounds[p]}to{bounds[p + 1]}", in_h=in_hw if first else h, in_w=in_hw if first else h,
            in_c=in_c_img if first else c, blocks=tuple(blocks[b_lo:b_hi + 1]), has_stem=first,
            stem_c_out=stem_c if first else 0, has_head=last, num_classes=classes if last else 0,
            microbatch=microbatch, num_microbatches=num_microbatches, seed=seed,
            first_from=j_lo, last_to=(j_hi + 1) if ends_inside else 0)
        specs.append(spec)
        # parameters: same names, block indices shifted by b_lo
        ix = []
        for e in W.param_layout(spec):
            nm = e.name
            if nm.startswith("block"):
                k, rest = nm[5:].split(".", 1)
                nm = f"block{int(k) + b_lo}.{rest}"
            we = whole_off[nm]
            assert we.shape == e.shape, (nm, we.shape, e.shape)
            ix.append(np.arange(we.offset, we.offset + we.size))
        param_index.append(np.concatenate(ix) if ix else np.zeros(0, dtype=np.int64))
        # messages
        if not first:
            messages.append(Message("act", p - 1, p))
        if spec.has_skip_in:
            messages.append(Message("skip", open_skip.pop(b_lo), p))
        if spec.has_skip_out:
            open_skip[b_hi] = p
    assert not open_skip
    all_ix = np.sort(np.concatenate(param_index))
    assert all_ix.size == W.n_params(whole) and np.array_equal(all_ix, np.arange(all_ix.size)), "every parameter has one owner"
    return CutModel(specs, whole, param_index, messages)


# ----------------------------------------------------------------------------------------------------------
# Forward / Backward lists and the rank-sorted message order
# ----------------------------------------------------------------------------------------------------------
@dataclass
class RankLists:
    """What one rank exchanges per micro-batch.  forward_recv / forward_send are walked in this order in the
    forward pass; the backward pass walks backward_recv (gradients of what was sent) and backward_send
    (gradients of what was received)."""
    forward_recv: List[Message]
    forward_send: List[Message]
    backward_recv: List[Message]
    backward_send: List[Message]


def dependency_lists(cm: CutModel, sort_by_rank: bool = True) -> List[RankLists]:
    """Per rank: receives ordered by source rank and sends ordered by destination rank, so that a rank's first
    message goes to the rank that holds the next layer.  sort_by_rank=False gives the opposite order (farthest
    partner first), which is what an unsorted walk over the skip connections can produce."""
    out = []
    for p in range(cm.n_parts):
        recv = sorted((m for m in cm.messages if m.dst == p), key=lambda m: m.src, reverse=not sort_by_rank)
        send = sorted((m for m in cm.messages if m.src == p), key=lambda m: m.dst, reverse=not sort_by_rank)
        # backward: gradients flow the other way; the nearest partner in that direction comes first
        brecv = sorted((m for m in cm.messages if m.src == p), key=lambda m: -m.dst, reverse=not sort_by_rank)
        bsend = sorted((m for m in cm.messages if m.dst == p), key=lambda m: -m.src, reverse=not sort_by_rank)
        out.append(RankLists(recv, send, brecv, bsend))
    return out


def replay_blocking(lists: Sequence[RankLists], direction: str = "forward") -> bool:
    """Replays one pass under blocking, unbuffered semantics: a rank posts its receives in list order, then
    computes, then posts its sends in list order, and every send or receive completes only when its partner has
    reached the matching call.  Returns True if all ranks finish, False on deadlock."""
    n = len(lists)
    progs = []
    for r in lists:
        rc, sd = (r.forward_recv, r.forward_send) if direction == "forward" else (r.backward_recv, r.backward_send)
        if direction == "forward":
            ops = [("recv", m.src, m) for m in rc] + [("send", m.dst, m) for m in sd]
        else:   # gradient of message m travels from m.dst back to m.src
            ops = [("recv", m.dst, m) for m in rc] + [("send", m.src, m) for m in sd]
        progs.append(ops)
    pc = [0] * n
    while True:
        moved = False
        for a in range(n):
            if pc[a] >= len(progs[a]):
                continue
            kind, b, msg = progs[a][pc[a]]
            if pc[b] >= len(progs[b]):
                continue
            kind_b, partner_b, msg_b = progs[b][pc[b]]
            if partner_b == a and msg_b == msg and kind_b != kind:
                pc[a] += 1
                pc[b] += 1
                moved = True
        if all(pc[r] >= len(progs[r]) for r in range(n)):
            return True
        if not moved:
            return False
