"""Bucket layouts for bca_plan_create, built on the host from a list of tensor sizes.

Sec. 2.1 of the paper: data-parallel frameworks collect gradients into buckets of a fixed capacity, in the order
backward produces them (the model's last tensors first; Alg. 1 runs b = B ... 1).  Two common ways of filling the
buckets are offered; both only prepare the arrays that Plan.from_layout marshals, and hold none of the method's
arithmetic.  Any other layout can be given to Plan directly as (tensor list, segments)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence

import numpy as np


@dataclass
class BucketLayout:
    """Segment s covers elements [seg_begin[s], seg_begin[s] + seg_len[s]) of tensor seg_tensor[s]; bucket b owns
    segments bucket_seg_off[b] .. bucket_seg_off[b + 1] - 1 in that order; bucket 0 is the first one ready."""
    tensor_numel: np.ndarray      # uint64 [n_tensors]
    bucket_seg_off: np.ndarray    # uint64 [n_buckets + 1]
    seg_tensor: np.ndarray        # uint32 [n_segments]
    seg_begin: np.ndarray         # uint64 [n_segments]
    seg_len: np.ndarray           # uint64 [n_segments]

    @property
    def n_tensors(self) -> int:
        return int(self.tensor_numel.shape[0])

    @property
    def n_buckets(self) -> int:
        return int(self.bucket_seg_off.shape[0]) - 1

    @property
    def n_elements(self) -> int:
        return int(self.tensor_numel.sum())


def _order(n: int, reverse: bool) -> np.ndarray:
    return np.arange(n - 1, -1, -1) if reverse else np.arange(n)


def flat_split(tensor_numel: Sequence[int], cap_elems: int, reverse: bool = True) -> BucketLayout:
    """The tensors laid end to end (last one first when `reverse`) and cut every `cap_elems` elements; a tensor that
    straddles a cut is split into several segments.  Tensors without elements get no segment."""
    if cap_elems <= 0:
        raise ValueError("cap_elems must be positive")
    numel = np.asarray(tensor_numel, dtype=np.uint64)
    order = _order(numel.shape[0], reverse)
    sizes = numel[order].astype(np.int64)
    start = np.concatenate([[0], np.cumsum(sizes)])            # position of each tensor (in `order`) in the flat stream
    total = int(start[-1])
    cuts = np.arange(0, total, cap_elems, dtype=np.int64)       # first position of every bucket
    edges = np.unique(np.concatenate([start[:-1][sizes > 0], cuts, [total]]))
    seg_lo, seg_hi = edges[:-1], edges[1:]
    keep = seg_hi > seg_lo
    seg_lo, seg_hi = seg_lo[keep], seg_hi[keep]
    which = np.searchsorted(start, seg_lo, side="right") - 1    # index into `order`; skips tensors without elements
    n_buckets = max(1, len(cuts))
    bucket_of_seg = seg_lo // cap_elems
    off = np.searchsorted(bucket_of_seg, np.arange(n_buckets + 1), side="left")
    return BucketLayout(numel, off.astype(np.uint64), order[which].astype(np.uint32),
                        (seg_lo - start[which]).astype(np.uint64), (seg_hi - seg_lo).astype(np.uint64))


def whole_tensors(tensor_numel: Sequence[int], cap_elems: int, reverse: bool = True) -> BucketLayout:
    """Whole tensors are appended to the current bucket (last tensor first when `reverse`); a new bucket is opened
    once the current one holds `cap_elems` elements or more."""
    numel = np.asarray(tensor_numel, dtype=np.uint64)
    seg_tensor, off, fill = [], [0], 0
    for t in _order(numel.shape[0], reverse):
        if fill >= cap_elems and len(seg_tensor) > off[-1]:
            off.append(len(seg_tensor))
            fill = 0
        seg_tensor.append(int(t))
        fill += int(numel[t])
    off.append(len(seg_tensor))
    seg_tensor = np.asarray(seg_tensor, dtype=np.uint32)
    return BucketLayout(numel, np.asarray(off, dtype=np.uint64), seg_tensor, np.zeros(len(seg_tensor), np.uint64),
                        numel[seg_tensor] if len(seg_tensor) else np.zeros(0, np.uint64))
