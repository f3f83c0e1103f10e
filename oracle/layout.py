"""Bucket -> parameter mapping of the shadow node (oracle side, test infrastructure).

Follows section 4.2.2 of the paper ("Mapping Bucket to Model Parameters"):
parameters are bin-packed into buckets starting from the LAST model tensor and
working backwards; a tensor joins the open bucket while the bucket stays within
the maximum size (25 MB in DDP); a tensor larger than the maximum gets a bucket
of its own.  A tensor is never split, and inside a bucket every tensor is an
offset view (no copies), in the order in which it was added.

Reading taken where the text is loose: sizes are counted in gradient bytes; the
bucket that is formed first (last layers) has id 0.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple


@dataclass
class Segment:
    tensor: int        # index in model order
    offset: int        # element offset inside the bucket
    numel: int
    weight_decay: bool


@dataclass
class Bucket:
    numel: int = 0
    segments: List[Segment] = field(default_factory=list)


@dataclass
class Layout:
    buckets: List[Bucket]
    bucket_of_tensor: List[int]

    @property
    def num_params(self) -> int:
        return sum(b.numel for b in self.buckets)

    def logical_starts(self) -> List[int]:
        """Start of each bucket in the bucket-major, unpadded element order."""
        out, acc = [], 0
        for b in self.buckets:
            out.append(acc)
            acc += b.numel
        return out


def build_layout(tensors: Sequence[Tuple[int, bool]], grad_elem_bytes: int, cap_bytes: int,
                 bucket_of_tensor: Optional[Sequence[int]] = None) -> Layout:
    """tensors: (numel, weight_decay) in model order (first layer first)."""
    T = len(tensors)
    assign = [-1] * T
    if bucket_of_tensor is not None:
        if len(bucket_of_tensor) != T:
            raise ValueError("bucket_of_tensor length")
        assign = [int(b) for b in bucket_of_tensor]
        nb = max(assign) + 1 if T else 0
        if sorted(set(assign)) != list(range(nb)):
            raise ValueError("bucket ids must be dense")
    else:
        cur = -1          # id of the open bucket, -1 = none open
        cur_bytes = 0
        nb = 0
        for t in range(T - 1, -1, -1):
            size = tensors[t][0] * grad_elem_bytes
            if size > cap_bytes:
                assign[t] = nb          # alone; whatever was open is closed
                nb += 1
                cur = -1
                continue
            if cur < 0 or cur_bytes + size > cap_bytes:
                cur = nb
                nb += 1
                cur_bytes = 0
            assign[t] = cur
            cur_bytes += size
    buckets = [Bucket() for _ in range(nb)]
    # members are laid out in the order they were added: last tensor first
    for t in range(T - 1, -1, -1):
        b = buckets[assign[t]]
        n, wd = tensors[t]
        b.segments.append(Segment(t, b.numel, int(n), bool(wd)))
        b.numel += int(n)
    return Layout(buckets, assign)
