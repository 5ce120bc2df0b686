"""Block granularity (the paper's Section 6 remark: from layers to blocks, one block holding many small
layers): segment sizes for a plan in which every tensor below a size is merged with its neighbour.
Sizes only: the flat buffers stay as they are, a block is a run of consecutive tensors."""
from __future__ import annotations

from typing import List, Sequence


def merge_small(sizes: Sequence[int], min_elems: int) -> List[int]:
    """Consecutive tensors are gathered until the block holds at least `min_elems` elements; a short
    tail joins the block before it.  The blocks' boundaries are a subset of the tensors'."""
    out: List[int] = []
    acc = 0
    for n in sizes:
        acc += int(n)
        if acc >= min_elems:
            out.append(acc)
            acc = 0
    if acc:
        if out:
            out[-1] += acc
        else:
            out.append(acc)
    return out
