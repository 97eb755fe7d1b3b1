"""Balanced tensor fragmentation -- TEST INFRASTRUCTURE ONLY (part of the CPU oracle).

Appendix C, "Balanced tensor fragmentation": the Q tensors of the model are packed into P
fragments by greedy number partitioning -- walk the tensors in descending order of size and
put each one into the fragment whose total size is currently the smallest.

The paper does not say how ties are broken.  Reading taken: tensors of equal size keep their
original order (stable sort), and among equally light fragments the lowest index wins.
"""
from __future__ import annotations

from typing import List, Sequence


def balanced_fragments(sizes: Sequence[int], num_fragments: int) -> List[int]:
    """fragment_of[i] = index of the fragment that tensor i is put in."""
    if num_fragments < 1:
        raise ValueError("need at least one fragment")
    order = sorted(range(len(sizes)), key=lambda i: -int(sizes[i]))   # stable: ties keep order
    load = [0] * num_fragments
    fragment_of = [0] * len(sizes)
    for i in order:
        p = min(range(num_fragments), key=lambda k: load[k])          # first lightest fragment
        fragment_of[i] = p
        load[p] += int(sizes[i])
    return fragment_of


def fragment_loads(sizes: Sequence[int], fragment_of: Sequence[int], num_fragments: int) -> List[int]:
    load = [0] * num_fragments
    for s, p in zip(sizes, fragment_of):
        load[p] += int(s)
    return load
