"""Lexicographic relabelling of the coordinates of a sparse tensor (input preparation, torch ops only).

Section 7 of the paper reorders the data before the computation with an algorithm built on doubly
lexical ordering: one mode is sorted per iteration, all modes in turn.  This module holds the
relabelling used for the on/off experiment of bench.py: in the iteration for mode n the nonzeros
are sorted lexicographically by their coordinates in the other modes (current labels), and the
indices of mode n are renumbered in the order in which they first appear in that sorted list --
i.e. by their lexicographically smallest "row" of other-mode coordinates, earlier label first
among equals.  That is the first level of the partition refinement a full doubly lexical ordering
performs; indices without a nonzero keep their relative order after all others.

Nothing here does arithmetic on values: the result is the same tensor with renamed indices, and a
dense operand indexed by mode n has to be permuted with `labels[n]` to give the same product.
"""
from typing import List, Sequence, Tuple

import torch


def _lex_order(cols: Sequence[torch.Tensor], sizes: Sequence[int]) -> torch.Tensor:
    """Stable permutation that sorts the positions lexicographically by cols[0], cols[1], ..."""
    total_bits = sum(max(1, int(s - 1).bit_length()) for s in sizes)
    if total_bits <= 62:
        key = torch.zeros_like(cols[0])
        for c, s in zip(cols, sizes):
            key = key * int(s) + c
        return torch.sort(key, stable=True).indices
    perm = torch.arange(cols[0].numel(), device=cols[0].device)
    for c in reversed(cols):                       # least significant first, stable passes
        perm = perm[torch.sort(c[perm], stable=True).indices]
    return perm


def lexi_relabel(coords: Sequence[torch.Tensor], dims: Sequence[int], sweeps: int = 1
                 ) -> Tuple[List[torch.Tensor], List[torch.Tensor]]:
    """Returns (new coordinates, labels) with new_coords[n] = labels[n][coords[n]] (int64 tensors)."""
    order = len(coords)
    cur = [c.to(torch.int64).clone() for c in coords]
    dev = cur[0].device
    labels = [torch.arange(int(d), dtype=torch.int64, device=dev) for d in dims]
    nnz = cur[0].numel()
    for _ in range(sweeps):
        for n in range(order):
            others = [m for m in range(order) if m != n]
            perm = _lex_order([cur[m] for m in others], [dims[m] for m in others])
            idx_sorted = cur[n][perm]
            first = torch.full((int(dims[n]),), nnz, dtype=torch.int64, device=dev)
            first.scatter_reduce_(0, idx_sorted, torch.arange(nnz, dtype=torch.int64, device=dev), reduce="amin")
            rank_of = torch.empty(int(dims[n]), dtype=torch.int64, device=dev)
            rank_of[torch.sort(first, stable=True).indices] = torch.arange(int(dims[n]), dtype=torch.int64, device=dev)
            cur[n] = rank_of[cur[n]]
            labels[n] = rank_of[labels[n]]
            del perm, idx_sorted, first, rank_of
    return cur, labels


def sort_nonzeros(coords: Sequence[torch.Tensor], dims: Sequence[int], vals: torch.Tensor):
    """The nonzeros in lexicographic order of (coords[0], coords[1], ...), as the packers expect them."""
    perm = _lex_order(list(coords), list(dims))
    return [c[perm] for c in coords], vals[perm]


__all__ = ["lexi_relabel", "sort_nonzeros"]
