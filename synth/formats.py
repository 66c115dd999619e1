"""Packing of sorted coordinate lists into per-level pos/crd storage.

The storage follows the paper's per-dimension attributes (Section 4, "Tensor
Storage Format"; Table "Generated code to access nonzeros coordinates"):

  D   dense               pos = [size],            no crd
  CU  compressed-unique   pos = segment offsets,   crd = unique coordinates
  CN  compressed-nonunique pos = [0, nnz],         crd = every coordinate
  S   singleton           no pos,                  crd = one coordinate per parent position

This module only lays data out; it performs none of the contractions.  Inputs
are torch tensors (any device); coordinates must be lexicographically sorted and
free of duplicates.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import torch

D, CU, CN, S = 0, 1, 2, 3
TAG_NAMES = {D: "D", CU: "CU", CN: "CN", S: "S"}


@dataclass
class LevelTensor:
    """A sparse tensor as per-level pos/crd int32 arrays plus one fp64 vals array."""
    dims: List[int]
    tags: List[int]
    pos: List[Optional[torch.Tensor]]
    crd: List[Optional[torch.Tensor]]
    vals: torch.Tensor
    name: str = ""
    meta: dict = field(default_factory=dict)

    @property
    def order(self) -> int:
        return len(self.dims)

    @property
    def nnz(self) -> int:
        return int(self.vals.numel())

    def to(self, device) -> "LevelTensor":
        mv = lambda t: None if t is None else t.to(device)
        return LevelTensor(list(self.dims), list(self.tags), [mv(p) for p in self.pos],
                           [mv(c) for c in self.crd], self.vals.to(device), self.name, dict(self.meta))

    def format_name(self) -> str:
        return "[" + ",".join(TAG_NAMES[t] for t in self.tags) + "]"


def _i32(t: torch.Tensor) -> torch.Tensor:
    return t.to(torch.int32).contiguous()


def _segment_pos(parent_ids: torch.Tensor, nparents: int) -> torch.Tensor:
    """Offsets of the runs of a sorted parent-id list: pos[m]..pos[m+1] are the children of m."""
    counts = torch.bincount(parent_ids, minlength=nparents) if parent_ids.numel() else \
        torch.zeros(nparents, dtype=torch.int64, device=parent_ids.device)
    pos = torch.zeros(nparents + 1, dtype=torch.int64, device=parent_ids.device)
    torch.cumsum(counts, 0, out=pos[1:])
    return pos


def _run_heads(*keys: torch.Tensor) -> torch.Tensor:
    """Boolean mask: element p starts a new run of equal key tuples."""
    n = keys[0].numel()
    head = torch.ones(n, dtype=torch.bool, device=keys[0].device)
    if n > 1:
        same = torch.ones(n - 1, dtype=torch.bool, device=keys[0].device)
        for k in keys:
            same &= k[1:] == k[:-1]
        head[1:] = ~same
    return head


def pack_csr(nrows: int, ncols: int, rows, cols, vals) -> LevelTensor:
    """[D, CU]: row level dense, column level compressed-unique."""
    dev = vals.device
    pos2 = _segment_pos(rows.to(torch.int64), nrows)
    return LevelTensor([nrows, ncols], [D, CU],
                       [torch.tensor([nrows], dtype=torch.int32, device=dev), _i32(pos2)],
                       [None, _i32(cols)], vals.contiguous(), "CSR")


def pack_dcsr(nrows: int, ncols: int, rows, cols, vals) -> LevelTensor:
    """[CU, CU]: only rows that hold a nonzero are stored."""
    dev = vals.device
    head = _run_heads(rows)
    crd1 = rows[head]
    stored_row = torch.cumsum(head.to(torch.int64), 0) - 1          # position of each nnz's row in crd1
    pos2 = _segment_pos(stored_row, int(crd1.numel()))
    pos1 = torch.tensor([0, int(crd1.numel())], dtype=torch.int32, device=dev)
    return LevelTensor([nrows, ncols], [CU, CU], [pos1, _i32(pos2)], [_i32(crd1), _i32(cols)],
                       vals.contiguous(), "DCSR")


def pack_coo(dims, coords, vals) -> LevelTensor:
    """[CN, S, ...]: root level keeps every coordinate; the others are singletons."""
    dev = vals.device
    n = int(vals.numel())
    order = len(dims)
    pos = [torch.tensor([0, n], dtype=torch.int32, device=dev)] + [None] * (order - 1)
    return LevelTensor(list(dims), [CN] + [S] * (order - 1), pos, [_i32(c) for c in coords],
                       vals.contiguous(), "COO")


def pack_csf3(dims, i, j, k, vals) -> LevelTensor:
    """[CU, CU, CU]: slices, fibers, nonzeros of an order-3 tensor."""
    dev = vals.device
    fiber_head = _run_heads(i, j)
    fi, fj = i[fiber_head], j[fiber_head]
    fiber_of_nnz = torch.cumsum(fiber_head.to(torch.int64), 0) - 1
    nfib = int(fi.numel())
    pos3 = _segment_pos(fiber_of_nnz, nfib)
    slice_head = _run_heads(fi)
    crd1 = fi[slice_head]
    slice_of_fiber = torch.cumsum(slice_head.to(torch.int64), 0) - 1
    n1 = int(crd1.numel())
    pos2 = _segment_pos(slice_of_fiber, n1)
    pos1 = torch.tensor([0, n1], dtype=torch.int32, device=dev)
    return LevelTensor(list(dims), [CU, CU, CU], [pos1, _i32(pos2), _i32(pos3)],
                       [_i32(crd1), _i32(fj), _i32(k)], vals.contiguous(), "CSF")
