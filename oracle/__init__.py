"""CPU oracle (TEST INFRASTRUCTURE ONLY -- never imported by the product package).

Thin numpy front-end of `comet_oracle.c`: each function takes a coordinate list and dense
operands as numpy arrays and returns the defining sum of the operation (Section 8.2 of the
paper, "Sparse Tensor Operations") together with A = sum |term| per output element.  Only
the tests, the smoke check and the benchmark's CPU-baseline leg may use this package; it
shares no code with the HIP path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "comet_oracle.c")
_LIB = os.path.join(_HERE, "libcomet_oracle.so")
_lib = None

D, CU, CN, S = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, no FMA contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_group_pairs.restype = ctypes.c_int64
        for name in ("oracle_spmv", "oracle_spmm", "oracle_ttv", "oracle_ttm", "oracle_mttkrp", "oracle_walk"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


_I64 = ctypes.c_int64


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError("oracle %s failed with code %d" % (what, rc))


def spmv(rows, cols, vals, shape: Sequence[int], x) -> Tuple[np.ndarray, np.ndarray]:
    """y_i = sum_j x_ij v_j over the coordinate list; returns (y, A)."""
    I, J = int(shape[0]), int(shape[1])
    rows, cols, vals, x = _i32(rows), _i32(cols), _f64(vals), _f64(x)
    assert x.shape == (J,) and rows.shape == cols.shape == vals.shape
    y, ya = np.empty(I), np.empty(I)
    _check(_load().oracle_spmv(_I64(vals.size), _p(rows), _p(cols), _p(vals), _I64(I), _I64(J),
                               _p(x), _p(y), _p(ya)), "spmv")
    return y, ya


def spmm(rows, cols, vals, shape: Sequence[int], U) -> Tuple[np.ndarray, np.ndarray]:
    """Y_ir = sum_j x_ij U_jr; U is (J, R) row-major; returns (Y, A) of shape (I, R)."""
    I, J = int(shape[0]), int(shape[1])
    rows, cols, vals, U = _i32(rows), _i32(cols), _f64(vals), _f64(U)
    assert U.ndim == 2 and U.shape[0] == J
    R = U.shape[1]
    Y, Ya = np.empty((I, R)), np.empty((I, R))
    _check(_load().oracle_spmm(_I64(vals.size), _p(rows), _p(cols), _p(vals), _I64(I), _I64(J),
                               _I64(R), _p(U), _p(Y), _p(Ya)), "spmm")
    return Y, Ya


def axpby(alpha: float, prod, prod_abs, beta: float, old) -> Tuple[np.ndarray, np.ndarray]:
    """alpha * prod + beta * old element by element (the in-place update of Section 6.2, Step III, with the usual
    two scalars); beta == 0 does not read `old`, alpha == 0 does not read `prod`.  Returns (result, sum of |terms|)."""
    prod, prod_abs, old = _f64(prod), _f64(prod_abs), _f64(old)
    assert prod.shape == prod_abs.shape == old.shape
    out, out_abs = np.empty(prod.shape), np.empty(prod.shape)
    _check(_load().oracle_axpby(_I64(prod.size), ctypes.c_double(alpha), _p(prod), _p(prod_abs), ctypes.c_double(beta),
                                _p(old), _p(out), _p(out_abs)), "axpby")
    return out, out_abs


def group_pairs(ci, cj) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Distinct (i, j) pairs in lexicographic order: (gid per nonzero, gi, gj)."""
    ci, cj = _i32(ci), _i32(cj)
    n = ci.size
    gid = np.empty(n, dtype=np.int64)
    gi, gj = np.empty(n, dtype=np.int32), np.empty(n, dtype=np.int32)
    g = _load().oracle_group_pairs(_I64(n), _p(ci), _p(cj), _p(gid), _p(gi), _p(gj))
    if g < 0:
        raise ValueError("oracle group_pairs failed")
    return gid, gi[:g].copy(), gj[:g].copy()


def ttv(ci, cj, ck, vals, dims: Sequence[int], v) -> Dict[str, np.ndarray]:
    """Y(i,j) = sum_k X(i,j,k) v(k); the output lists the distinct (i,j) in lexicographic order."""
    ck, vals, v = _i32(ck), _f64(vals), _f64(v)
    K = int(dims[2])
    assert v.shape == (K,)
    gid, gi, gj = group_pairs(ci, cj)
    g = gi.size
    y, ya = np.empty(g), np.empty(g)
    _check(_load().oracle_ttv(_I64(vals.size), _p(gid), _p(ck), _p(vals), _I64(K), _p(v), _I64(g),
                              _p(y), _p(ya)), "ttv")
    return {"i": gi, "j": gj, "vals": y, "abs": ya}


def ttm(ci, cj, ck, vals, dims: Sequence[int], U) -> Dict[str, np.ndarray]:
    """Y(i,j,r) = sum_k X(i,j,k) U(k,r); one row of R values per distinct (i,j)."""
    ck, vals, U = _i32(ck), _f64(vals), _f64(U)
    K = int(dims[2])
    assert U.ndim == 2 and U.shape[0] == K
    R = U.shape[1]
    gid, gi, gj = group_pairs(ci, cj)
    g = gi.size
    Y, Ya = np.empty((g, R)), np.empty((g, R))
    _check(_load().oracle_ttm(_I64(vals.size), _p(gid), _p(ck), _p(vals), _I64(K), _I64(R), _p(U),
                              _I64(g), _p(Y), _p(Ya)), "ttm")
    return {"i": gi, "j": gj, "vals": Y, "abs": Ya}


def mttkrp(ci, cj, ck, vals, dims: Sequence[int], B, C) -> Tuple[np.ndarray, np.ndarray]:
    """M(i,r) = sum_{j,k} X(i,j,k) B(j,r) C(k,r); returns (M, A) of shape (I, R)."""
    ci, cj, ck, vals, B, C = _i32(ci), _i32(cj), _i32(ck), _f64(vals), _f64(B), _f64(C)
    I, J, K = (int(d) for d in dims)
    assert B.ndim == 2 and C.ndim == 2 and B.shape[0] == J and C.shape[0] == K and B.shape[1] == C.shape[1]
    R = B.shape[1]
    M, Ma = np.empty((I, R)), np.empty((I, R))
    _check(_load().oracle_mttkrp(_I64(vals.size), _p(ci), _p(cj), _p(ck), _p(vals), _I64(I), _I64(J),
                                 _I64(K), _I64(R), _p(B), _p(C), _p(M), _p(Ma)), "mttkrp")
    return M, Ma


# ---- any mode (Section 8.2 writes TTV / TTM for a general mode n and spells out n = 1) -----------------
# Only the roles of the coordinate arrays change: the contracted (or, for MTTKRP, the output) mode
# takes the place the functions above give to their fixed mode, the other two keep their order.
def _other_modes(mode: int) -> Tuple[int, int]:
    assert mode in (0, 1, 2)
    a, b = [m for m in range(3) if m != mode]
    return a, b


def ttv_mode(coords, vals, dims: Sequence[int], mode: int, v) -> Dict[str, np.ndarray]:
    """Y = X x_mode v: the sum runs over mode `mode` (0-based); the output lists the distinct
    coordinate pairs of the two remaining modes (in their original order), lexicographically."""
    a, b = _other_modes(mode)
    return ttv(coords[a], coords[b], coords[mode], vals, (dims[a], dims[b], dims[mode]), v)


def ttm_mode(coords, vals, dims: Sequence[int], mode: int, U) -> Dict[str, np.ndarray]:
    """Y = X x_mode U with U of shape (dims[mode], R): R values per distinct pair of the other modes."""
    a, b = _other_modes(mode)
    return ttm(coords[a], coords[b], coords[mode], vals, (dims[a], dims[b], dims[mode]), U)


def mttkrp_mode(coords, vals, dims: Sequence[int], mode: int, factors) -> Tuple[np.ndarray, np.ndarray]:
    """M(i_mode, r) = sum over the other two modes of X(i0,i1,i2) * F_a(i_a, r) * F_b(i_b, r),
    factors indexed by mode (factors[mode] unused); returns (M, A) of shape (dims[mode], R)."""
    a, b = _other_modes(mode)
    return mttkrp(coords[mode], coords[a], coords[b], vals, (dims[mode], dims[a], dims[b]), factors[a], factors[b])


def walk(tags: Sequence[int], pos: Sequence[Optional[np.ndarray]], crd: Sequence[Optional[np.ndarray]],
         nvals: int) -> Tuple[np.ndarray, np.ndarray]:
    """Expand per-level storage to coordinates: (coords[nvals, order], times each value was reached)."""
    order = len(tags)
    tg = _i32(list(tags))
    keep: List[np.ndarray] = []
    pos_ptrs = (ctypes.c_void_p * order)()
    crd_ptrs = (ctypes.c_void_p * order)()
    pos_len = (ctypes.c_int64 * order)()
    crd_len = (ctypes.c_int64 * order)()
    for l in range(order):
        for arr, ptrs, lens in ((pos[l], pos_ptrs, pos_len), (crd[l], crd_ptrs, crd_len)):
            if arr is None:
                ptrs[l], lens[l] = None, 0
            else:
                a = _i32(arr)
                keep.append(a)
                ptrs[l], lens[l] = a.ctypes.data, a.size
    coords = np.zeros((nvals, order), dtype=np.int32)
    seen = np.zeros(max(nvals, 1), dtype=np.int32)
    _check(_load().oracle_walk(ctypes.c_int(order), _p(tg), pos_ptrs, pos_len, crd_ptrs, crd_len,
                               _I64(nvals), _p(coords), _p(seen)), "walk")
    return coords, seen[:nvals]


def compressed_pair_levels(gi: np.ndarray, gj: np.ndarray) -> Dict[str, np.ndarray]:
    """[CU, CU] storage of a sorted list of distinct (i, j) pairs: the expected structure of a
    sparse TTV/TTM result whose input compresses both leading modes.  Level 1 keeps each
    distinct i once; pos2[m]..pos2[m+1] delimits the pairs of the m-th stored i (Section 4, CU)."""
    gi, gj = np.asarray(gi, dtype=np.int32), np.asarray(gj, dtype=np.int32)
    n = gi.size
    if n == 0:
        heads = np.zeros(0, dtype=np.int64)
    else:
        heads = np.flatnonzero(np.concatenate(([True], gi[1:] != gi[:-1])))
    pos2 = np.concatenate((heads, [n])).astype(np.int32)
    return {"pos1": np.array([0, heads.size], dtype=np.int32), "crd1": gi[heads].copy(),
            "pos2": pos2, "crd2": gj.copy()}
