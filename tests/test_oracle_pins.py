"""Pins of the CPU oracle to things other than itself (CPU only).

  * exact rational brute force over the dense array (tiny tensors, all densities),
  * a hand-worked example stored under tests/golden/,
  * library routines where the operation reduces to one (SciPy CSR product, numpy einsum),
  * invariants and special cases that follow from the definitions,
  * planted mistakes: a transposed operand / swapped index must be caught by the pins above.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from synth import generate as gen
from synth import formats as fmt
from util import assert_values_close, np_

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")


# ------------------------------------------------------------------------------------------
# exact brute force on the dense array (Section 8.2 definitions, literally)
# ------------------------------------------------------------------------------------------
def _dense_from_coo(shape, coords, vals):
    Xd = np.zeros(shape)
    for idx, a in zip(zip(*coords), vals):
        assert Xd[idx] == 0.0
        Xd[idx] = a
    return Xd


def _fr(x):
    return Fraction(float(x))


def brute_spmm(Xd, U):
    I, J = Xd.shape
    R = U.shape[1]
    out = np.zeros((I, R))
    for i in range(I):
        for r in range(R):
            out[i, r] = float(sum((_fr(Xd[i, j]) * _fr(U[j, r]) for j in range(J)), Fraction(0)))
    return out


def brute_ttm(Xd, U):
    I, J, K = Xd.shape
    R = U.shape[1]
    out = np.zeros((I, J, R))
    for i in range(I):
        for j in range(J):
            for r in range(R):
                out[i, j, r] = float(sum((_fr(Xd[i, j, k]) * _fr(U[k, r]) for k in range(K)), Fraction(0)))
    return out


def brute_mttkrp(Xd, B, C):
    I, J, K = Xd.shape
    R = B.shape[1]
    out = np.zeros((I, R))
    for i in range(I):
        for r in range(R):
            out[i, r] = float(sum((_fr(Xd[i, j, k]) * _fr(B[j, r]) * _fr(C[k, r])
                                   for j in range(J) for k in range(K)), Fraction(0)))
    return out


TIGHT = 4 * np.finfo(np.float64).eps   # the compensated oracle should sit within a few ulp of exact


def _assert_tight(got, exact, absum):
    got, exact, absum = map(np.asarray, (got, exact, absum))
    assert np.all(np.abs(got - exact) <= TIGHT * np.maximum(absum, np.abs(exact)) + 1e-300)


@pytest.mark.parametrize("density", [0.0, 0.1, 0.5, 1.0])
@pytest.mark.parametrize("shape", [(5, 7), (8, 3), (1, 6)])
def test_matrix_ops_match_exact_dense_brute_force(density, shape):
    seed = int(density * 10) + shape[0]
    rows, cols, vals = gen.bernoulli_matrix(shape[0], shape[1], density, seed)
    rows, cols, vals = np_(rows), np_(cols), np_(vals)
    Xd = _dense_from_coo(shape, (rows, cols), vals)
    U = np_(gen.dense_operand(seed, 0, (shape[1], 3)))
    Y, Ya = oracle.spmm(rows, cols, vals, shape, U)
    _assert_tight(Y, brute_spmm(Xd, U), Ya)
    y, ya = oracle.spmv(rows, cols, vals, shape, U[:, 1])
    _assert_tight(y, brute_spmm(Xd, U[:, 1:2])[:, 0], ya)
    assert np.allclose(Ya, np.abs(Xd) @ np.abs(U))


@pytest.mark.parametrize("density", [0.0, 0.1, 0.5, 1.0])
@pytest.mark.parametrize("dims", [(3, 4, 5), (6, 2, 7), (2, 8, 1)])
def test_tensor_ops_match_exact_dense_brute_force(density, dims):
    seed = int(density * 10) + dims[0]
    i, j, k, vals = (np_(t) for t in gen.bernoulli_tensor3(dims, density, seed))
    Xd = _dense_from_coo(dims, (i, j, k), vals)
    U = np_(gen.dense_operand(seed, 0, (dims[2], 3)))
    B = np_(gen.dense_operand(seed, 1, (dims[1], 3)))
    full = brute_ttm(Xd, U)
    Y = oracle.ttm(i, j, k, vals, dims, U)
    # the sparse result lists exactly the (i,j) pairs that hold a stored nonzero, in order
    pairs = sorted(set(zip(i.tolist(), j.tolist())))
    assert list(zip(Y["i"].tolist(), Y["j"].tolist())) == pairs
    for g, (a, b) in enumerate(pairs):
        _assert_tight(Y["vals"][g], full[a, b], Y["abs"][g])
    mask = np.ones(dims[:2], bool)
    for a, b in pairs:
        mask[a, b] = False
    assert np.all(full[mask] == 0.0)
    yv = oracle.ttv(i, j, k, vals, dims, U[:, 2])
    assert list(zip(yv["i"].tolist(), yv["j"].tolist())) == pairs
    for g, (a, b) in enumerate(pairs):
        _assert_tight(yv["vals"][g], full[a, b, 2], yv["abs"][g])
    M, Ma = oracle.mttkrp(i, j, k, vals, dims, B, U)
    _assert_tight(M, brute_mttkrp(Xd, B, U), Ma)


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("dims", [(3, 4, 5), (6, 2, 7)])
def test_any_mode_ops_match_exact_dense_brute_force(mode, dims):
    """Mode-n TTV / TTM / MTTKRP against the literal sums on the dense array with the contracted
    (output) axis moved to the place the mode-3 (mode-1) brute force expects it."""
    seed = 40 + mode + dims[0]
    coords = tuple(np_(t) for t in gen.bernoulli_tensor3(dims, 0.4, seed))
    vals, coords = coords[3], coords[:3]
    Xd = _dense_from_coo(dims, coords, vals)
    F = [np_(gen.dense_operand(seed, m, (dims[m], 3))) for m in range(3)]
    a, b = [m for m in range(3) if m != mode]
    full = brute_ttm(np.moveaxis(Xd, mode, 2), F[mode])          # indexed (i_a, i_b, r)
    Y = oracle.ttm_mode(coords, vals, dims, mode, F[mode])
    pairs = sorted(set(zip(coords[a].tolist(), coords[b].tolist())))
    assert list(zip(Y["i"].tolist(), Y["j"].tolist())) == pairs
    for g, (x, y) in enumerate(pairs):
        _assert_tight(Y["vals"][g], full[x, y], Y["abs"][g])
    yv = oracle.ttv_mode(coords, vals, dims, mode, F[mode][:, 1])
    assert list(zip(yv["i"].tolist(), yv["j"].tolist())) == pairs
    for g, (x, y) in enumerate(pairs):
        _assert_tight(yv["vals"][g], full[x, y, 1], yv["abs"][g])
    M, Ma = oracle.mttkrp_mode(coords, vals, dims, mode, F)
    _assert_tight(M, brute_mttkrp(np.moveaxis(Xd, mode, 0), F[a], F[b]), Ma)


# ------------------------------------------------------------------------------------------
# hand-worked example
# ------------------------------------------------------------------------------------------
def test_hand_example_matrix():
    g = json.load(open(GOLD))["matrix"]
    c = g["coo"]
    y, _ = oracle.spmv(c["rows"], c["cols"], c["vals"], g["shape"], g["x"])
    assert y.tolist() == g["spmv"]
    Y, _ = oracle.spmm(c["rows"], c["cols"], c["vals"], g["shape"], np.array(g["B"], float))
    assert Y.tolist() == g["spmm"]


def test_hand_example_tensor():
    g = json.load(open(GOLD))["tensor"]
    c = g["coo"]
    y = oracle.ttv(c["i"], c["j"], c["k"], c["vals"], g["shape"], g["v"])
    assert (y["i"].tolist(), y["j"].tolist(), y["vals"].tolist()) == (g["ttv"]["i"], g["ttv"]["j"], g["ttv"]["vals"])
    Y = oracle.ttm(c["i"], c["j"], c["k"], c["vals"], g["shape"], np.array(g["U"], float))
    assert (Y["i"].tolist(), Y["j"].tolist(), Y["vals"].tolist()) == (g["ttm"]["i"], g["ttm"]["j"], g["ttm"]["vals"])
    M, _ = oracle.mttkrp(c["i"], c["j"], c["k"], c["vals"], g["shape"], np.array(g["Bf"], float),
                         np.array(g["Cf"], float))
    assert M.tolist() == g["mttkrp"]


_TAG = {"D": 0, "CU": 1, "CN": 2, "S": 3}


def _lv(d):
    arr = lambda a: None if a is None else np.array(a, dtype=np.int32)
    return [_TAG[t] for t in d["tags"]], [arr(p) for p in d["pos"]], [arr(c) for c in d["crd"]]


def test_hand_example_level_walk():
    """Each storage of the same matrix/tensor expands to the same coordinate list."""
    g = json.load(open(GOLD))
    m = g["matrix"]
    want = np.stack([m["coo"]["rows"], m["coo"]["cols"]], 1)
    for name in ("csr", "dcsr", "coo_levels"):
        tags, pos, crd = _lv(m[name])
        coords, seen = oracle.walk(tags, pos, crd, 5)
        assert np.array_equal(coords, want), name
        assert np.all(seen == 1)
    t = g["tensor"]
    tags, pos, crd = _lv(t["csf"])
    coords, seen = oracle.walk(tags, pos, crd, 6)
    assert np.array_equal(coords, np.stack([t["coo"]["i"], t["coo"]["j"], t["coo"]["k"]], 1))
    assert np.all(seen == 1)


def test_hand_example_compressed_levels():
    """The hand-written [CU,CU,CU] arrays of the example pin both the oracle's expected-structure helper and
    the packer that feeds the GPU tests, array by array."""
    t = json.load(open(GOLD))["tensor"]
    c, want = t["coo"], t["csf"]
    # expected structure of a sparse result over the distinct (i, j) pairs = levels 1 and 2 of the example
    lv = oracle.compressed_pair_levels(np.array(t["ttv"]["i"]), np.array(t["ttv"]["j"]))
    assert lv["pos1"].tolist() == want["pos"][0] and lv["crd1"].tolist() == want["crd"][0]
    assert lv["pos2"].tolist() == want["pos"][1] and lv["crd2"].tolist() == want["crd"][1]
    assert all(lv[k].dtype == np.int32 for k in lv)
    L = fmt.pack_csf3(t["shape"], torch.tensor(c["i"]), torch.tensor(c["j"]), torch.tensor(c["k"]),
                          torch.tensor(c["vals"], dtype=torch.float64))
    assert list(L.tags) == [1, 1, 1]
    for l in range(3):
        assert L.pos[l].tolist() == want["pos"][l], "pos of level %d" % l
        assert L.crd[l].tolist() == want["crd"][l], "crd of level %d" % l
        assert L.pos[l].dtype == torch.int32 and L.crd[l].dtype == torch.int32
    assert L.vals.tolist() == c["vals"]
    m = json.load(open(GOLD))["matrix"]
    mc = m["coo"]
    args = (m["shape"][0], m["shape"][1], torch.tensor(mc["rows"]), torch.tensor(mc["cols"]), torch.tensor(mc["vals"], dtype=torch.float64))
    for pack, name in ((fmt.pack_csr, "csr"), (fmt.pack_dcsr, "dcsr")):
        P = pack(*args)
        for l in range(2):
            assert (None if P.pos[l] is None else P.pos[l].tolist()) == m[name]["pos"][l], name
            assert (None if P.crd[l] is None else P.crd[l].tolist()) == m[name]["crd"][l], name
    # a planted mistake: the pair list with its columns swapped must not give the example's arrays
    bad = oracle.compressed_pair_levels(np.array(t["ttv"]["j"]), np.array(t["ttv"]["i"]))
    assert bad["crd1"].tolist() != want["crd"][0] or bad["pos2"].tolist() != want["pos"][1]


def test_compressed_unique_stores_a_shared_row_coordinate_once():
    """Section 4, CU: two nonzeros of one row share a single stored row coordinate;
    CN: pos holds only the start and the extent of crd; S: one coordinate per parent position."""
    rows, cols = torch.tensor([3, 3, 7]), torch.tensor([1, 5, 2])
    vals = torch.tensor([1.0, 2.0, 3.0], dtype=torch.float64)
    T = fmt.pack_dcsr(9, 6, rows, cols, vals)
    assert T.crd[0].tolist() == [3, 7] and T.pos[0].tolist() == [0, 2] and T.pos[1].tolist() == [0, 2, 3]
    C = fmt.pack_coo((9, 6), (rows, cols), vals)
    assert C.pos[0].tolist() == [0, 3] and C.pos[1] is None and C.crd[0].tolist() == [3, 3, 7]
    R = fmt.pack_csr(9, 6, rows, cols, vals)
    assert R.pos[0].tolist() == [9] and R.crd[0] is None
    assert R.pos[1].tolist() == [0, 0, 0, 0, 2, 2, 2, 2, 3, 3]


def test_dense_leaf_level_indexes_row_major():
    """A [CU, D] tensor (dense trailing level, as in a TTM result): value position = parent*size + r
    (Section 6.2 Step II, dense index update)."""
    tags = [1, 0]
    pos = [np.array([0, 2], np.int32), np.array([3], np.int32)]
    crd = [np.array([4, 9], np.int32), None]
    coords, seen = oracle.walk(tags, pos, crd, 6)
    assert coords.tolist() == [[4, 0], [4, 1], [4, 2], [9, 0], [9, 1], [9, 2]]
    assert np.all(seen == 1)


# ------------------------------------------------------------------------------------------
# library routines
# ------------------------------------------------------------------------------------------
def test_spmv_spmm_against_scipy_csr():
    import scipy.sparse as sp
    c = gen.config_spmm(seed=3, scale=0.002, R=8)
    rows, cols, vals = (np_(t) for t in c["coo"])
    n = c["dims"][0]
    A = sp.csr_matrix((vals, (rows, cols)), shape=(n, n))
    B = np_(c["B"])
    Y, Ya = oracle.spmm(rows, cols, vals, (n, n), B)
    assert_values_close(A @ B, Y, Ya, "spmm vs scipy")
    y, ya = oracle.spmv(rows, cols, vals, (n, n), B[:, 0])
    assert_values_close(A @ B[:, 0], y, ya, "spmv vs scipy")


def test_tensor_ops_against_einsum():
    dims = (9, 11, 13)
    i, j, k, vals = (np_(t) for t in gen.bernoulli_tensor3(dims, 0.2, 5))
    Xd = _dense_from_coo(dims, (i, j, k), vals)
    U, B = np_(gen.dense_operand(5, 0, (13, 6))), np_(gen.dense_operand(5, 1, (11, 6)))
    Y = oracle.ttm(i, j, k, vals, dims, U)
    assert_values_close(Y["vals"], np.einsum("ijk,kr->ijr", Xd, U)[Y["i"], Y["j"]], Y["abs"], "ttm")
    y = oracle.ttv(i, j, k, vals, dims, U[:, 0])
    assert_values_close(y["vals"], np.einsum("ijk,k->ij", Xd, U[:, 0])[y["i"], y["j"]], y["abs"], "ttv")
    M, Ma = oracle.mttkrp(i, j, k, vals, dims, B, U)
    assert_values_close(M, np.einsum("ijk,jr,kr->ir", Xd, B, U), Ma, "mttkrp")


# ------------------------------------------------------------------------------------------
# invariants and special cases
# ------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def small_matrix():
    c = gen.config_spmm(seed=1, scale=0.001, R=4)
    return tuple(np_(t) for t in c["coo"]), c["dims"], np_(c["B"])


@pytest.fixture(scope="module")
def small_tensor():
    c = gen.config_mttkrp(seed=2, scale=2e-5, R=4, chunk=1 << 16)
    return tuple(np_(t) for t in c["coo"]), c["dims"], np_(c["B"]), np_(c["C"])


def test_spmv_of_ones_is_row_sums(small_matrix):
    (rows, cols, vals), (I, J), _ = small_matrix
    y, ya = oracle.spmv(rows, cols, vals, (I, J), np.ones(J))
    ref = np.zeros(I)
    np.add.at(ref, rows, vals)
    assert_values_close(ref, y, ya, "row sums")


def test_spmv_identity_returns_x():
    n = 17
    x = np_(gen.dense_operand(0, 0, (n,)))
    y, _ = oracle.spmv(np.arange(n), np.arange(n), np.ones(n), (n, n), x)
    assert np.array_equal(y, x)


def test_spmm_with_ones_repeats_row_sums_and_columns_are_spmv(small_matrix):
    """The paper's example program fills B with 1.0 (Listing 'example program'): every column of C
    is then the vector of row sums.  Column r of SpMM is SpMV with B[:, r]."""
    (rows, cols, vals), (I, J), B = small_matrix
    Y, Ya = oracle.spmm(rows, cols, vals, (I, J), np.ones((J, 3)))
    y1, _ = oracle.spmv(rows, cols, vals, (I, J), np.ones(J))
    for r in range(3):
        assert np.array_equal(Y[:, r], y1)
    Y, _ = oracle.spmm(rows, cols, vals, (I, J), B)
    for r in range(B.shape[1]):
        assert np.array_equal(Y[:, r], oracle.spmv(rows, cols, vals, (I, J), B[:, r])[0])


def test_ttm_columns_are_ttv_and_rank_one_ttm_is_ttv(small_tensor):
    (i, j, k, vals), dims, B, C = small_tensor
    Y = oracle.ttm(i, j, k, vals, dims, C)
    for r in range(C.shape[1]):
        y = oracle.ttv(i, j, k, vals, dims, C[:, r])
        assert np.array_equal(Y["vals"][:, r], y["vals"])
        assert np.array_equal(Y["i"], y["i"]) and np.array_equal(Y["j"], y["j"])


def test_ttm_one_hot_column_extracts_a_slice(small_tensor):
    (i, j, k, vals), dims, B, C = small_tensor
    k0 = int(k[len(k) // 2])
    U = np.zeros((dims[2], 1))
    U[k0, 0] = 1.0
    Y = oracle.ttm(i, j, k, vals, dims, U)
    got = {(a, b): v for a, b, v in zip(Y["i"], Y["j"], Y["vals"][:, 0]) if v != 0.0}
    want = {(a, b): v for a, b, c, v in zip(i, j, k, vals) if c == k0}
    assert got == want


def test_ttv_on_a_single_layer_tensor_scales_the_matrix():
    rows, cols, vals = (np_(t) for t in gen.bernoulli_matrix(7, 9, 0.3, 4))
    y = oracle.ttv(rows, cols, np.zeros_like(rows), vals, (7, 9, 1), np.array([2.5]))
    assert np.array_equal(y["vals"], 2.5 * vals)
    assert np.array_equal(y["i"], rows) and np.array_equal(y["j"], cols)


def test_mttkrp_rank_one_is_ttv_applied_twice(small_tensor):
    """M(i) = sum_j b_j (sum_k X(i,j,k) c_k): TTV along mode 3, then the matrix-vector product
    of the (i,j) result with b."""
    (i, j, k, vals), dims, B, C = small_tensor
    M, Ma = oracle.mttkrp(i, j, k, vals, dims, B[:, :1], C[:, :1])
    y = oracle.ttv(i, j, k, vals, dims, C[:, 0])
    m2, _ = oracle.spmv(y["i"], y["j"], y["vals"], dims[:2], B[:, 0])
    assert_values_close(m2, M[:, 0], Ma[:, 0], "mttkrp R=1")


def test_mttkrp_with_unit_B_is_row_sum_of_ttm_and_columns_are_independent(small_tensor):
    (i, j, k, vals), dims, B, C = small_tensor
    M, Ma = oracle.mttkrp(i, j, k, vals, dims, np.ones_like(B), C)
    Y = oracle.ttm(i, j, k, vals, dims, C)
    ref = np.zeros_like(M)
    np.add.at(ref, Y["i"], Y["vals"])
    assert_values_close(ref, M, Ma, "B=1")
    M4, _ = oracle.mttkrp(i, j, k, vals, dims, B, C)
    M2, _ = oracle.mttkrp(i, j, k, vals, dims, B[:, :2].copy(), C[:, :2].copy())
    assert np.array_equal(M4[:, :2], M2)


def test_linearity(small_tensor):
    (i, j, k, vals), dims, B, C = small_tensor
    u, w = C[:, 0], C[:, 1]
    a = oracle.ttv(i, j, k, vals, dims, u + w)
    b, c = oracle.ttv(i, j, k, vals, dims, u), oracle.ttv(i, j, k, vals, dims, w)
    assert_values_close(a["vals"], b["vals"] + c["vals"], b["abs"] + c["abs"], "additivity")
    d = oracle.ttv(i, j, k, 4.0 * vals, dims, u)     # scaling by a power of two is exact
    assert np.array_equal(d["vals"], 4.0 * b["vals"])


def test_storage_order_does_not_change_which_pairs_come_out(small_tensor):
    (i, j, k, vals), dims, B, C = small_tensor
    p = np.random.default_rng(0).permutation(len(vals))
    a = oracle.ttv(i, j, k, vals, dims, C[:, 0])
    b = oracle.ttv(i[p], j[p], k[p], vals[p], dims, C[:, 0])
    assert np.array_equal(a["i"], b["i"]) and np.array_equal(a["j"], b["j"])
    assert_values_close(b["vals"], a["vals"], a["abs"], "permuted storage order")


def test_compensated_sum_survives_cancellation():
    n = 4001
    vals = np.ones(n)
    x = np.concatenate(([1e16], np.ones(n - 2), [-1e16]))
    y, ya = oracle.spmv(np.zeros(n, int), np.arange(n), vals, (1, n), x)
    assert y[0] == float(n - 2)
    assert ya[0] == pytest.approx(2e16)


# ------------------------------------------------------------------------------------------
# pack -> walk is the identity for every supported level tuple
# ------------------------------------------------------------------------------------------
def test_pack_then_walk_is_identity():
    rows, cols, vals = gen.bernoulli_matrix(13, 11, 0.15, 8)
    want = np.stack([np_(rows), np_(cols)], 1)
    for T in (fmt.pack_csr(13, 11, rows, cols, vals), fmt.pack_dcsr(13, 11, rows, cols, vals),
              fmt.pack_coo((13, 11), (rows, cols), vals)):
        coords, seen = oracle.walk(T.tags, [np_(p) for p in T.pos], [np_(c) for c in T.crd], T.nnz)
        assert np.array_equal(coords, want), T.name
        assert np.all(seen == 1)
    dims = (6, 5, 9)
    i, j, k, vals = gen.bernoulli_tensor3(dims, 0.2, 9)
    want = np.stack([np_(i), np_(j), np_(k)], 1)
    for T in (fmt.pack_csf3(dims, i, j, k, vals), fmt.pack_coo(dims, (i, j, k), vals)):
        coords, seen = oracle.walk(T.tags, [np_(p) for p in T.pos], [np_(c) for c in T.crd], T.nnz)
        assert np.array_equal(coords, want), T.name
        assert np.all(seen == 1)


def test_csr_and_dcsr_of_one_matrix_give_the_same_product():
    rows, cols, vals = gen.bernoulli_matrix(20, 15, 0.05, 10)
    x = np_(gen.dense_operand(10, 0, (15,)))
    outs = []
    for T in (fmt.pack_csr(20, 15, rows, cols, vals), fmt.pack_dcsr(20, 15, rows, cols, vals)):
        coords, _ = oracle.walk(T.tags, [np_(p) for p in T.pos], [np_(c) for c in T.crd], T.nnz)
        outs.append(oracle.spmv(coords[:, 0], coords[:, 1], np_(T.vals), (20, 15), x)[0])
    assert np.array_equal(outs[0], outs[1])


def test_expected_output_structure_of_sparse_results(small_tensor):
    (i, j, k, vals), dims, B, C = small_tensor
    y = oracle.ttv(i, j, k, vals, dims, C[:, 0])
    lv = oracle.compressed_pair_levels(y["i"], y["j"])
    T = fmt.pack_csf3(dims, *(torch.from_numpy(a) for a in (i.astype(np.int64), j.astype(np.int64),
                                                           k.astype(np.int64), vals)))
    assert np.array_equal(lv["pos1"], np_(T.pos[0])) and np.array_equal(lv["crd1"], np_(T.crd[0]))
    assert np.array_equal(lv["pos2"], np_(T.pos[1])) and np.array_equal(lv["crd2"], np_(T.crd[1]))
    assert len(y["vals"]) == T.crd[1].numel() == len(set(zip(i.tolist(), j.tolist())))
    assert int(np_(T.pos[2])[-1]) == len(vals)


# ------------------------------------------------------------------------------------------
# planted mistakes: the pins above must notice them
# ------------------------------------------------------------------------------------------
def test_pins_catch_transposed_or_swapped_operands():
    shape = (5, 7)
    rows, cols, vals = (np_(t) for t in gen.bernoulli_matrix(*shape, 0.5, 11))
    Xd = _dense_from_coo(shape, (rows, cols), vals)
    U = np_(gen.dense_operand(11, 0, (7, 7)))
    exact = brute_spmm(Xd, U)
    wrong, _ = oracle.spmm(rows, cols, vals, shape, np.ascontiguousarray(U.T))   # transposed operand
    assert np.abs(wrong - exact).max() > 1e-3
    dims = (4, 4, 4)
    i, j, k, v = (np_(t) for t in gen.bernoulli_tensor3(dims, 0.5, 12))
    Xd = _dense_from_coo(dims, (i, j, k), v)
    B, C = np_(gen.dense_operand(12, 0, (4, 2))), np_(gen.dense_operand(12, 1, (4, 2)))
    exact = brute_mttkrp(Xd, B, C)
    swapped, _ = oracle.mttkrp(i, j, k, v, dims, C, B)                             # factors swapped
    assert np.abs(swapped - exact).max() > 1e-3
    moved, _ = oracle.mttkrp(j, i, k, v, dims, B, C)                               # wrong output mode
    assert np.abs(moved - exact).max() > 1e-3


@pytest.mark.parametrize("alpha,beta", [(1.0, 1.0), (-0.75, 2.5), (3.0, 0.0), (0.0, -1.5), (0.0, 0.0)])
def test_scaled_accumulating_result_matches_exact_brute_force(alpha, beta):
    """oracle.axpby (the in-place update of Section 6.2, Step III, with two scalars) against exact rational
    arithmetic on a small SpMM: alpha * A B + beta * C for every element; what is not to be read may be NaN."""
    shape = (6, 5)
    rows, cols, vals = gen.bernoulli_matrix(shape[0], shape[1], 0.4, 17)
    rows, cols, vals = np_(rows), np_(cols), np_(vals)
    Xd = _dense_from_coo(shape, (rows, cols), vals)
    U = np_(gen.dense_operand(17, 0, (shape[1], 3)))
    C0 = np_(gen.dense_operand(17, 1, (shape[0], 3)))
    Y, Ya = oracle.spmm(rows, cols, vals, shape, U)
    exact = np.zeros_like(C0)
    for i in range(shape[0]):
        for r in range(3):
            prod = sum((_fr(Xd[i, j]) * _fr(U[j, r]) for j in range(shape[1])), Fraction(0))
            exact[i, r] = float(_fr(alpha) * prod + _fr(beta) * _fr(C0[i, r]))
    old = C0.copy()
    if beta == 0.0:
        old[:] = np.nan                      # must not be read
    prod_in = Y.copy()
    if alpha == 0.0:
        prod_in[:] = np.nan                  # must not be read
    out, out_abs = oracle.axpby(alpha, prod_in, Ya, beta, old)
    assert np.all(np.isfinite(out))
    _assert_tight(out, exact, out_abs + 1e-300)
    want_abs = (abs(alpha) * (np.abs(Xd) @ np.abs(U)) if alpha != 0.0 else 0.0) + (np.abs(beta * C0) if beta != 0.0 else 0.0)
    assert np.allclose(out_abs, want_abs)


def test_accumulating_twice_doubles_the_product():
    """beta = 1 adds: starting from zeros, two accumulations of A x give exactly 2 A x (a power of two)."""
    rows, cols, vals = (np_(a) for a in gen.bernoulli_matrix(9, 7, 0.5, 5))
    x = np_(gen.dense_operand(5, 0, (7,)))
    y, ya = oracle.spmv(rows, cols, vals, (9, 7), x)
    once, _ = oracle.axpby(1.0, y, ya, 1.0, np.zeros(9))
    twice, _ = oracle.axpby(1.0, y, ya, 1.0, once)
    assert np.array_equal(once, y) and np.array_equal(twice, 2.0 * y)


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The C oracle, built with -fsanitize=address,undefined, runs every entry point on hand-made inputs
    (tests/sanitize/oracle_driver.c: values worked out by hand from Section 8.2, empty inputs, a coordinate out
    of range) without a report: no access outside the arrays, no leak, no undefined arithmetic."""
    import os
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", os.path.join(root, "oracle", "comet_oracle.c"),
           os.path.join(root, "tests", "sanitize", "oracle_driver.c"), "-lm", "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower():
        pytest.skip("sanitizer runtime not installed: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "ok" in run.stdout and "ERROR" not in run.stderr and "runtime error" not in run.stderr
