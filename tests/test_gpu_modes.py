"""GPU parity for the operations along any mode, reached by re-storing the tensor in another level
order (comet_tensor_reorder), and for the conversions the same call performs.

Index results (the new pos / crd arrays) are compared bit for bit with the level arrays packed on
the CPU from the permuted, sorted coordinate list, and walked by the oracle back to the original
coordinates; values against the oracle's mode-n sums with the tolerance of tests/util.py.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from synth import formats as fmt
from synth import generate as gen
from util import assert_index_equal, assert_values_close, np_

from test_gpu_parity import TENSOR_CASES, MATRIX_CASES

pytestmark = pytest.mark.gpu

PERMS = list(itertools.permutations(range(3)))
CASES = ["zipf_ttv", "zipf_mttkrp", "mode_of_two", "single_slice", "long_fiber", "empty", "single"]


@pytest.fixture(scope="module")
def comet():
    from paper_2102_05187_amd import build
    build.build_if_missing()
    import paper_2102_05187_amd as c
    return c


def say(msg):
    print(msg, flush=True)


def dev(t):
    return t.to("cuda")


def sorted_by(coords, vals, order):
    """The coordinate list sorted lexicographically by coords[order[0]], coords[order[1]], ..."""
    if vals.numel() == 0:
        return [coords[m] for m in order], vals
    keys = np.stack([np_(coords[m]) for m in reversed(order)])
    perm = torch.from_numpy(np.lexsort(keys))
    return [coords[m][perm] for m in order], vals[perm]


def source_handle(comet, dims, coords, vals, layout):
    i, j, k = coords
    if layout == "csf":
        return comet.from_levels(fmt.pack_csf3(dims, i, j, k, vals).to("cuda"))
    if layout == "coo":
        return comet.from_levels(fmt.pack_coo(dims, (i, j, k), vals).to("cuda"))
    g = torch.Generator().manual_seed(11)
    p = torch.randperm(vals.numel(), generator=g)
    L = fmt.pack_coo(dims, (i[p], j[p], k[p]), vals[p]).to("cuda")
    return comet.from_levels(L, flags=0)           # not sorted: must not be validated as a sorted list


def check_levels(T, want):
    assert T.levels() == list(want.tags)
    assert T.dims() == list(want.dims)
    for l in range(len(want.dims)):
        for what, got, ref in (("pos", T.pos(l), want.pos[l]), ("crd", T.crd(l), want.crd[l])):
            assert (got is None) == (ref is None), "%s[%d] present on one side only" % (what, l)
            if ref is not None:
                assert_index_equal(np_(got), np_(ref), "%s[%d]" % (what, l))
    assert np.array_equal(np_(T.vals()), np_(want.vals))      # values are moved, never recomputed


@pytest.mark.parametrize("layout", ["csf", "coo", "coo_shuffled"])
@pytest.mark.parametrize("perm", PERMS)
@pytest.mark.parametrize("name", CASES)
def test_reorder_builds_the_expected_levels(comet, name, perm, layout):
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    say("reorder case=%s perm=%s layout=%s nnz=%d" % (name, perm, layout, vals.numel()))
    X = source_handle(comet, dims, (i, j, k), vals, layout)
    T = comet.comet_tensor_reorder(X, perm)
    torch.cuda.synchronize()
    assert T.mode_of_level() == list(perm)
    (a, b, c), sv = sorted_by((i, j, k), vals, perm)
    pdims = [dims[m] for m in perm]
    check_levels(T, fmt.pack_csf3(pdims, a, b, c, sv))
    # the oracle's walk of the new levels visits every value once, at the permuted coordinates
    tags = T.levels()
    coords, times = oracle.walk(tags, [np_(T.pos(l)) for l in range(3)], [np_(T.crd(l)) for l in range(3)],
                                int(vals.numel()))
    assert np.all(times == 1)
    for l, m in enumerate(perm):
        assert_index_equal(coords[:, l], np_((a, b, c)[l]), "walked coordinate of mode %d" % m)


@pytest.mark.parametrize("R", [1, 16])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("name", CASES)
def test_ttv_ttm_along_any_mode(comet, name, mode, R):
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    say("ttv/ttm case=%s mode=%d R=%d nnz=%d" % (name, mode, R, vals.numel()))
    X = source_handle(comet, dims, (i, j, k), vals, "csf")
    a, b = [m for m in range(3) if m != mode]
    Xr = comet.comet_tensor_reorder(X, (a, b, mode))
    coords = (np_(i), np_(j), np_(k))
    if R == 1:
        v = gen.dense_operand(21, mode, (dims[mode],))
        Y = comet.comet_ttv(Xr, mode, dev(v))
        ref = oracle.ttv_mode(coords, np_(vals), dims, mode, np_(v))
        got = np_(Y.vals())
    else:
        U = gen.dense_operand(22, mode, (dims[mode], R))
        Y = comet.comet_ttm(Xr, mode, dev(U))
        ref = oracle.ttm_mode(coords, np_(vals), dims, mode, np_(U))
        got = np_(Y.vals()).reshape(-1, R)
        assert Y.levels() == [1, 1, 0] and Y.dims() == [dims[a], dims[b], R]
    torch.cuda.synchronize()
    want = oracle.compressed_pair_levels(ref["i"], ref["j"])
    assert Y.mode_of_level()[:2] == [a, b]
    assert_index_equal(np_(Y.pos(0)), want["pos1"], "pos1")
    assert_index_equal(np_(Y.crd(0)), want["crd1"], "crd1")
    assert_index_equal(np_(Y.pos(1)), want["pos2"], "pos2")
    assert_index_equal(np_(Y.crd(1)), want["crd2"], "crd2")
    assert_values_close(got, ref["vals"], ref["abs"], "mode-%d contraction of %s" % (mode, name))


@pytest.mark.parametrize("R", [8, 64])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("name", CASES)
def test_mttkrp_for_any_mode(comet, name, mode, R):
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    say("mttkrp case=%s mode=%d R=%d nnz=%d" % (name, mode, R, vals.numel()))
    X = source_handle(comet, dims, (i, j, k), vals, "coo")
    a, b = [m for m in range(3) if m != mode]
    Xr = comet.comet_tensor_reorder(X, (mode, a, b))
    F = [gen.dense_operand(23, m, (dims[m], R)) for m in range(3)]
    M = torch.full((dims[mode], R), float("nan"), dtype=torch.float64, device="cuda")
    comet.comet_mttkrp(Xr, mode, [None if m == mode else dev(F[m]) for m in range(3)], M)
    torch.cuda.synchronize()
    ref, absum = oracle.mttkrp_mode((np_(i), np_(j), np_(k)), np_(vals), dims, mode, [np_(f) for f in F])
    assert_values_close(np_(M), ref, absum, "mode-%d mttkrp of %s" % (mode, name))


@pytest.mark.parametrize("layout", ["csr", "dcsr", "coo", "coo_shuffled"])
@pytest.mark.parametrize("name", ["zipf_rows", "edge_lengths", "hypersparse", "empty", "single"])
def test_matrix_conversion_and_transpose(comet, name, layout):
    (nrows, ncols), (rows, cols, vals) = MATRIX_CASES[name]
    say("matrix reorder case=%s layout=%s nnz=%d" % (name, layout, vals.numel()))
    if layout == "csr":
        X = comet.from_levels(fmt.pack_csr(nrows, ncols, rows, cols, vals).to("cuda"))
    elif layout == "dcsr":
        X = comet.from_levels(fmt.pack_dcsr(nrows, ncols, rows, cols, vals).to("cuda"))
    elif layout == "coo":
        X = comet.from_levels(fmt.pack_coo((nrows, ncols), (rows, cols), vals).to("cuda"))
    else:
        p = torch.randperm(vals.numel(), generator=torch.Generator().manual_seed(12))
        X = comet.from_levels(fmt.pack_coo((nrows, ncols), (rows[p], cols[p]), vals[p]).to("cuda"), flags=0)
    same = comet.comet_tensor_reorder(X, (0, 1))
    check_levels(same, fmt.pack_dcsr(nrows, ncols, rows, cols, vals))
    At = comet.comet_tensor_reorder(X, (1, 0))
    assert At.mode_of_level() == [1, 0]
    keys = np.lexsort(np.stack([np_(rows), np_(cols)])) if vals.numel() else np.zeros(0, dtype=np.int64)
    perm = torch.from_numpy(keys)
    check_levels(At, fmt.pack_dcsr(ncols, nrows, cols[perm], rows[perm], vals[perm]))
    # y = A^T x through the transposed storage
    x = gen.dense_operand(24, 0, (nrows,))
    y = comet.comet_spmv(At, dev(x))
    torch.cuda.synchronize()
    ref, absum = oracle.spmv(np_(cols), np_(rows), np_(vals), (ncols, nrows), np_(x))
    assert_values_close(np_(y), ref, absum, "transposed spmv %s" % name)


@pytest.mark.parametrize("target", ["csr", "dcsr", "coo"])
@pytest.mark.parametrize("layout", ["csr", "dcsr", "coo_shuffled"])
@pytest.mark.parametrize("name", ["zipf_rows", "edge_lengths", "hypersparse", "empty", "single"])
def test_matrix_format_conversion(comet, name, layout, target):
    """COO (in any order) / CSR / DCSR to CSR / DCSR / sorted COO, straight and transposed: level arrays
    bit for bit against the packers, then a product through the converted handle against the oracle."""
    (nrows, ncols), (rows, cols, vals) = MATRIX_CASES[name]
    say("convert case=%s %s -> %s nnz=%d" % (name, layout, target, vals.numel()))
    if layout == "csr":
        X = comet.from_levels(fmt.pack_csr(nrows, ncols, rows, cols, vals).to("cuda"))
    elif layout == "dcsr":
        X = comet.from_levels(fmt.pack_dcsr(nrows, ncols, rows, cols, vals).to("cuda"))
    else:
        p = torch.randperm(vals.numel(), generator=torch.Generator().manual_seed(13))
        X = comet.from_levels(fmt.pack_coo((nrows, ncols), (rows[p], cols[p]), vals[p]).to("cuda"), flags=0)
    tags = {"csr": [0, 1], "dcsr": [1, 1], "coo": [2, 3]}[target]
    pack = {"csr": fmt.pack_csr, "dcsr": fmt.pack_dcsr,
            "coo": lambda a, b, r, c, v: fmt.pack_coo((a, b), (r, c), v)}[target]
    T = comet.comet_tensor_convert(X, (0, 1), tags)
    check_levels(T, pack(nrows, ncols, rows, cols, vals))
    keys = np.lexsort(np.stack([np_(rows), np_(cols)])) if vals.numel() else np.zeros(0, dtype=np.int64)
    perm = torch.from_numpy(keys)
    Tt = comet.comet_tensor_convert(X, (1, 0), tags)
    check_levels(Tt, pack(ncols, nrows, cols[perm], rows[perm], vals[perm]))
    assert Tt.mode_of_level() == [1, 0]
    if target != "coo":
        x = gen.dense_operand(25, 0, (ncols,))
        y = comet.comet_spmv(T, dev(x))
        torch.cuda.synchronize()
        ref, absum = oracle.spmv(np_(rows), np_(cols), np_(vals), (nrows, ncols), np_(x))
        assert_values_close(np_(y), ref, absum, "spmv through converted %s" % target)


@pytest.mark.parametrize("name", ["zipf_ttv", "mode_of_two", "empty", "single"])
def test_tensor_to_sorted_coordinate_list(comet, name):
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    X = source_handle(comet, dims, (i, j, k), vals, "csf")
    for perm in ((0, 1, 2), (2, 0, 1)):
        T = comet.comet_tensor_convert(X, perm, [2, 3, 3])
        (a, b, c), sv = sorted_by((i, j, k), vals, perm)
        check_levels(T, fmt.pack_coo([dims[m] for m in perm], (a, b, c), sv))
        if name != "empty":                      # and it is accepted as a validated sorted list again
            v = gen.dense_operand(26, 0, (dims[perm[2]],))
            Y = comet.comet_ttv(T, perm[2], dev(v))
            # the result follows the handle's level order: pairs of (mode perm[0], mode perm[1])
            co = (i, j, k)
            ref = oracle.ttv(np_(co[perm[0]]), np_(co[perm[1]]), np_(co[perm[2]]), np_(vals),
                             [dims[m] for m in perm], np_(v))
            torch.cuda.synchronize()
            assert_index_equal(np_(Y.crd(0)), ref["i"], "coo result crd0")
            assert_index_equal(np_(Y.crd(1)), ref["j"], "coo result crd1")
            assert_values_close(np_(Y.vals()), ref["vals"], ref["abs"], "ttv on converted coo")
    with pytest.raises(comet.CometError) as e:
        comet.comet_tensor_convert(X, (0, 1, 2), [0, 1, 1])
    assert e.value.status == 4


@pytest.mark.parametrize("perm", [(0, 1, 2), (2, 0, 1), (1, 2, 0)])
@pytest.mark.parametrize("dims", [(2_902_330, 2_143_368, 25_495_389), (532_924, 17_262_471, 2_480_308),
                                  ((1 << 31) - 1, (1 << 31) - 1, (1 << 31) - 1)])
def test_reorder_with_mode_sizes_beyond_one_sort_key(comet, dims, perm):
    """Mode sizes like those of the paper's largest tensors (Table "Description of sparse tensors"): the
    three coordinates need 69 / 67 / 93 bits, more than one 64-bit sort key; the nonzeros (few, spread over
    the whole index range, some sharing root and middle coordinates) must still come out in order."""
    n = 50_000
    raw = gen.rng.uniform01(77, 5, 3 * n).reshape(3, n)
    co = [torch.clamp((raw[m] * dims[m]).to(torch.int64), max=dims[m] - 1) for m in range(3)]
    co[0][: n // 2] = co[0][0]                   # half the nonzeros in one slice ...
    co[1][: n // 4] = co[1][0]                   # ... a quarter in one fiber of it
    co[2][: n // 4] = (torch.arange(n // 4, dtype=torch.int64) * 97) % dims[2]      # (distinct inside that fiber)
    key = [tuple(int(c[p]) for c in co) for p in range(n)]
    assert len(set(key)) == n                    # distinct coordinates
    vals = gen.rng.uniform_pm1(77, 6, n)
    L = fmt.pack_coo(dims, tuple(co), vals).to("cuda")
    X = comet.from_levels(L, flags=0)            # unsorted list
    say("wide-key reorder dims=%s perm=%s" % (dims, perm))
    T = comet.comet_tensor_reorder(X, perm)
    (a, b, c), sv = sorted_by(tuple(co), vals, perm)
    check_levels(T, fmt.pack_csf3([dims[m] for m in perm], a, b, c, sv))
    Tc = comet.comet_tensor_convert(X, perm, [2, 3, 3])
    check_levels(Tc, fmt.pack_coo([dims[m] for m in perm], (a, b, c), sv))
    # and an operation on the result: TTV along the last level's mode (operand far larger than LDS)
    if dims[perm[2]] < (1 << 27):
        v = gen.dense_operand(78, 0, (dims[perm[2]],))
        Y = comet.comet_ttv(T, perm[2], dev(v))
        ref = oracle.ttv(np_(a), np_(b), np_(c), np_(sv), [dims[m] for m in perm], np_(v))
        torch.cuda.synchronize()
        assert_values_close(np_(Y.vals()), ref["vals"], ref["abs"], "ttv after wide-key reorder")


def test_reorder_errors(comet):
    dims, (i, j, k, vals) = TENSOR_CASES["mode_of_two"]
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, vals).to("cuda"))
    for bad in ((0, 1, 1), (0, 1, 3), (-1, 0, 1)):
        with pytest.raises(comet.CometError) as e:
            comet.comet_tensor_reorder(X, bad)
        assert e.value.status == 1
    # the same coordinate stored twice in a coordinate list
    ci = torch.tensor([1, 0, 1], dtype=torch.int64)
    L = fmt.pack_coo((3, 3, 3), (ci, ci, ci), torch.ones(3, dtype=torch.float64)).to("cuda")
    with pytest.raises(comet.CometError) as e:
        comet.comet_tensor_reorder(comet.from_levels(L, flags=0), (0, 1, 2))
    assert e.value.status == 2
    # an operation names a mode that the handle does not keep in the required level
    Xr = comet.comet_tensor_reorder(X, (1, 2, 0))
    with pytest.raises(comet.CometError) as e:
        comet.comet_ttv(Xr, 2, torch.ones(dims[2], dtype=torch.float64, device="cuda"))
    assert e.value.status == 4
    with pytest.raises(comet.CometError) as e:
        comet.comet_mttkrp(Xr, 0, [None, torch.ones((dims[1], 4), dtype=torch.float64, device="cuda"),
                                   torch.ones((dims[2], 4), dtype=torch.float64, device="cuda")])
    assert e.value.status == 4
    # a reordered handle can be reordered again; modes keep their original numbers
    back = comet.comet_tensor_reorder(Xr, (0, 1, 2))
    check_levels(back, fmt.pack_csf3(dims, i, j, k, vals))
