"""GPU parity: every operation through the C ABI against the CPU oracle, element by element.

Sizes here are small enough for the oracle to finish in well under a second while still spanning
several kernel tiles (4096 nonzeros each) and a ragged tail.  Index outputs must be bit-exact;
values must satisfy |gpu - ref| <= 1e-10*|ref| + 1e-12*A with A = sum |term| from the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
from synth import formats as fmt
from synth import generate as gen
from util import assert_index_equal, assert_values_close, np_

pytestmark = pytest.mark.gpu

# 1 = simple kernels, 2 = tiled with every specialisation, 3 = tiled in the plain per-tile form, 0 = the library's own choice
VARIANTS = [1, 2, 3, 0]


@pytest.fixture(scope="module")
def comet():
    from paper_2102_05187_amd import build
    build.build_if_missing()
    import paper_2102_05187_amd as c
    return c


def dev(t):
    return None if t is None else t.to("cuda")


def say(msg):
    print(msg, flush=True)


# ----------------------------------------------------------------------------------------------
# matrices
# ----------------------------------------------------------------------------------------------
def _matrix_cases():
    cases = {}
    c = gen.config_spmv(seed=0)
    cases["config1"] = (c["dims"], c["coo"])
    c = gen.config_spmm(seed=0, scale=0.004)
    cases["zipf_rows"] = (c["dims"], c["coo"])
    n = 3000
    # one row holds every nonzero; all other rows empty (leading and trailing empties)
    cols = torch.arange(n, dtype=torch.int64)
    cases["one_full_row"] = ((9, n), (torch.full((n,), 4, dtype=torch.int64), cols,
                                      gen.rng.uniform_pm1(5, 3, n)))
    # rows of length 63 / 64 / 65 / 10000 / 1 and empty rows in between
    lens = torch.tensor([63, 0, 64, 65, 0, 0, 10000, 1, 1, 0, 4097, 4095, 0], dtype=torch.int64)
    cases["edge_lengths"] = ((len(lens), 20000), gen.matrix_from_row_lengths(len(lens), 20000, lens, 7))
    cases["empty"] = ((5, 7), (torch.zeros(0, dtype=torch.int64), torch.zeros(0, dtype=torch.int64),
                              torch.zeros(0, dtype=torch.float64)))
    cases["single"] = ((5, 7), (torch.tensor([3]), torch.tensor([6]), torch.tensor([2.5], dtype=torch.float64)))
    # one row cut over ~150 tiles (more than one group of the hierarchical carry fix-up), then a short one
    lens = torch.tensor([3, 600000, 0, 70000, 5], dtype=torch.int64)
    cases["long_row"] = ((len(lens), 700000), gen.matrix_from_row_lengths(len(lens), 700000, lens, 8))
    # hypersparse: far more rows than nonzeros
    r, cc, v = gen.bernoulli_matrix(20000, 50, 0.001, 9)
    cases["hypersparse"] = ((20000, 50), (r, cc, v))
    return cases


MATRIX_CASES = _matrix_cases()


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("layout", ["csr", "dcsr"])
@pytest.mark.parametrize("name", list(MATRIX_CASES))
def test_spmv(comet, name, layout, variant):
    (I, J), (rows, cols, vals) = MATRIX_CASES[name]
    say("spmv case=%s layout=%s variant=%d nnz=%d" % (name, layout, variant, vals.numel()))
    pack = fmt.pack_csr if layout == "csr" else fmt.pack_dcsr
    A = comet.from_levels(pack(I, J, rows, cols, vals).to("cuda")).set_variant(variant)
    x = gen.dense_operand(1, 0, (J,))
    y = torch.full((I,), float("nan"), dtype=torch.float64, device="cuda")
    comet.comet_spmv(A, dev(x), y)
    torch.cuda.synchronize()
    ref, absum = oracle.spmv(np_(rows), np_(cols), np_(vals), (I, J), np_(x))
    assert_values_close(np_(y), ref, absum, "spmv %s" % name)
    y2 = comet.comet_spmv(A, dev(x))
    torch.cuda.synchronize()
    assert torch.equal(y, y2), "two runs differ"


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("R", [1, 8, 16, 32, 64, 96])
@pytest.mark.parametrize("name,layout", [("zipf_rows", "csr"), ("edge_lengths", "csr"), ("edge_lengths", "dcsr"),
                                         ("empty", "csr"), ("hypersparse", "dcsr"), ("hypersparse", "csr"),
                                         ("long_row", "csr")])
def test_spmm(comet, name, layout, R, variant):
    (I, J), (rows, cols, vals) = MATRIX_CASES[name]
    say("spmm case=%s layout=%s R=%d variant=%d nnz=%d" % (name, layout, R, variant, vals.numel()))
    pack = fmt.pack_csr if layout == "csr" else fmt.pack_dcsr
    A = comet.from_levels(pack(I, J, rows, cols, vals).to("cuda")).set_variant(variant)
    B = gen.dense_operand(2, 0, (J, R))
    C = torch.full((I, R), float("nan"), dtype=torch.float64, device="cuda")
    comet.comet_spmm(A, dev(B), C)
    torch.cuda.synchronize()
    ref, absum = oracle.spmm(np_(rows), np_(cols), np_(vals), (I, J), np_(B))
    assert_values_close(np_(C), ref, absum, "spmm %s R=%d" % (name, R))


HEAVY_ROW = 128      # rows of at least this many nonzeros go to the heavy-row sweep of SpMM


def _heavy_row_matrix():
    """1.3 M nonzeros in 300 000 columns; rows of 127 / 128 / 129 nonzeros around the heavy-row threshold, long
    rows first, last and next to each other, rows longer than a tile and than a unit, empty and short rows."""
    J = 300_000
    block = [5000, 0, 128, 127, 129, 1, 4096, 3, 8192, 8193, 300, 0, 0, 2, 20000, 255, 256, 7, 4095, 4097]
    lens = torch.tensor([9000] + block * 20 + [128, 1, 6000], dtype=torch.int64)
    return (lens.numel(), J), gen.matrix_from_row_lengths(lens.numel(), J, lens, 21)


@pytest.mark.parametrize("variant", [2, 0, 3])
@pytest.mark.parametrize("R", [16, 32, 48, 64, 24])
@pytest.mark.parametrize("name,layout", [("heavy_rows", "csr"), ("heavy_rows", "dcsr"), ("zipf_large", "csr")])
def test_spmm_with_heavy_rows(comet, name, layout, R, variant):
    """Matrices for which SpMM hands the long rows to the heavy-row sweep and leaves them out of the tiled
    kernel (ranks 16, 32, 48, 64; rank 24 and variant 3 stay on the tiled kernel alone).  Every element."""
    if name == "heavy_rows":
        (I, J), (rows, cols, vals) = _heavy_row_matrix()
    else:
        c = gen.config_spmm(seed=2, scale=0.2)
        (I, J), (rows, cols, vals) = c["dims"], c["coo"]
    say("spmm heavy case=%s layout=%s R=%d variant=%d nnz=%d" % (name, layout, R, variant, vals.numel()))
    pack = fmt.pack_csr if layout == "csr" else fmt.pack_dcsr
    A = comet.from_levels(pack(I, J, rows, cols, vals).to("cuda")).set_variant(variant)
    hrows, hnnz = A.heavy_plan()
    lens = torch.bincount(rows, minlength=I)
    assert hrows == int((lens >= HEAVY_ROW).sum()) and hnnz == int(lens[lens >= HEAVY_ROW].sum()) and hrows > 0
    B = gen.dense_operand(2, 0, (J, R))
    C = torch.full((I, R), float("nan"), dtype=torch.float64, device="cuda")
    comet.comet_spmm(A, dev(B), C)
    C2 = torch.full((I, R), float("nan"), dtype=torch.float64, device="cuda")
    comet.comet_spmm(A, dev(B), C2)
    torch.cuda.synchronize()
    ref, absum = oracle.spmm(np_(rows), np_(cols), np_(vals), (I, J), np_(B))
    assert_values_close(np_(C), ref, absum, "spmm %s R=%d" % (name, R))
    assert torch.equal(C, C2), "two runs differ"


def test_lean_handles_plan_no_sweeps_and_give_the_same_results(comet):
    """COMET_LEAN: no sweep plans and none of their copies; SpMM and TTM then run on the tiled kernels alone."""
    (I, J), (rows, cols, vals) = _heavy_row_matrix()
    L = fmt.pack_csr(I, J, rows, cols, vals).to("cuda")
    full = comet.from_levels(L)
    lean = comet.from_levels(L, flags=comet.COMET_VALIDATE | comet.COMET_LEAN)
    assert full.heavy_plan()[0] > 0 and full.heavy_stream_bytes() > 0
    assert lean.heavy_plan() == (0, 0) and lean.heavy_stream_bytes() == 0
    B = dev(gen.dense_operand(2, 0, (J, 32)))
    ref, absum = oracle.spmm(np_(rows), np_(cols), np_(vals), (I, J), np_(B))
    assert_values_close(np_(comet.comet_spmm(lean, B)), ref, absum, "lean spmm")
    assert_values_close(np_(comet.comet_spmm(full, B)), ref, absum, "spmm with the sweep")
    dims, (i, j, k, v), _ = _heavy_fiber_tensor()
    T = fmt.pack_csf3(dims, i, j, k, v).to("cuda")
    lean3 = comet.from_levels(T, flags=comet.COMET_VALIDATE | comet.COMET_LEAN)
    assert lean3.heavy_plan() == (0, 0) and lean3.heavy_stream_bytes() == 0
    U = gen.dense_operand(4, 0, (dims[2], 16))
    Y = comet.comet_ttm(lean3, 2, dev(U))
    torch.cuda.synchronize()
    reft = oracle.ttm(np_(i), np_(j), np_(k), np_(v), dims, np_(U))
    assert_values_close(np_(Y.vals()).reshape(-1, 16), reft["vals"], reft["abs"], "lean ttm")


@pytest.mark.parametrize("R", [1, 16])
@pytest.mark.parametrize("name", ["zipf_rows", "edge_lengths", "hypersparse", "empty", "single"])
def test_products_of_a_coordinate_list_matrix(comet, name, R):
    """[CN,S] input works through the compressed copy the handle builds for itself."""
    (I, J), (rows, cols, vals) = MATRIX_CASES[name]
    A = comet.from_levels(fmt.pack_coo((I, J), (rows, cols), vals).to("cuda"))
    if R == 1:
        x = gen.dense_operand(61, 0, (J,))
        y = torch.full((I,), float("nan"), dtype=torch.float64, device="cuda")
        comet.comet_spmv(A, dev(x), y)
        torch.cuda.synchronize()
        ref, absum = oracle.spmv(np_(rows), np_(cols), np_(vals), (I, J), np_(x))
        assert_values_close(np_(y), ref, absum, "coo spmv %s" % name)
    else:
        B = gen.dense_operand(61, 1, (J, R))
        C = torch.full((I, R), float("nan"), dtype=torch.float64, device="cuda")
        comet.comet_spmm(A, dev(B), C)
        torch.cuda.synchronize()
        ref, absum = oracle.spmm(np_(rows), np_(cols), np_(vals), (I, J), np_(B))
        assert_values_close(np_(C), ref, absum, "coo spmm %s" % name)


def test_spmm_of_ones_gives_row_sums_in_every_column(comet):
    """The paper's example program: B filled with 1.0."""
    (I, J), (rows, cols, vals) = MATRIX_CASES["zipf_rows"]
    A = comet.from_levels(fmt.pack_csr(I, J, rows, cols, vals).to("cuda"))
    C = comet.comet_spmm(A, torch.ones((J, 32), dtype=torch.float64, device="cuda"))
    y = comet.comet_spmv(A, torch.ones(J, dtype=torch.float64, device="cuda"))
    torch.cuda.synchronize()
    ref, absum = oracle.spmv(np_(rows), np_(cols), np_(vals), (I, J), np.ones(J))
    assert_values_close(np_(y), ref, absum, "row sums")
    for r in range(32):
        assert_values_close(np_(C[:, r]), ref, absum, "column %d" % r)


# ----------------------------------------------------------------------------------------------
# order-3 tensors
# ----------------------------------------------------------------------------------------------
def _tensor_cases():
    cases = {}
    c = gen.config_ttv(seed=0, scale=4e-4, chunk=1 << 18)
    cases["zipf_ttv"] = (c["dims"], c["coo"])
    c = gen.config_ttm(seed=0, scale=3e-4, chunk=1 << 18)
    cases["zipf_ttm"] = (c["dims"], c["coo"])
    c = gen.config_mttkrp(seed=0, scale=2e-4, chunk=1 << 18)
    cases["zipf_mttkrp"] = (c["dims"], c["coo"])
    # a mode of size 2 (one of the paper's tensors has such a mode) and fibers of length 1 only
    i, j, k, v = gen.bernoulli_tensor3((300, 40, 2), 0.3, 3)
    cases["mode_of_two"] = ((300, 40, 2), (i, j, k, v))
    i, j, k, v = gen.bernoulli_tensor3((64, 64, 1), 0.4, 4)
    cases["unit_fibers"] = ((64, 64, 1), (i, j, k, v))
    # one slice holds everything: a single slice cut over many tiles, with long and short fibers
    i, j, k, v = gen.bernoulli_tensor3((1, 50, 700), 0.6, 5)
    cases["single_slice"] = ((7, 50, 700), (i + 3, j, k, v))
    # one fiber holds everything
    n = 9000
    cases["single_fiber"] = ((3, 3, n), (torch.ones(n, dtype=torch.int64), torch.full((n,), 2, dtype=torch.int64),
                                         torch.arange(n, dtype=torch.int64), gen.rng.uniform_pm1(6, 3, n)))
    # one slice / one fiber cut over far more than 64 tiles
    i, j, k, v = gen.bernoulli_tensor3((1, 600, 1000), 0.6, 7)
    cases["long_slice"] = ((5, 600, 1000), (i + 2, j, k, v))
    n = 300000
    cases["long_fiber"] = ((2, 2, n), (torch.zeros(n, dtype=torch.int64), torch.ones(n, dtype=torch.int64),
                                       torch.arange(n, dtype=torch.int64), gen.rng.uniform_pm1(8, 3, n)))
    z = torch.zeros(0, dtype=torch.int64)
    cases["empty"] = ((4, 5, 6), (z, z, z, torch.zeros(0, dtype=torch.float64)))
    cases["single"] = ((4, 5, 6), (torch.tensor([2]), torch.tensor([4]), torch.tensor([5]),
                                   torch.tensor([-1.5], dtype=torch.float64)))
    return cases


TENSOR_CASES = _tensor_cases()


def _check_sparse_result_structure(Y, X_levels, ref, layout):
    """pos/crd of the result must be bit-identical to the expected structure."""
    if layout == "csf":
        want = oracle.compressed_pair_levels(ref["i"], ref["j"])
        assert Y.levels()[:2] == [1, 1]
        assert_index_equal(np_(Y.pos(0)), want["pos1"], "pos1")
        assert_index_equal(np_(Y.crd(0)), want["crd1"], "crd1")
        assert_index_equal(np_(Y.pos(1)), want["pos2"], "pos2")
        assert_index_equal(np_(Y.crd(1)), want["crd2"], "crd2")
        # and identical to the input's own level arrays
        assert torch.equal(Y.pos(1).cpu(), X_levels.pos[1].cpu()) and torch.equal(Y.crd(1).cpu(), X_levels.crd[1].cpu())
    else:
        assert Y.levels() == [2, 3]
        assert_index_equal(np_(Y.pos(0)), np.array([0, len(ref["i"])]), "pos")
        assert_index_equal(np_(Y.crd(0)), ref["i"], "crd1")
        assert_index_equal(np_(Y.crd(1)), ref["j"], "crd2")


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("layout", ["csf", "coo"])
@pytest.mark.parametrize("name", list(TENSOR_CASES))
def test_ttv(comet, name, layout, variant):
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    say("ttv case=%s layout=%s variant=%d nnz=%d" % (name, layout, variant, vals.numel()))
    L = (fmt.pack_csf3(dims, i, j, k, vals) if layout == "csf" else fmt.pack_coo(dims, (i, j, k), vals)).to("cuda")
    X = comet.from_levels(L).set_variant(variant)
    v = gen.dense_operand(3, 0, (dims[2],))
    Y = comet.comet_ttv(X, 2, dev(v))
    torch.cuda.synchronize()
    ref = oracle.ttv(np_(i), np_(j), np_(k), np_(vals), dims, np_(v))
    _check_sparse_result_structure(Y, L, ref, layout)
    assert Y.dims() == list(dims[:2])
    assert_values_close(np_(Y.vals()), ref["vals"], ref["abs"], "ttv %s" % name)
    first = Y.vals()
    comet.comet_ttv(X, 2, dev(v), Y)            # reuse of the result handle
    torch.cuda.synchronize()
    assert torch.equal(first, Y.vals())


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("R", [1, 8, 16, 32, 64])
@pytest.mark.parametrize("name", ["zipf_ttm", "mode_of_two", "single_slice", "single_fiber", "long_fiber", "empty",
                                  "single"])
def test_ttm(comet, name, R, variant):
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    say("ttm case=%s R=%d variant=%d nnz=%d" % (name, R, variant, vals.numel()))
    L = fmt.pack_csf3(dims, i, j, k, vals).to("cuda")
    X = comet.from_levels(L).set_variant(variant)
    U = gen.dense_operand(4, 0, (dims[2], R))
    Y = comet.comet_ttm(X, 2, dev(U))
    torch.cuda.synchronize()
    ref = oracle.ttm(np_(i), np_(j), np_(k), np_(vals), dims, np_(U))
    _check_sparse_result_structure(Y, L, ref, "csf")
    assert Y.levels() == [1, 1, 0] and Y.dims() == [dims[0], dims[1], R]
    assert_index_equal(np_(Y.pos(2)), np.array([R]), "dense level size")
    assert_values_close(np_(Y.vals()).reshape(-1, R), ref["vals"], ref["abs"], "ttm %s R=%d" % (name, R))


def _heavy_fiber_tensor(K=3000):
    """1.1 M nonzeros; fibers of 255 / 256 / 257 nonzeros around the heavy-fiber threshold, fibers that fill
    most of the last mode, fibers next to each other and alone in their slice, short ones in between; the last
    mode spans three (rank 16) or six (rank 32) windows of operand rows, the last of them ragged."""
    block = [2500, 256, 255, 257, 1, 1024, 3, 2700, 2600, 300, 2, 1500, 511, 512, 7, 2047, 2049, 40, 600]
    lens = torch.tensor([2650] + block * 65 + [256, 1, 2000], dtype=torch.int64)
    J = 7
    rows, cols, vals = gen.matrix_from_row_lengths(lens.numel(), K, lens, 22)
    I = (lens.numel() + J - 1) // J
    return (I, J, K), (rows // J, rows % J, cols, vals), lens


@pytest.mark.parametrize("layout", ["csf", "coo"])
@pytest.mark.parametrize("R,variant", [(16, 0), (32, 0), (16, 2), (32, 2), (16, 3), (16, 1), (8, 0), (64, 0)])
def test_ttm_with_heavy_fibers(comet, R, variant, layout):
    """A tensor whose long fibers go to the heavy-fiber sweep of TTM (ranks 16 and 32; the other ranks and
    variants 1 and 3 stay on the kernels that take every fiber).  Every element, two runs bit for bit."""
    dims, (i, j, k, vals), lens = _heavy_fiber_tensor()
    say("ttm heavy fibers layout=%s R=%d variant=%d nnz=%d" % (layout, R, variant, vals.numel()))
    L = (fmt.pack_csf3(dims, i, j, k, vals) if layout == "csf" else fmt.pack_coo(dims, (i, j, k), vals)).to("cuda")
    X = comet.from_levels(L).set_variant(variant)
    if layout == "csf":
        hf, hn = X.heavy_plan()
        assert hf == int((lens >= 256).sum()) and hn == int(lens[lens >= 256].sum()) and hn * 4 >= vals.numel()
    U = gen.dense_operand(4, 0, (dims[2], R))
    Y = comet.comet_ttm(X, 2, dev(U))
    torch.cuda.synchronize()
    ref = oracle.ttm(np_(i), np_(j), np_(k), np_(vals), dims, np_(U))
    assert_values_close(np_(Y.vals()).reshape(-1, R), ref["vals"], ref["abs"], "ttm heavy fibers R=%d" % R)
    first = Y.vals().clone()
    comet.comet_ttm(X, 2, dev(U), Y)
    torch.cuda.synchronize()
    assert torch.equal(first, Y.vals()), "two runs differ"


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("R", [1, 8, 16, 64])
@pytest.mark.parametrize("name", ["zipf_mttkrp", "zipf_ttv", "mode_of_two", "single_slice", "single_fiber", "long_slice",
                                  "long_fiber", "empty", "single"])
def test_mttkrp(comet, name, R, variant):
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    say("mttkrp case=%s R=%d variant=%d nnz=%d" % (name, R, variant, vals.numel()))
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, vals).to("cuda")).set_variant(variant)
    B, C = gen.dense_operand(5, 0, (dims[1], R)), gen.dense_operand(5, 1, (dims[2], R))
    M = torch.full((dims[0], R), float("nan"), dtype=torch.float64, device="cuda")
    comet.comet_mttkrp(X, 0, [None, dev(B), dev(C)], M)
    torch.cuda.synchronize()
    ref, absum = oracle.mttkrp(np_(i), np_(j), np_(k), np_(vals), dims, np_(B), np_(C))
    assert_values_close(np_(M), ref, absum, "mttkrp %s R=%d" % (name, R))


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("R", [1, 16, 24])
@pytest.mark.parametrize("name", ["zipf_ttm", "zipf_mttkrp", "mode_of_two", "single_slice", "long_fiber", "empty", "single"])
def test_ttm_and_mttkrp_on_a_sorted_coordinate_list(comet, name, R, variant):
    """[CN,S,S] input: TTM returns the distinct (i,j) as a coordinate list with a dense last level
    ([CN,S,D]); MTTKRP fills the dense matrix.  Both against the oracle, index arrays bit for bit."""
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    say("coo ttm/mttkrp case=%s R=%d variant=%d nnz=%d" % (name, R, variant, vals.numel()))
    X = comet.from_levels(fmt.pack_coo(dims, (i, j, k), vals).to("cuda")).set_variant(variant)
    U = gen.dense_operand(51, 0, (dims[2], R))
    Y = comet.comet_ttm(X, 2, dev(U))
    torch.cuda.synchronize()
    ref = oracle.ttm(np_(i), np_(j), np_(k), np_(vals), dims, np_(U))
    assert Y.levels() == [2, 3, 0] and Y.dims() == [dims[0], dims[1], R]
    assert_index_equal(np_(Y.pos(0)), np.array([0, len(ref["i"])]), "pos")
    assert_index_equal(np_(Y.crd(0)), ref["i"], "crd1")
    assert_index_equal(np_(Y.crd(1)), ref["j"], "crd2")
    assert_index_equal(np_(Y.pos(2)), np.array([R]), "dense level size")
    assert_values_close(np_(Y.vals()).reshape(-1, R), ref["vals"], ref["abs"], "coo ttm %s" % name)
    first = Y.vals()
    comet.comet_ttm(X, 2, dev(U), Y)             # reuse of the result handle
    torch.cuda.synchronize()
    assert torch.equal(first, Y.vals())
    B = gen.dense_operand(51, 1, (dims[1], R))
    M = torch.full((dims[0], R), float("nan"), dtype=torch.float64, device="cuda")
    comet.comet_mttkrp(X, 0, [None, dev(B), dev(U)], M)
    torch.cuda.synchronize()
    refm, absm = oracle.mttkrp(np_(i), np_(j), np_(k), np_(vals), dims, np_(B), np_(U))
    assert_values_close(np_(M), refm, absm, "coo mttkrp %s" % name)


def test_mttkrp_rank_one_is_ttv_twice_on_the_gpu(comet):
    """The sparse TTV result is itself a [CU,CU] matrix handle, so SpMV applies to it."""
    dims, (i, j, k, vals) = TENSOR_CASES["zipf_mttkrp"]
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, vals).to("cuda"))
    B, C = gen.dense_operand(5, 0, (dims[1], 1)), gen.dense_operand(5, 1, (dims[2], 1))
    M = comet.comet_mttkrp(X, 0, [None, dev(B), dev(C)])
    Y = comet.comet_ttv(X, 2, dev(C[:, 0].contiguous()))
    Ym = comet.comet_tensor_create(Y.dims(), Y.levels(), [Y.pos(0), Y.pos(1)], [Y.crd(0), Y.crd(1)], Y.vals())
    m2 = comet.comet_spmv(Ym, dev(B[:, 0].contiguous()))
    torch.cuda.synchronize()
    ref, absum = oracle.mttkrp(np_(i), np_(j), np_(k), np_(vals), dims, np_(B), np_(C))
    assert_values_close(np_(M), ref, absum, "mttkrp")
    assert_values_close(np_(m2), ref[:, 0], absum[:, 0], "ttv then spmv")


# ----------------------------------------------------------------------------------------------
# error paths (forced from the host; no kernel is launched on invalid data)
# ----------------------------------------------------------------------------------------------
def _i32(x):
    return torch.tensor(x, dtype=torch.int32, device="cuda")


def test_invalid_descriptors_are_rejected(comet):
    vals = torch.ones(3, dtype=torch.float64, device="cuda")
    good = dict(dims=[2, 4], levels=[0, 1], pos=[_i32([2]), _i32([0, 1, 3])], crd=[None, _i32([0, 1, 3])], vals=vals)
    comet.comet_tensor_create(**good)

    def bad(status, **kw):
        with pytest.raises(comet.CometError) as e:
            comet.comet_tensor_create(**{**good, **kw})
        assert e.value.status == status, e.value

    bad(2, pos=[_i32([3]), _i32([0, 1, 3])])                       # dense size != dim
    bad(2, pos=[_i32([2]), _i32([0, 1])])                          # pos too short
    bad(2, pos=[_i32([2]), _i32([0, 2, 1])])                       # pos not monotone / wrong end
    bad(2, pos=[_i32([2]), _i32([1, 1, 3])])                       # pos does not start at 0
    bad(2, crd=[None, _i32([0, 3, 1])])                            # unsorted inside a segment
    bad(2, crd=[None, _i32([0, 1, 4])])                            # coordinate out of range
    bad(2, crd=[None, _i32([0, 1, 1])])                            # duplicate inside a segment
    bad(4, levels=[0, 0], pos=[_i32([2]), _i32([4])], crd=[None, None],
        vals=torch.ones(8, dtype=torch.float64, device="cuda"))    # [D,D] is not a sparse tuple we take
    bad(2, levels=[2, 3], pos=[_i32([1, 3]), None], crd=[_i32([0, 1, 1]), _i32([0, 1, 3])])   # CN pos[0] != 0
    bad(2, levels=[2, 3], pos=[_i32([0, 3]), None], crd=[_i32([1, 0, 1]), _i32([0, 1, 3])])   # COO unsorted
    bad(2, levels=[2, 3], pos=[_i32([0, 3]), None], crd=[_i32([0, 1, 1]), _i32([0, 3, 3])])   # COO duplicate


def test_shape_mode_and_rank_errors(comet):
    dims, (i, j, k, vals) = TENSOR_CASES["mode_of_two"]
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, vals).to("cuda"))
    v = torch.ones(dims[2], dtype=torch.float64, device="cuda")
    for mode in (0, 1):
        with pytest.raises(comet.CometError) as e:
            comet.comet_ttv(X, mode, torch.ones(dims[mode], dtype=torch.float64, device="cuda"))
        assert e.value.status == 4
    with pytest.raises(comet.CometError) as e:
        comet.comet_ttv(X, 2, torch.ones(dims[2] + 1, dtype=torch.float64, device="cuda"))
    assert e.value.status == 3
    B = torch.ones((dims[1], 4), dtype=torch.float64, device="cuda")
    C = torch.ones((dims[2], 4), dtype=torch.float64, device="cuda")
    with pytest.raises(comet.CometError) as e:
        comet.comet_mttkrp(X, 1, [torch.ones((dims[0], 4), dtype=torch.float64, device="cuda"), None, C])
    assert e.value.status == 4
    with pytest.raises(comet.CometError) as e:
        comet.comet_spmv(X, v)
    assert e.value.status in (3, 4)
    Y = comet.comet_ttv(X, 2, v)
    with pytest.raises(comet.CometError) as e:       # a TTV result handle cannot be reused for TTM
        comet.comet_ttm(X, 2, C, Y)
    assert e.value.status == 1
    comet.comet_mttkrp(X, 0, [None, B, C])


def test_operations_follow_the_stream_they_are_given(comet):
    """Work is enqueued on the caller's stream: issued on a side stream behind a long-running fill of the
    operand, the product must see the filled operand, and the result must be complete once that stream
    (not the default one) has been waited for."""
    (n, m), (rows, cols, vals) = MATRIX_CASES["zipf_rows"]
    A = comet.from_levels(fmt.pack_csr(n, m, rows, cols, vals).to("cuda"))
    R = 16
    Bh = gen.dense_operand(31, 0, (m, R))
    side = torch.cuda.Stream()
    B = torch.zeros((m, R), dtype=torch.float64, device="cuda")
    C = torch.full((n, R), float("nan"), dtype=torch.float64, device="cuda")
    junk = torch.empty(1 << 26, dtype=torch.float64, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(4):
            junk.fill_(1.0)                      # keeps the side stream busy ahead of the copy
        B.copy_(dev(Bh), non_blocking=True)
        comet.comet_spmm(A, B, C)                 # binding passes the current (side) stream
    side.synchronize()
    ref, absum = oracle.spmm(np_(rows), np_(cols), np_(vals), (n, m), np_(Bh))
    assert_values_close(np_(C), ref, absum, "spmm on a side stream")


def test_copy_flag_detaches_from_caller_arrays(comet):
    (I, J), (rows, cols, vals) = MATRIX_CASES["config1"]
    L = fmt.pack_csr(I, J, rows, cols, vals).to("cuda")
    A = comet.comet_tensor_create(L.dims, L.tags, L.pos, L.crd, L.vals, comet.COMET_COPY | comet.COMET_VALIDATE)
    x = dev(gen.dense_operand(1, 0, (J,)))
    y1 = comet.comet_spmv(A, x).clone()
    L.vals.zero_()
    L.crd[1].zero_()
    y2 = comet.comet_spmv(A, x)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)


def test_empty_slices_and_fibers_are_accepted_and_contribute_nothing(comet):
    """A stored slice without fibers and a stored fiber without nonzeros (reading R19): the level walker
    reaches every value exactly once, TTV keeps one (zero) value for the empty fiber, MTTKRP leaves the
    rows of the empty slice and of the unstored index at zero."""
    dims = (4, 3, 5)
    tags = [1, 1, 1]
    pos = [np.array([0, 3], np.int32), np.array([0, 2, 2, 3], np.int32), np.array([0, 2, 2, 4], np.int32)]
    crd = [np.array([0, 1, 3], np.int32), np.array([0, 2, 1], np.int32), np.array([1, 3, 0, 4], np.int32)]
    vals = np.array([1.5, -2.0, 0.25, 4.0])
    coords, seen = oracle.walk(tags, pos, crd, 4)
    assert np.all(seen == 1)
    X = comet.comet_tensor_create(dims, tags, [torch.from_numpy(p).cuda() for p in pos],
                                  [torch.from_numpy(c).cuda() for c in crd], torch.from_numpy(vals).cuda())
    v = gen.dense_operand(9, 0, (5,))
    B, C = gen.dense_operand(9, 1, (3, 16)), gen.dense_operand(9, 2, (5, 16))
    for variant in VARIANTS:
        X.set_variant(variant)
        Y = comet.comet_ttv(X, 2, dev(v))
        M = torch.full((4, 16), float("nan"), dtype=torch.float64, device="cuda")
        comet.comet_mttkrp(X, 0, [None, dev(B), dev(C)], M)
        torch.cuda.synchronize()
        ref = oracle.ttv(coords[:, 0], coords[:, 1], coords[:, 2], vals, dims, np_(v))
        got = np_(Y.vals())
        assert got.shape == (3,) and got[1] == 0.0                      # the empty fiber (0, 2)
        assert_values_close(got[[0, 2]], ref["vals"], ref["abs"], "ttv with an empty fiber")
        refM, absM = oracle.mttkrp(coords[:, 0], coords[:, 1], coords[:, 2], vals, dims, np_(B), np_(C))
        assert_values_close(np_(M), refM, absM, "mttkrp with an empty slice")
        assert bool((M[1] == 0).all()) and bool((M[2] == 0).all())


def test_operations_replay_from_a_captured_graph(comet):
    """After a first (allocating) call every operation only enqueues kernels, so it can be captured into a
    HIP graph; each replay -- with eager work and synchronisations in between -- must reproduce the eager
    result bit for bit (the kernels use no atomics and clear their scratch themselves)."""
    (n, m), (rows, cols, vals) = MATRIX_CASES["zipf_rows"]
    A = comet.from_levels(fmt.pack_csr(n, m, rows, cols, vals).to("cuda"))
    dims, (i, j, k, tv) = TENSOR_CASES["zipf_mttkrp"]
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, tv).to("cuda"))
    R = 16
    B = dev(gen.dense_operand(41, 0, (m, R)))
    x = dev(gen.dense_operand(41, 1, (m,)))
    U = dev(gen.dense_operand(41, 2, (dims[2], R)))
    Fb, Fc = dev(gen.dense_operand(41, 3, (dims[1], R))), U
    v = dev(gen.dense_operand(41, 4, (dims[2],)))
    C = torch.empty((n, R), dtype=torch.float64, device="cuda")
    y = torch.empty(n, dtype=torch.float64, device="cuda")
    M = torch.empty((dims[0], R), dtype=torch.float64, device="cuda")
    Yv = comet.comet_ttv(X, 2, v)
    Ym = comet.comet_ttm(X, 2, U)

    def run_all():
        comet.comet_spmm(A, B, C)
        comet.comet_spmv(A, x, y)
        comet.comet_ttv(X, 2, v, Yv)
        comet.comet_ttm(X, 2, U, Ym)
        comet.comet_mttkrp(X, 0, [None, Fb, Fc], M)

    run_all()                                    # first calls: scratch gets allocated here
    torch.cuda.synchronize()
    want = [t.clone() for t in (C, y, M, Yv.vals(), Ym.vals())]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_all()                                # warm-up on the capture stream
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run_all()
    for rep in range(3):
        for t in (C, y, M):
            t.fill_(float("nan"))                # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = (C, y, M, Yv.vals(), Ym.vals())
        for a, b in zip(got, want):
            assert torch.equal(a, b), "replay %d differs from the eager result" % rep


def test_the_sweeps_replay_from_a_captured_graph(comet):
    """SpMM with its heavy-row sweep and TTM with its heavy-fiber sweep (each with the tiled kernel on the copy
    of the other rows / fibers) are kernel launches only once the scratch exists: captured and replayed, with
    eager work in between, they reproduce the eager results bit for bit."""
    (I, J), (rows, cols, vals) = _heavy_row_matrix()
    A = comet.from_levels(fmt.pack_csr(I, J, rows, cols, vals).to("cuda"))
    dims, (i, j, k, tv), _ = _heavy_fiber_tensor()
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, tv).to("cuda"))
    assert A.heavy_plan()[0] > 0 and X.heavy_plan()[0] > 0
    A.reserve(32)
    X.reserve(16)
    B = dev(gen.dense_operand(43, 0, (J, 32)))
    U = dev(gen.dense_operand(43, 1, (dims[2], 16)))
    C = torch.empty((I, 32), dtype=torch.float64, device="cuda")
    Y = comet.comet_ttm(X, 2, U)

    def run_all():
        comet.comet_spmm(A, B, C)
        comet.comet_ttm(X, 2, U, Y)

    run_all()
    torch.cuda.synchronize()
    want = [C.clone(), Y.vals().clone()]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_all()
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run_all()
    for rep in range(3):
        C.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, want[0]) and torch.equal(Y.vals(), want[1]), "replay %d differs from the eager result" % rep
