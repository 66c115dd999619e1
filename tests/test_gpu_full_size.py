"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

SpMM, TTV (both formats), TTM and MTTKRP at rank 16 are compared with the oracle on EVERY output element
(the oracle walks all 18.5 M - 150 M nonzeros; tens of seconds of host time each).  The cases whose oracle run
would take minutes (MTTKRP at rank 64, the re-stored modes, the results beyond 2^31 values) check sampled
output rows / fibers / slices -- random ones plus the heaviest, which are cut over the most kernel tiles --
against the oracle run on exactly the nonzeros that feed them.  Every case also checks what holds at any
size: index outputs bit-identical to the expected structure, rows without stored nonzeros exactly zero.

The oracle is always fed from the seeded generator's own coordinate list (i, j, k, vals), never from
anything the library produced: a re-stored tensor is first compared, as a whole, with a torch sort of the
packed original coordinates, and the oracle then gets the original nonzeros in that order.
"""
import numpy as np
import pytest
import torch

import oracle
from synth import formats as fmt
from synth import generate as gen
from util import assert_values_close, np_

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.fixture(scope="module")
def comet():
    from paper_2102_05187_amd import build
    build.build_if_missing()
    import paper_2102_05187_amd as c
    return c


def say(msg):
    print(msg, flush=True)


def ranges_to_index(starts: torch.Tensor, ends: torch.Tensor):
    """Concatenated positions of the half-open ranges, plus the range number of every position."""
    lens = (ends - starts).to(torch.int64)
    which = torch.repeat_interleave(torch.arange(lens.numel(), device=starts.device), lens)
    offs = torch.cumsum(lens, 0) - lens
    idx = starts.to(torch.int64)[which] + (torch.arange(int(lens.sum()), device=starts.device) - offs[which])
    return idx, which


def sample_ids(n, count, must, seed):
    g = torch.Generator().manual_seed(seed)
    ids = torch.randint(0, n, (count,), generator=g)
    ids = torch.unique(torch.cat([ids, torch.as_tensor(must, dtype=torch.int64)]))
    return ids.to(DEV)


@pytest.fixture(scope="module")
def spmm_config():
    c = gen.config_spmm(seed=0, device=DEV, R=32)
    rows, cols, vals = c["coo"]
    n = c["dims"][0]
    say("spmm full size nnz=%d: oracle over every nonzero" % vals.numel())
    ref, absum = oracle.spmm(np_(rows), np_(cols), np_(vals), (n, n), np_(c["B"]))
    say("  oracle done")
    return c, ref, absum


@pytest.mark.parametrize("layout", ["csr", "dcsr"])
def test_spmm_config(comet, spmm_config, layout):
    """Every element of C at the headline size, for the matrix stored [D,CU] and [CU,CU]."""
    c, ref, absum = spmm_config
    rows, cols, vals = c["coo"]
    n = c["dims"][0]
    L = (fmt.pack_csr if layout == "csr" else fmt.pack_dcsr)(n, n, rows, cols, vals)
    A = comet.from_levels(L)
    C = torch.full((n, 32), float("nan"), dtype=torch.float64, device=DEV)
    comet.comet_spmm(A, c["B"], C)
    torch.cuda.synchronize()
    assert_values_close(np_(C), ref, absum, "spmm %s, every row" % layout)


def test_spmm_axpby_config(comet, spmm_config):
    """C = alpha A B + beta C at the headline size (heavy-row sweep and tiled kernel together), every element."""
    c, ref, absum = spmm_config
    rows, cols, vals = c["coo"]
    n = c["dims"][0]
    A = comet.from_levels(fmt.pack_csr(n, n, rows, cols, vals))
    old = gen.dense_operand(0, 7, (n, 32), DEV)
    C = old.clone()
    comet.comet_spmm_axpby(A, -1.25, c["B"], 0.5, C)
    torch.cuda.synchronize()
    want, want_abs = oracle.axpby(-1.25, ref, absum, 0.5, np_(old))
    assert_values_close(np_(C), want, want_abs, "spmm_axpby, every row")


def test_spmv_on_the_spmm_matrix(comet, spmm_config):
    """SpMV at a size where it is not launch-bound: the headline matrix with one dense column (x is 8 MB, so
    the gathers go through L1 / L2 rather than LDS).  Every element of y."""
    c, _, _ = spmm_config
    rows, cols, vals = c["coo"]
    n = c["dims"][0]
    x = c["B"][:, 0].contiguous()
    A = comet.from_levels(fmt.pack_csr(n, n, rows, cols, vals))
    y = torch.full((n,), float("nan"), dtype=torch.float64, device=DEV)
    comet.comet_spmv(A, x, y)
    torch.cuda.synchronize()
    ref, absum = oracle.spmv(np_(rows), np_(cols), np_(vals), (n, n), np_(x))
    assert_values_close(np_(y), ref, absum, "spmv on the spmm matrix, every row")


@pytest.fixture(scope="module")
def ttv_config():
    return gen.config_ttv(seed=0, device=DEV)


_TTV_REF = {}


def _ttv_reference(c):
    """The oracle's TTV of the whole 50 M-nonzero tensor (computed once, shared by the CSF and COO cases)."""
    if "ref" not in _TTV_REF:
        i, j, k, vals = c["coo"]
        say("  oracle ttv over all %d nonzeros" % vals.numel())
        _TTV_REF["ref"] = oracle.ttv(np_(i), np_(j), np_(k), np_(vals), c["dims"], np_(c["v"]))
        say("  oracle done")
    return _TTV_REF["ref"]


def _fiber_sample(L, count, seed):
    pos3 = L.pos[2].to(torch.int64)
    lens = pos3[1:] - pos3[:-1]
    heavy = torch.topk(lens, 4).indices.cpu()
    fids = sample_ids(lens.numel(), count, heavy, seed)
    idx, which = ranges_to_index(pos3[fids], pos3[fids + 1])
    return fids, idx, which


def test_ttv_csf_config(comet, ttv_config):
    c = ttv_config
    i, j, k, vals = c["coo"]
    L = fmt.pack_csf3(c["dims"], i, j, k, vals)
    say("ttv csf full size nnz=%d fibers=%d" % (vals.numel(), L.crd[1].numel()))
    X = comet.from_levels(L)
    Y = comet.comet_ttv(X, 2, c["v"])
    torch.cuda.synchronize()
    for l in range(2):                    # structure: the result's levels are the input's, bit for bit
        assert torch.equal(Y.pos(l), L.pos[l]) and torch.equal(Y.crd(l), L.crd[l])
    ref = _ttv_reference(c)
    assert len(ref["vals"]) == L.crd[1].numel()
    assert_values_close(np_(Y.vals()), ref["vals"], ref["abs"], "ttv csf, every fiber")


def test_ttv_coo_config(comet, ttv_config):
    c = ttv_config
    i, j, k, vals = c["coo"]
    Lc = fmt.pack_coo(c["dims"], (i, j, k), vals)
    say("ttv coo full size nnz=%d" % vals.numel())
    X = comet.from_levels(Lc)
    Y = comet.comet_ttv(X, 2, c["v"])
    torch.cuda.synchronize()
    # structure: the distinct (i,j) pairs in order = run heads of the sorted coordinate list
    head = torch.ones(i.numel(), dtype=torch.bool, device=DEV)
    head[1:] = (i[1:] != i[:-1]) | (j[1:] != j[:-1])
    assert torch.equal(Y.crd(0), i[head].to(torch.int32)) and torch.equal(Y.crd(1), j[head].to(torch.int32))
    assert Y.pos(0).tolist() == [0, int(head.sum())]
    ref = _ttv_reference(c)
    assert np.array_equal(np_(Y.crd(0)), ref["i"]) and np.array_equal(np_(Y.crd(1)), ref["j"])
    assert_values_close(np_(Y.vals()), ref["vals"], ref["abs"], "ttv coo, every run")


def test_ttm_config(comet):
    c = gen.config_ttm(seed=0, device=DEV, R=16)
    i, j, k, vals = c["coo"]
    L = fmt.pack_csf3(c["dims"], i, j, k, vals)
    say("ttm full size nnz=%d fibers=%d" % (vals.numel(), L.crd[1].numel()))
    X = comet.from_levels(L)
    Y = comet.comet_ttm(X, 2, c["U"])
    torch.cuda.synchronize()
    for l in range(2):
        assert torch.equal(Y.pos(l), L.pos[l]) and torch.equal(Y.crd(l), L.crd[l])
    assert Y.pos(2).tolist() == [16] and Y.levels() == [1, 1, 0]
    say("  oracle ttm over all %d nonzeros" % vals.numel())
    ref = oracle.ttm(np_(i), np_(j), np_(k), np_(vals), c["dims"], np_(c["U"]))
    say("  oracle done")
    assert ref["vals"].shape == (L.crd[1].numel(), 16)
    assert_values_close(np_(Y.vals()).reshape(-1, 16), ref["vals"], ref["abs"], "ttm, every fiber")
    del Y, X
    # the same tensor as a sorted coordinate list: the result lists the distinct (i,j) and carries the same values
    Xc = comet.from_levels(fmt.pack_coo(c["dims"], (i, j, k), vals))
    Yc = comet.comet_ttm(Xc, 2, c["U"])
    torch.cuda.synchronize()
    assert Yc.levels() == [2, 3, 0] and Yc.pos(0).tolist() == [0, ref["i"].size]
    assert np.array_equal(np_(Yc.crd(0)), ref["i"]) and np.array_equal(np_(Yc.crd(1)), ref["j"])
    assert_values_close(np_(Yc.vals()).reshape(-1, 16), ref["vals"], ref["abs"], "ttm on a coordinate list, every fiber")


@pytest.mark.parametrize("R", [16, 64])
def test_mttkrp_config(comet, R):
    c = gen.config_mttkrp(seed=0, device=DEV, R=R)
    i, j, k, vals = c["coo"]
    dims = c["dims"]
    L = fmt.pack_csf3(dims, i, j, k, vals)
    say("mttkrp full size R=%d nnz=%d fibers=%d slices=%d" % (R, vals.numel(), L.crd[1].numel(), L.crd[0].numel()))
    X = comet.from_levels(L)
    M = torch.full((dims[0], R), float("nan"), dtype=torch.float64, device=DEV)
    comet.comet_mttkrp(X, 0, [None, c["B"], c["C"]], M)
    torch.cuda.synchronize()
    if R == 16:
        say("  oracle mttkrp over all %d nonzeros" % vals.numel())
        ref, absum = oracle.mttkrp(np_(i), np_(j), np_(k), np_(vals), dims, np_(c["B"]), np_(c["C"]))
        say("  oracle done")
        assert_values_close(np_(M), ref, absum, "mttkrp R=16, every row")
        # the same tensor as a sorted coordinate list (works through a compressed copy inside the handle)
        Xc = comet.from_levels(fmt.pack_coo(dims, (i, j, k), vals))
        Mc = torch.full((dims[0], R), float("nan"), dtype=torch.float64, device=DEV)
        comet.comet_mttkrp(Xc, 0, [None, c["B"], c["C"]], Mc)
        torch.cuda.synchronize()
        assert_values_close(np_(Mc), ref, absum, "mttkrp R=16 on a coordinate list, every row")
    else:
        pos2, pos3 = L.pos[1].to(torch.int64), L.pos[2].to(torch.int64)
        first = pos3[pos2[:-1]]
        last = pos3[pos2[1:]]
        heavy = torch.topk(last - first, 2).indices.cpu()       # the Zipf head slices: cut over thousands of tiles
        sids = sample_ids(first.numel(), 600, heavy, 5)
        idx, which = ranges_to_index(first[sids], last[sids])
        say("  oracle on %d nonzeros of %d sampled slices" % (idx.numel(), sids.numel()))
        ref, absum = oracle.mttkrp(np_(which), np_(j[idx]), np_(k[idx]), np_(vals[idx]), (sids.numel(), dims[1], dims[2]),
                                   np_(c["B"]), np_(c["C"]))
        rows = L.crd[0].to(torch.int64)[sids]
        assert_values_close(np_(M[rows]), ref, absum, "mttkrp sampled slices R=%d" % R)
    # rows whose index is not stored at the root level receive nothing
    stored = torch.zeros(dims[0], dtype=torch.bool, device=DEV)
    stored[L.crd[0].to(torch.int64)] = True
    assert bool((M[~stored] == 0.0).all())
    assert not bool(torch.isnan(M).any())


def _expand_csf(T):
    """Coordinates per level of every nonzero of a [CU,CU,CU] handle (torch index work only)."""
    pos2, pos3 = T.pos(1).to(torch.int64), T.pos(2).to(torch.int64)
    fib_of_nnz = torch.repeat_interleave(torch.arange(pos3.numel() - 1, device=DEV), pos3[1:] - pos3[:-1])
    slice_of_fib = torch.repeat_interleave(torch.arange(pos2.numel() - 1, device=DEV), pos2[1:] - pos2[:-1])
    c1 = T.crd(1).to(torch.int64)[fib_of_nnz]
    c0 = T.crd(0).to(torch.int64)[slice_of_fib][fib_of_nnz]
    return c0, c1, T.crd(2).to(torch.int64), fib_of_nnz


def _sorted_original(coords, vals, dims, order):
    """The generator's nonzeros sorted by the level order `order` (a torch sort of the packed key): the
    per-level coordinate arrays, the values, the order itself, and the packed keys.  Nothing here comes
    from the library."""
    a, b, c = (coords[m].to(torch.int64) for m in order)
    key = (a * dims[order[1]] + b) * dims[order[2]] + c
    skey, perm = torch.sort(key)
    assert bool((skey[1:] > skey[:-1]).all())
    return (a[perm], b[perm], c[perm]), vals[perm], perm, skey


def _assert_restored(Xr, ref_levels, ref_vals, skey, dims, order):
    """Every coordinate and value of the re-stored handle against the sorted original, plus its structure:
    fibers and slices start exactly where the sorted original changes its (root, middle) / root prefix."""
    c0, c1, c2, _ = _expand_csf(Xr)
    assert torch.equal((c0 * dims[order[1]] + c1) * dims[order[2]] + c2, skey)
    assert torch.equal(Xr.vals(), ref_vals)
    fkey = skey // dims[order[2]]
    fhead = torch.ones_like(fkey, dtype=torch.bool)
    fhead[1:] = fkey[1:] != fkey[:-1]
    fstart = torch.nonzero(fhead).flatten()
    pos3 = Xr.pos(2).to(torch.int64)
    assert pos3.numel() == fstart.numel() + 1 and torch.equal(pos3[:-1], fstart) and int(pos3[-1]) == skey.numel()
    skey2 = fkey[fstart] // dims[order[1]]
    shead = torch.ones_like(skey2, dtype=torch.bool)
    shead[1:] = skey2[1:] != skey2[:-1]
    sstart = torch.nonzero(shead).flatten()
    pos2 = Xr.pos(1).to(torch.int64)
    assert pos2.numel() == sstart.numel() + 1 and torch.equal(pos2[:-1], sstart) and int(pos2[-1]) == fstart.numel()
    return fstart, sstart


def test_first_mode_ttv_config(comet, ttv_config):
    """Section 8.2 writes TTV for the first mode: y_jk = sum_i x_ijk v_i.  The tensor is re-stored in
    the order (1, 2, 0) on the device, checked as a whole against a sort of the packed coordinates,
    then contracted; sampled output fibers against the oracle."""
    c = ttv_config
    i, j, k, vals = c["coo"]
    dims = c["dims"]
    L = fmt.pack_csf3(dims, i, j, k, vals)
    X = comet.from_levels(L)
    say("first-mode ttv full size nnz=%d" % vals.numel())
    Xr = comet.comet_tensor_reorder(X, (1, 2, 0))
    torch.cuda.synchronize()
    assert Xr.mode_of_level() == [1, 2, 0] and Xr.dims() == [dims[1], dims[2], dims[0]]
    # whole-structure check: the walked coordinates are the original ones sorted by (j, k, i)
    key = (j * dims[2] + k) * dims[0] + i
    skey, perm = torch.sort(key)
    assert bool((skey[1:] > skey[:-1]).all())
    c0, c1, c2, fib_of_nnz = _expand_csf(Xr)
    assert torch.equal((c0 * dims[2] + c1) * dims[0] + c2, skey)
    assert torch.equal(Xr.vals(), vals[perm])
    pos2 = Xr.pos(1).to(torch.int64)
    assert bool((pos2[1:] > pos2[:-1]).all())            # no empty slices or fibers are produced
    del key, skey, perm
    v = gen.dense_operand(0, 7, (dims[0],), DEV)
    Y = comet.comet_ttv(Xr, 0, v)
    torch.cuda.synchronize()
    pos3 = Xr.pos(2).to(torch.int64)
    lens = pos3[1:] - pos3[:-1]
    heavy = torch.topk(lens, 4).indices.cpu()
    fids = sample_ids(lens.numel(), 4000, heavy, 6)
    idx, which = ranges_to_index(pos3[fids], pos3[fids + 1])
    # oracle on the nonzeros of the sampled (j,k) fibers, in the original mode numbering
    ref = oracle.ttv_mode((np_(c2[idx]), np_(c0[idx]), np_(c1[idx])), np_(Xr.vals()[idx]), dims, 0, np_(v))
    assert len(ref["vals"]) == fids.numel()
    assert_values_close(np_(Y.vals()[fids]), ref["vals"], ref["abs"], "first-mode ttv sampled fibers")


def test_first_mode_ttm_config(comet):
    """TTM along the first mode at the benchmark size (the form Section 8.2 writes out), on the tensor
    re-stored in the order (1, 2, 0); sampled output fibers against the oracle."""
    c = gen.config_ttm(seed=0, device=DEV, R=16)
    i, j, k, vals = c["coo"]
    dims = c["dims"]
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, vals))
    Xr = comet.comet_tensor_reorder(X, (1, 2, 0))
    torch.cuda.synchronize()
    say("first-mode ttm full size nnz=%d fibers=%d" % (vals.numel(), Xr.crd(1).numel()))
    U = gen.dense_operand(0, 8, (dims[0], 16), DEV)
    Y = comet.comet_ttm(Xr, 0, U)
    torch.cuda.synchronize()
    assert Y.levels() == [1, 1, 0] and Y.dims() == [dims[1], dims[2], 16] and Y.mode_of_level()[:2] == [1, 2]
    # the re-stored tensor as a whole against a sort of the generator's own coordinates ...
    order = (1, 2, 0)
    lv, svals, perm, skey = _sorted_original((i, j, k), vals, dims, order)
    fstart, _ = _assert_restored(Xr, lv, svals, skey, dims, order)
    # ... and the oracle on the ORIGINAL nonzeros of sampled output fibers (positions in the sorted original)
    fend = torch.cat([fstart[1:], torch.tensor([skey.numel()], device=DEV)])
    heavy = torch.topk(fend - fstart, 4).indices.cpu()
    fids = sample_ids(fstart.numel(), 3000, heavy, 7)
    idx, which = ranges_to_index(fstart[fids], fend[fids])
    src = perm[idx]
    ref = oracle.ttm_mode((np_(i[src]), np_(j[src]), np_(k[src])), np_(vals[src]), dims, 0, np_(U))
    assert len(ref["vals"]) == fids.numel()
    assert_values_close(np_(Y.vals().reshape(-1, 16)[fids]), ref["vals"], ref["abs"], "first-mode ttm sampled fibers")


def test_second_mode_mttkrp_config(comet):
    """MTTKRP for the second mode at the benchmark size, on the tensor re-stored in the order (1, 0, 2);
    sampled output rows (the heaviest slices among them) against the oracle."""
    R = 16
    c = gen.config_mttkrp(seed=0, device=DEV, R=R)
    i, j, k, vals = c["coo"]
    dims = c["dims"]
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, vals))
    Xr = comet.comet_tensor_reorder(X, (1, 0, 2))
    del X
    torch.cuda.synchronize()
    F = [gen.dense_operand(0, 8 + m, (dims[m], R), DEV) for m in range(3)]
    M = torch.full((dims[1], R), float("nan"), dtype=torch.float64, device=DEV)
    comet.comet_mttkrp(Xr, 1, [F[0], None, F[2]], M)
    torch.cuda.synchronize()
    # the re-stored tensor as a whole against a sort of the generator's own coordinates ...
    order = (1, 0, 2)
    lv, svals, perm, skey = _sorted_original((i, j, k), vals, dims, order)
    fstart, sstart = _assert_restored(Xr, lv, svals, skey, dims, order)
    del skey, svals
    # ... and the oracle on the ORIGINAL nonzeros of sampled output rows (slices of the sorted original)
    first = fstart[sstart]
    last = torch.cat([first[1:], torch.tensor([vals.numel()], device=DEV)])
    heavy = torch.topk(last - first, 2).indices.cpu()
    sids = sample_ids(first.numel(), 500, heavy, 8)
    idx, which = ranges_to_index(first[sids], last[sids])
    say("second-mode mttkrp full size: oracle on %d nonzeros of %d sampled slices" % (idx.numel(), sids.numel()))
    src = perm[idx]
    rows = j[src[torch.searchsorted(which, torch.arange(sids.numel(), device=DEV))]].to(torch.int64)   # mode-1 index of each sampled slice
    # a private numbering of the sampled rows keeps the oracle's output small: row `which` stands for j = rows[which]
    ref, absum = oracle.mttkrp_mode((np_(i[src]), np_(which), np_(k[src])), np_(vals[src]),
                                    (dims[0], sids.numel(), dims[2]), 1, [np_(F[0]), None, np_(F[2])])
    assert_values_close(np_(M[rows]), ref, absum, "second-mode mttkrp sampled slices")
    stored = torch.zeros(dims[1], dtype=torch.bool, device=DEV)
    stored[torch.unique(j)] = True
    assert bool((M[~stored] == 0.0).all()) and not bool(torch.isnan(M).any())


def test_spmm_with_an_operand_beyond_4_gib(comet):
    """The dense operand is 4.6 GB: row offsets inside it do not fit 32-bit byte offsets (the kernels count
    them in doubles).  Every output row against the oracle."""
    nrows, ncols, R = 100_000, 9_000_000, 64
    lens = torch.full((nrows,), 8, dtype=torch.int64, device=DEV)
    lens[::1000] = 3000
    rows, cols, vals = gen.matrix_from_row_lengths(nrows, ncols, lens, 5, DEV)
    say("spmm with a %.1f GB operand, nnz=%d" % (ncols * R * 8 / 1e9, vals.numel()))
    assert int(cols.max()) * R * 8 > (1 << 32)
    A = comet.from_levels(fmt.pack_csr(nrows, ncols, rows, cols, vals))
    B = gen.dense_operand(5, 0, (ncols, R), DEV)
    C = comet.comet_spmm(A, B)
    torch.cuda.synchronize()
    ref, absum = oracle.spmm(np_(rows), np_(cols), np_(vals), (nrows, ncols), np_(B))
    assert_values_close(np_(C), ref, absum, "spmm, operand beyond 4 GiB")


def test_ttm_result_with_more_than_2_31_values(comet):
    """38.9 M fibers x R = 64 gives 2.49 * 10^9 result values (19.9 GB): more than an int32 position can
    count, which is fine for a dense last level.  Sampled fibers against the oracle."""
    R = 64
    c = gen.config_mttkrp(seed=0, device=DEV, R=R)
    i, j, k, vals = c["coo"]
    dims = c["dims"]
    L = fmt.pack_csf3(dims, i, j, k, vals)
    X = comet.from_levels(L)
    U = c["C"]
    Y = comet.comet_ttm(X, 2, U)
    torch.cuda.synchronize()
    nfib = int(L.crd[1].numel())
    say("ttm with %d fibers x %d = %d result values" % (nfib, R, nfib * R))
    assert nfib * R > (1 << 31) and Y.dims() == [dims[0], dims[1], R]
    fids, idx, which = _fiber_sample(L, 2000, 9)
    fids = torch.unique(torch.cat([fids, torch.tensor([nfib - 1, nfib - 2], device=DEV)]))   # rows past 2^31 values
    pos3 = L.pos[2].to(torch.int64)
    idx, which = ranges_to_index(pos3[fids], pos3[fids + 1])
    ref = oracle.ttm(np_(i[idx]), np_(j[idx]), np_(k[idx]), np_(vals[idx]), dims, np_(U))
    got = Y.vals(copy=False).reshape(-1, R)[fids]
    assert_values_close(np_(got), ref["vals"], ref["abs"], "ttm sampled fibers of a result beyond 2^31 values")
