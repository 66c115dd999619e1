"""Seeded sweep of small random shapes through every operation, format, kernel family and mode.

The fixed cases of test_gpu_parity.py pin the edges that were thought of; this sweep draws shapes,
densities, ranks (odd ones too), formats and mode orders from a counter-based generator so that tile,
chunk, lane-group and segment boundaries fall in many different relative positions.  Every element is
compared with the oracle (index arrays bit for bit, values with the tolerance of tests/util.py).
"""
import os

import numpy as np
import pytest
import torch

import oracle
from synth import formats as fmt
from synth import generate as gen
from util import assert_index_equal, assert_values_close, np_

pytestmark = pytest.mark.gpu

# number of seeded blocks per test; raise it (COMET_SWEEP_BLOCKS=200) for a longer soak of the same code
BLOCKS = int(os.environ.get("COMET_SWEEP_BLOCKS", "10"))


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


def pick(rng, seq):
    return seq[int(rng.integers(len(seq)))]


def random_matrix(rng, seed):
    nrows = int(rng.integers(1, 3000))
    ncols = int(rng.integers(1, 6000))
    kind = pick(rng, ["bernoulli", "lengths", "zipf"])
    if kind == "bernoulli":
        nrows = min(nrows, max(1, 2_000_000 // ncols))
        dens = min(1.0, float(rng.uniform(0.0, 30000.0 / (nrows * ncols))))
        rows, cols, vals = gen.bernoulli_matrix(nrows, ncols, dens, seed)
    else:
        if kind == "zipf":
            lens = gen.zipf_row_lengths(nrows, float(rng.uniform(1.1, 2.5)), max(1, ncols // 4), seed)
        else:
            lens = torch.from_numpy(rng.integers(0, max(2, min(ncols // 4, 40)), nrows)).to(torch.int64)
            lens[torch.from_numpy(rng.random(nrows) < 0.3)] = 0          # plenty of empty rows
            if rng.random() < 0.5:                                         # one long row across tile boundaries
                lens[int(rng.integers(nrows))] = min(ncols // 4, int(rng.integers(1000, 9000)))
        lens = torch.clamp(lens, max=max(0, ncols // 4))
        rows, cols, vals = gen.matrix_from_row_lengths(nrows, ncols, lens, seed)
    return (nrows, ncols), (rows, cols, vals)


def random_tensor(rng, seed):
    dims = (int(rng.integers(1, 60)), int(rng.integers(1, 80)), int(rng.integers(1, 400)))
    cells = dims[0] * dims[1] * dims[2]
    dens = min(1.0, float(rng.uniform(0.0, 40000.0 / cells)))
    i, j, k, vals = gen.bernoulli_tensor3(dims, dens, seed)
    return dims, (i, j, k, vals)


@pytest.mark.parametrize("block", range(BLOCKS))
def test_random_matrices(comet, block):
    rng = np.random.default_rng(1000 + block)
    for case in range(20):
        seed = 100 * block + case
        (I, J), (rows, cols, vals) = random_matrix(rng, seed)
        layout = pick(rng, ["csr", "dcsr"])
        variant = pick(rng, [0, 1, 2])
        R = pick(rng, [1, 1, 2, 3, 5, 8, 12, 16, 17, 24, 32, 33, 48, 64, 100])
        say("matrix sweep block=%d case=%d %dx%d nnz=%d %s variant=%d R=%d" % (block, case, I, J, vals.numel(), layout, variant, R))
        pack = fmt.pack_csr if layout == "csr" else fmt.pack_dcsr
        A = comet.from_levels(pack(I, J, rows, cols, vals).to("cuda")).set_variant(variant)
        if R == 1:
            x = gen.dense_operand(seed, 0, (J,))
            y = torch.full((I,), float("nan"), dtype=torch.float64, device="cuda")
            comet.comet_spmv(A, dev(x), y)
            torch.cuda.synchronize()
            ref, absum = oracle.spmv(np_(rows), np_(cols), np_(vals), (I, J), np_(x))
            assert_values_close(np_(y), ref, absum, "spmv sweep %d/%d" % (block, case))
        else:
            B = gen.dense_operand(seed, 1, (J, R))
            C = torch.full((I, R), float("nan"), dtype=torch.float64, device="cuda")
            comet.comet_spmm(A, dev(B), C)
            torch.cuda.synchronize()
            ref, absum = oracle.spmm(np_(rows), np_(cols), np_(vals), (I, J), np_(B))
            assert_values_close(np_(C), ref, absum, "spmm sweep %d/%d" % (block, case))


@pytest.mark.parametrize("block", range(BLOCKS))
def test_random_tensors(comet, block):
    rng = np.random.default_rng(2000 + block)
    for case in range(15):
        seed = 1000 + 100 * block + case
        dims, (i, j, k, vals) = random_tensor(rng, seed)
        coords = (np_(i), np_(j), np_(k))
        variant = pick(rng, [0, 1, 2])
        mode = pick(rng, [0, 1, 2])
        R = pick(rng, [1, 2, 3, 7, 8, 16, 20, 32, 64, 65])
        source = pick(rng, ["csf", "coo"])
        say("tensor sweep block=%d case=%d dims=%s nnz=%d mode=%d variant=%d R=%d from %s" % (
            block, case, dims, vals.numel(), mode, variant, R, source))
        L = fmt.pack_csf3(dims, i, j, k, vals) if source == "csf" else fmt.pack_coo(dims, (i, j, k), vals)
        X = comet.from_levels(L.to("cuda"))
        a, b = [m for m in range(3) if m != mode]
        # leaf contraction of mode `mode`
        Xl = (X if (mode == 2 and source == "csf") else comet.comet_tensor_reorder(X, (a, b, mode))).set_variant(variant)
        v = gen.dense_operand(seed, 0, (dims[mode],))
        Y = comet.comet_ttv(Xl, mode, dev(v))
        ref = oracle.ttv_mode(coords, np_(vals), dims, mode, np_(v))
        torch.cuda.synchronize()
        want = oracle.compressed_pair_levels(ref["i"], ref["j"])
        assert_index_equal(np_(Y.pos(1)), want["pos2"], "ttv pos2")
        assert_index_equal(np_(Y.crd(0)), want["crd1"], "ttv crd1")
        assert_index_equal(np_(Y.crd(1)), want["crd2"], "ttv crd2")
        assert_values_close(np_(Y.vals()), ref["vals"], ref["abs"], "ttv sweep %d/%d" % (block, case))
        U = gen.dense_operand(seed, 1, (dims[mode], R))
        Ym = comet.comet_ttm(Xl, mode, dev(U))
        refm = oracle.ttm_mode(coords, np_(vals), dims, mode, np_(U))
        torch.cuda.synchronize()
        assert_values_close(np_(Ym.vals()).reshape(-1, R), refm["vals"], refm["abs"], "ttm sweep %d/%d" % (block, case))
        # the same tensor as a sorted coordinate list
        if mode == 2:
            Xc = comet.from_levels(fmt.pack_coo(dims, (i, j, k), vals).to("cuda")).set_variant(variant)
            Yc = comet.comet_ttv(Xc, 2, dev(v))
            torch.cuda.synchronize()
            assert_index_equal(np_(Yc.crd(0)), ref["i"], "coo ttv crd1")
            assert_index_equal(np_(Yc.crd(1)), ref["j"], "coo ttv crd2")
            assert_values_close(np_(Yc.vals()), ref["vals"], ref["abs"], "coo ttv sweep %d/%d" % (block, case))
            Yt = comet.comet_ttm(Xc, 2, dev(U))
            torch.cuda.synchronize()
            assert_index_equal(np_(Yt.crd(0)), refm["i"], "coo ttm crd1")
            assert_index_equal(np_(Yt.crd(1)), refm["j"], "coo ttm crd2")
            assert_values_close(np_(Yt.vals()).reshape(-1, R), refm["vals"], refm["abs"], "coo ttm sweep %d/%d" % (block, case))
        # MTTKRP for mode `mode`
        Xr = (X if (mode == 0 and source == "csf") else comet.comet_tensor_reorder(X, (mode, a, b))).set_variant(variant)
        F = [gen.dense_operand(seed, 2 + m, (dims[m], R)) for m in range(3)]
        M = torch.full((dims[mode], R), float("nan"), dtype=torch.float64, device="cuda")
        comet.comet_mttkrp(Xr, mode, [None if m == mode else dev(F[m]) for m in range(3)], M)
        torch.cuda.synchronize()
        refk, absk = oracle.mttkrp_mode(coords, np_(vals), dims, mode, [np_(f) for f in F])
        assert_values_close(np_(M), refk, absk, "mttkrp sweep %d/%d" % (block, case))
        if mode == 0 and source == "coo":        # the coordinate list itself, through its compressed copy
            M2 = comet.comet_mttkrp(X.set_variant(variant), 0, [None, dev(F[1]), dev(F[2])])
            torch.cuda.synchronize()
            assert_values_close(np_(M2), refk, absk, "coo mttkrp sweep %d/%d" % (block, case))
