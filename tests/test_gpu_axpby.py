"""GPU parity of the scaled / accumulating products (comet_spmv_axpby, comet_spmm_axpby, comet_mttkrp_axpby):
y = alpha * (product) + beta * y, through the C ABI, every element against the CPU oracle
(oracle.axpby applied to the oracle's product).  Same inputs, kernel variants and tolerance as
test_gpu_parity.py; what must not be read (the old result when beta == 0, the operands when alpha == 0) is
filled with NaN.
"""
import numpy as np
import pytest
import torch

import oracle
from synth import formats as fmt
from synth import generate as gen
from test_gpu_parity import MATRIX_CASES, TENSOR_CASES, VARIANTS, _heavy_row_matrix, comet, dev, say  # noqa: F401
from util import assert_values_close, np_

pytestmark = pytest.mark.gpu

SCALARS = [(1.0, 1.0), (-0.75, 2.5), (3.0, 0.0), (0.0, -1.5), (1.0, 0.0)]


def _old(shape, beta, seed):
    """The result's previous contents: seeded values, or NaN where they must not be read."""
    old = gen.dense_operand(seed, 9, shape)
    return old, (torch.full(shape, float("nan"), dtype=torch.float64) if beta == 0.0 else old)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("alpha,beta", SCALARS)
@pytest.mark.parametrize("layout", ["csr", "dcsr"])
@pytest.mark.parametrize("name", ["config1", "zipf_rows", "edge_lengths", "one_full_row", "hypersparse", "empty", "long_row"])
def test_spmv_axpby(comet, name, layout, alpha, beta, variant):
    (I, J), (rows, cols, vals) = MATRIX_CASES[name]
    say("spmv_axpby case=%s layout=%s alpha=%g beta=%g variant=%d" % (name, layout, alpha, beta, variant))
    pack = fmt.pack_csr if layout == "csr" else fmt.pack_dcsr
    A = comet.from_levels(pack(I, J, rows, cols, vals).to("cuda")).set_variant(variant)
    x = gen.dense_operand(1, 0, (J,))
    old, given = _old((I,), beta, 31)
    y = dev(given).clone()
    xin = torch.full((J,), float("nan"), dtype=torch.float64) if alpha == 0.0 else x
    comet.comet_spmv_axpby(A, alpha, dev(xin), beta, y)
    torch.cuda.synchronize()
    prod, pabs = oracle.spmv(np_(rows), np_(cols), np_(vals), (I, J), np_(x))
    ref, absum = oracle.axpby(alpha, prod, pabs, beta, np_(old))
    assert_values_close(np_(y), ref, absum, "spmv_axpby %s" % name)


@pytest.mark.parametrize("variant", [1, 2, 0])
@pytest.mark.parametrize("alpha,beta", SCALARS)
@pytest.mark.parametrize("R", [8, 32, 96])
@pytest.mark.parametrize("name,layout", [("zipf_rows", "csr"), ("edge_lengths", "csr"), ("edge_lengths", "dcsr"),
                                         ("hypersparse", "dcsr"), ("empty", "csr"), ("long_row", "csr")])
def test_spmm_axpby(comet, name, layout, R, alpha, beta, variant):
    (I, J), (rows, cols, vals) = MATRIX_CASES[name]
    say("spmm_axpby case=%s layout=%s R=%d alpha=%g beta=%g variant=%d" % (name, layout, R, alpha, beta, variant))
    pack = fmt.pack_csr if layout == "csr" else fmt.pack_dcsr
    A = comet.from_levels(pack(I, J, rows, cols, vals).to("cuda")).set_variant(variant)
    B = gen.dense_operand(2, 0, (J, R))
    old, given = _old((I, R), beta, 32)
    C = dev(given).clone()
    Bin = torch.full((J, R), float("nan"), dtype=torch.float64) if alpha == 0.0 else B
    comet.comet_spmm_axpby(A, alpha, dev(Bin), beta, C)
    torch.cuda.synchronize()
    prod, pabs = oracle.spmm(np_(rows), np_(cols), np_(vals), (I, J), np_(B))
    ref, absum = oracle.axpby(alpha, prod, pabs, beta, np_(old))
    assert_values_close(np_(C), ref, absum, "spmm_axpby %s R=%d" % (name, R))


@pytest.mark.parametrize("alpha,beta", [(1.0, 1.0), (-0.5, 2.0), (2.0, 0.0)])
@pytest.mark.parametrize("R", [16, 32, 64])
@pytest.mark.parametrize("layout", ["csr", "dcsr"])
def test_spmm_axpby_with_heavy_rows(comet, layout, R, alpha, beta):
    """The matrix whose long rows go through the heavy-row sweep: its reduction applies the scalars too."""
    (I, J), (rows, cols, vals) = _heavy_row_matrix()
    say("spmm_axpby heavy layout=%s R=%d alpha=%g beta=%g" % (layout, R, alpha, beta))
    pack = fmt.pack_csr if layout == "csr" else fmt.pack_dcsr
    A = comet.from_levels(pack(I, J, rows, cols, vals).to("cuda"))
    assert A.heavy_plan()[0] > 0
    B = gen.dense_operand(2, 0, (J, R))
    old, given = _old((I, R), beta, 33)
    C = dev(given).clone()
    comet.comet_spmm_axpby(A, alpha, dev(B), beta, C)
    torch.cuda.synchronize()
    prod, pabs = oracle.spmm(np_(rows), np_(cols), np_(vals), (I, J), np_(B))
    ref, absum = oracle.axpby(alpha, prod, pabs, beta, np_(old))
    assert_values_close(np_(C), ref, absum, "spmm_axpby heavy R=%d" % R)


def test_accumulating_into_zeros_equals_the_plain_product(comet):
    """beta = 1 on a zero result and alpha = 1, beta = 0 on NaN both give comet_spmm's result bit for bit."""
    (I, J), (rows, cols, vals) = MATRIX_CASES["zipf_rows"]
    A = comet.from_levels(fmt.pack_csr(I, J, rows, cols, vals).to("cuda"))
    B = dev(gen.dense_operand(2, 0, (J, 32)))
    plain = comet.comet_spmm(A, B)
    acc = torch.zeros((I, 32), dtype=torch.float64, device="cuda")
    comet.comet_spmm_axpby(A, 1.0, B, 1.0, acc)
    over = torch.full((I, 32), float("nan"), dtype=torch.float64, device="cuda")
    comet.comet_spmm_axpby(A, 1.0, B, 0.0, over)
    torch.cuda.synchronize()
    assert torch.equal(plain, acc) and torch.equal(plain, over)


@pytest.mark.parametrize("variant", [1, 2, 0])
@pytest.mark.parametrize("alpha,beta", SCALARS[:4])
@pytest.mark.parametrize("R", [1, 16, 64])
@pytest.mark.parametrize("name", ["zipf_mttkrp", "mode_of_two", "single_slice", "long_slice", "long_fiber", "empty", "single"])
def test_mttkrp_axpby(comet, name, R, alpha, beta, variant):
    dims, (i, j, k, vals) = TENSOR_CASES[name]
    say("mttkrp_axpby case=%s R=%d alpha=%g beta=%g variant=%d" % (name, R, alpha, beta, variant))
    X = comet.from_levels(fmt.pack_csf3(dims, i, j, k, vals).to("cuda")).set_variant(variant)
    B, C = gen.dense_operand(5, 0, (dims[1], R)), gen.dense_operand(5, 1, (dims[2], R))
    old, given = _old((dims[0], R), beta, 34)
    M = dev(given).clone()
    nan = lambda t: torch.full(tuple(t.shape), float("nan"), dtype=torch.float64)
    fs = [None, dev(nan(B) if alpha == 0.0 else B), dev(nan(C) if alpha == 0.0 else C)]
    comet.comet_mttkrp_axpby(X, 0, alpha, fs, beta, M)
    torch.cuda.synchronize()
    prod, pabs = oracle.mttkrp(np_(i), np_(j), np_(k), np_(vals), dims, np_(B), np_(C))
    ref, absum = oracle.axpby(alpha, prod, pabs, beta, np_(old))
    assert_values_close(np_(M), ref, absum, "mttkrp_axpby %s R=%d" % (name, R))


def test_mttkrp_axpby_on_a_coordinate_list(comet):
    dims, (i, j, k, vals) = TENSOR_CASES["zipf_mttkrp"]
    X = comet.from_levels(fmt.pack_coo(dims, (i, j, k), vals).to("cuda"))
    R = 16
    B, C = gen.dense_operand(5, 0, (dims[1], R)), gen.dense_operand(5, 1, (dims[2], R))
    old = gen.dense_operand(35, 9, (dims[0], R))
    M = dev(old).clone()
    comet.comet_mttkrp_axpby(X, 0, 0.5, [None, dev(B), dev(C)], 1.0, M)
    torch.cuda.synchronize()
    prod, pabs = oracle.mttkrp(np_(i), np_(j), np_(k), np_(vals), dims, np_(B), np_(C))
    ref, absum = oracle.axpby(0.5, prod, pabs, 1.0, np_(old))
    assert_values_close(np_(M), ref, absum, "mttkrp_axpby coo")
