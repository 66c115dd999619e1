"""The entry point for callers that cannot allocate (comet_spmv_static) against comet_spmv.

Collected last on purpose (the file name sorts after the other test files): the full test run stops at the
first failure, and a failure here must not hide the parity tests.
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


def _matrix(scale, seed):
    c = gen.config_spmm(seed=seed, device=DEV, scale=scale, R=1)
    rows, cols, vals = c["coo"]
    n = c["dims"][0]
    return n, rows, cols, vals, c["B"].reshape(-1).contiguous()


def _run_pair(comet, n, rows, cols, vals, x, layout):
    L = (fmt.pack_csr if layout == "csr" else fmt.pack_dcsr)(n, n, rows, cols, vals)
    A = comet.from_levels(L).set_variant(2)          # the tiled kernels: the ones that use the carry scratch
    want = torch.full((n,), float("nan"), dtype=torch.float64, device=DEV)
    comet.comet_spmv(A, x, want)
    got = torch.full((n,), float("nan"), dtype=torch.float64, device=DEV)
    comet.comet_spmv_static(A, x, got)
    torch.cuda.synchronize()
    return got, want


@pytest.mark.parametrize("layout", ["csr", "dcsr"])
def test_two_calls_in_a_row_the_second_smaller(comet, layout):
    """Both calls share the one static scratch array: the second, smaller problem must not be disturbed by
    what the first left there.  The same kernels run as in comet_spmv, so the results are bit-identical;
    both are also held to the oracle with the tolerance of the parity tests."""
    for scale, seed in ((0.2, 3), (0.02, 4)):        # 3.7 M nonzeros (rows cut over many chunks), then 370 K
        n, rows, cols, vals, x = _matrix(scale, seed)
        print("spmv_static layout=%s n=%d nnz=%d" % (layout, n, vals.numel()), flush=True)
        got, want = _run_pair(comet, n, rows, cols, vals, x, layout)
        assert torch.equal(got, want)
        ref, absum = oracle.spmv(np_(rows), np_(cols), np_(vals), (n, n), np_(x))
        assert_values_close(np_(got), ref, absum, "spmv_static %s" % layout)


def test_small_problem_on_the_automatic_path(comet):
    """The automatic choice sends a small matrix to kernels that need no scratch at all."""
    c = gen.config_spmv(seed=0, device=DEV)
    rows, cols, vals = c["coo"]
    n = c["dims"][0]
    A = comet.from_levels(fmt.pack_csr(n, n, rows, cols, vals))
    y = torch.full((n,), float("nan"), dtype=torch.float64, device=DEV)
    comet.comet_spmv_static(A, c["x"], y)
    torch.cuda.synchronize()
    ref, absum = oracle.spmv(np_(rows), np_(cols), np_(vals), (n, n), np_(c["x"]))
    assert_values_close(np_(y), ref, absum, "spmv_static config 1")


def test_rejects_what_does_not_fit_and_coordinate_lists(comet):
    # 96 M nonzeros need more than the 2 MiB of static scratch: refused, nothing is enqueued
    n, per = 1 << 20, 92
    rows = torch.arange(n, device=DEV).repeat_interleave(per)
    cols = (torch.arange(n * per, device=DEV) % per) * 11000 + rows % 9973      # increasing inside a row, < n
    vals = torch.ones(n * per, dtype=torch.float64, device=DEV)
    A = comet.from_levels(fmt.pack_csr(n, n, rows, cols, vals)).set_variant(2)
    x = torch.ones(n, dtype=torch.float64, device=DEV)
    y = torch.full((n,), 7.0, dtype=torch.float64, device=DEV)
    with pytest.raises(comet.CometError) as e:
        comet.comet_spmv_static(A, x, y)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
    del A, rows, cols, vals
    r = torch.tensor([0, 1, 1], device=DEV)
    c = torch.tensor([1, 0, 2], device=DEV)
    v = torch.ones(3, dtype=torch.float64, device=DEV)
    Ac = comet.from_levels(fmt.pack_coo((2, 3), (r, c), v))
    with pytest.raises(comet.CometError) as e:
        comet.comet_spmv_static(Ac, torch.ones(3, dtype=torch.float64, device=DEV), torch.zeros(2, dtype=torch.float64, device=DEV))
    assert e.value.status == 4
