"""The seeded input generators: determinism, structure, and the stated distributions (CPU only)."""
import numpy as np
import torch

from synth import generate as gen
from synth import rng


def test_streams_are_reproducible_and_offset_consistent():
    a = rng.uniform01(0, 3, 1000)
    b = rng.uniform01(0, 3, 400, offset=600)
    assert torch.equal(a[600:], b)
    assert not torch.equal(rng.uniform01(0, 4, 1000), a)
    assert float(a.min()) >= 0.0 and float(a.max()) < 1.0
    assert abs(float(a.mean()) - 0.5) < 0.05


def test_mix64_matches_the_published_splitmix64_finaliser():
    # first outputs of splitmix64 seeded with 0: state advances by the golden gamma, then mixes
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    gamma = 0x9E3779B97F4A7C15
    for n, w in enumerate(want, start=1):
        z = (n * gamma) & ((1 << 64) - 1)
        assert rng._mix64_int(z) == w
        t = torch.tensor([z - (1 << 64) if z >= (1 << 63) else z], dtype=torch.int64)
        got = int(rng.mix64(t)[0]) & ((1 << 64) - 1)
        assert got == w


def test_spmv_config_has_exactly_ten_distinct_sorted_columns_per_row():
    c = gen.config_spmv(seed=0)
    rows, cols, vals = c["coo"]
    assert rows.numel() == 40960
    assert torch.equal(torch.bincount(rows), torch.full((4096,), 10))
    key = rows * 4096 + cols
    assert bool((key[1:] > key[:-1]).all())
    assert float(vals.min()) >= -1.0 and float(vals.max()) < 1.0
    c2 = gen.config_spmv(seed=0)
    assert all(torch.equal(a, b) for a, b in zip(c["coo"], c2["coo"]))


def test_zipf_row_lengths_follow_the_clamped_law():
    n = 200_000
    l = gen.zipf_row_lengths(n, 1.8, 10_000, 0).numpy()
    from scipy.special import zeta
    z = float(zeta(1.8, 1))
    assert abs((l == 1).mean() - 1.0 / z) < 0.01
    assert abs((l == 2).mean() - 2 ** -1.8 / z) < 0.005
    assert l.max() <= 10_000 and l.min() >= 1


def test_tensor_generator_is_sorted_distinct_exact_count_and_deterministic():
    c = gen.config_ttm(seed=0, scale=1e-4, chunk=1 << 16)
    i, j, k, vals = c["coo"]
    I, J, K = c["dims"]
    assert vals.numel() == c["info"]["nnz"] == 10_000
    key = (i * J + j) * K + k
    assert bool((key[1:] > key[:-1]).all())
    assert int(i.max()) < I and int(j.max()) < J and int(k.max()) < K
    c2 = gen.config_ttm(seed=0, scale=1e-4, chunk=1 << 16)
    assert all(torch.equal(a, b) for a, b in zip(c["coo"], c2["coo"]))
    c3 = gen.config_ttm(seed=1, scale=1e-4, chunk=1 << 16)
    assert not torch.equal(c3["coo"][0], i)


def test_zipf_modes_are_skewed():
    c = gen.config_ttv(seed=0, scale=1e-3, chunk=1 << 18)
    i = c["coo"][0]
    counts = torch.bincount(i).sort(descending=True).values.double()
    assert counts[0] > 20 * counts[len(counts) // 2]


def test_mttkrp_factors_share_columns_across_ranks():
    a = gen.config_mttkrp(seed=0, scale=1e-5, R=16, chunk=1 << 14)
    b = gen.config_mttkrp(seed=0, scale=1e-5, R=64, chunk=1 << 14)
    assert torch.equal(a["B"], b["B"][:, :16]) and torch.equal(a["C"], b["C"][:, :16])


def test_lexi_relabel_renames_indices_and_orders_by_first_nonzero():
    """synth/lexi.py (Section 7 of the paper, reordering): the relabelled tensor is the same tensor under one
    permutation per mode, and after the iteration for a mode its indices are numbered in the order in which they
    first appear when the nonzeros are sorted by the other modes."""
    from synth import lexi
    dims = (7, 5, 6)
    i, j, k, vals = gen.bernoulli_tensor3(dims, 0.2, seed=3)
    (ni, nj, nk), labels = lexi.lexi_relabel((i, j, k), dims, sweeps=2)
    for n, d in enumerate(dims):
        assert sorted(labels[n].tolist()) == list(range(d))           # a permutation of the mode's indices
    dense = torch.zeros(dims, dtype=torch.float64)
    dense[i, j, k] = vals
    moved = torch.zeros(dims, dtype=torch.float64)
    moved[ni, nj, nk] = vals
    assert torch.equal(moved[labels[0]][:, labels[1]][:, :, labels[2]], dense)
    # hand example, one iteration for the rows of a 4 x 4 matrix: rows sorted by their smallest column
    rows = torch.tensor([0, 0, 1, 2, 3, 3])
    cols = torch.tensor([2, 3, 0, 1, 0, 3])
    (nr, nc), lab = lexi.lexi_relabel((rows, cols), (4, 4), sweeps=1)
    # rows: first appearance in column order: col 0 -> rows 1, 3; col 1 -> row 2; col 2 -> row 0
    assert lab[0].tolist() == [3, 0, 2, 1]
    # columns, with the new row labels (row 0 = old 1 has col 0; row 1 = old 3 has cols 0, 3; row 2 = old 2 has col 1; row 3 = old 0 has cols 2, 3)
    assert lab[1].tolist() == [0, 2, 3, 1]
    (sr, sc), sv = lexi.sort_nonzeros((nr, nc), (4, 4), torch.arange(6, dtype=torch.float64))
    key = (sr * 4 + sc).tolist()
    assert key == sorted(key) and len(set(key)) == 6
