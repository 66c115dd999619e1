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
