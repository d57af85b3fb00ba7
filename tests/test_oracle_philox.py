"""Pins for the oracle's factor generator (CPU only).

Known answers published with Philox4x32-10, an independent scalar big-integer
implementation, closed-form statistics of Box-Muller normals, and the entry
statistics of U V^T / sqrt(r) from the paper's CLT appendix.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

from oracle import philox as px


def _kat(golden_dir):
    rows = []
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[:4], w[4:6], w[6:]))
    return rows


def test_philox_known_answers(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = px.philox4x32_10(np.array(ctr), np.array(key))
        assert [int(x) for x in got] == want


def _philox_scalar(ctr, key):
    """Independent implementation with Python integers (different code shape:
    explicit 64-bit products, key schedule precomputed)."""
    keys = [((key[0] + i * 0x9E3779B9) % 2**32, (key[1] + i * 0xBB67AE85) % 2**32) for i in range(10)]
    c = list(ctr)
    for k0, k1 in keys:
        prod_a = 0xD2511F53 * c[0]
        prod_b = 0xCD9E8D57 * c[2]
        c = [(prod_b >> 32) ^ c[1] ^ k0, prod_b % 2**32, (prod_a >> 32) ^ c[3] ^ k1, prod_a % 2**32]
    return c


def test_scalar_implementation_agrees_with_kat(golden_dir):
    for ctr, key, want in _kat(golden_dir):
        assert _philox_scalar(ctr, key) == want


def test_vectorised_equals_scalar_on_random_counters():
    rng = np.random.default_rng(7)
    ctr = rng.integers(0, 2**32, size=(200, 4), dtype=np.uint64)
    key = rng.integers(0, 2**32, size=(200, 2), dtype=np.uint64)
    got = px.philox4x32_10(ctr, key)
    for i in range(200):
        assert [int(x) for x in got[i]] == _philox_scalar([int(x) for x in ctr[i]], [int(x) for x in key[i]])


def test_stream_layout_brute_force():
    """Entry (i, j) of a [rows, r] factor is lane (i*r+j) % 4 of block (i*r+j) // 4
    with counter (block, 0, tensor_id, 0) and key (seed lo, seed hi)."""
    seed, tid = 0x0123456789ABCDEF, 7
    for rows, r in [(5, 3), (4, 2), (3, 8), (7, 1), (2, 16)]:
        M = px.factor_matrix(seed, tid, rows, r)
        for i in range(rows):
            for j in range(r):
                e = i * r + j
                w = _philox_scalar([e // 4, 0, tid, 0], [seed & 0xFFFFFFFF, seed >> 32])
                a, b = (w[0], w[1]) if (e % 4) < 2 else (w[2], w[3])
                ua = (2 * (a >> 9) + 1) / 2**24
                ub = (2 * (b >> 9) + 1) / 2**24
                rho = math.sqrt(-2.0 * math.log(ua))
                z = rho * (math.cos(2 * math.pi * ub) if e % 2 == 0 else math.sin(2 * math.pi * ub))
                assert M[i, j] == np.float32(z)


def test_high_counter_word_and_key_split():
    w = px.factor_words((5 << 32) | 9, 3, 2, first_block=(1 << 32) + 4)
    assert [int(x) for x in w[0]] == _philox_scalar([4, 1, 3, 0], [9, 5])
    assert [int(x) for x in w[1]] == _philox_scalar([5, 1, 3, 0], [9, 5])


def test_streams_differ_by_seed_and_tensor():
    a = px.factor_matrix(1, 0, 64, 4)
    assert not np.array_equal(a, px.factor_matrix(2, 0, 64, 4))
    assert not np.array_equal(a, px.factor_matrix(1, 1, 64, 4))
    assert np.array_equal(a, px.factor_matrix(1, 0, 64, 4))
    assert px.u_tensor_id(6) == 6 and px.v_tensor_id(6) == 7


def test_uniform_grid_is_exact_in_fp32():
    w = np.array([0, 1, 511, 512, 2**32 - 1, 0x80000000], dtype=np.uint64)
    u = px.uniform_open01(w)
    assert u[0] == 2.0**-24 and u[2] == 2.0**-24 and u[3] == 3 * 2.0**-24
    assert u[4] == 1 - 2.0**-24 and u[5] == 0.5 + 2.0**-24
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    assert (u > 0).all() and (u < 1).all()


def test_normal_statistics_and_bounds():
    z = px.factor_matrix(2024, 0, 1 << 20, 4).reshape(-1)
    n = z.size
    assert abs(z.mean()) < 5 / math.sqrt(n)
    assert abs(z.var() - 1) < 5 * math.sqrt(2 / n)
    assert abs(stats.skew(z)) < 5 * math.sqrt(6 / n)
    assert abs(stats.kurtosis(z)) < 5 * math.sqrt(24 / n)
    # u >= 2^-24 bounds the radius: |z| <= sqrt(-2 ln 2^-24)
    assert np.abs(z).max() <= math.sqrt(48 * math.log(2)) + 1e-6
    assert stats.kstest(z[:200000], "norm").pvalue > 1e-3
    # even and odd lanes (cos and sin branches) are uncorrelated
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 5 / math.sqrt(n / 2)


def test_box_muller_pair_radius():
    w = px.factor_words(99, 5, 1000)
    z = px.normals_from_words(w)
    u = px.uniform_open01(w)
    np.testing.assert_allclose(z[:, 0]**2 + z[:, 1]**2, -2 * np.log(u[:, 0]), rtol=1e-12)
    np.testing.assert_allclose(z[:, 2]**2 + z[:, 3]**2, -2 * np.log(u[:, 2]), rtol=1e-12)
    np.testing.assert_allclose(np.arctan2(z[:, 1], z[:, 0]) % (2 * np.pi), 2 * np.pi * u[:, 1], atol=1e-9)


@pytest.mark.parametrize("r", [1, 4, 16, 64, 256])
def test_clt_entry_statistics(r):
    """Appendix (multivariate CLT): every entry of U V^T / sqrt(r) has mean 0
    and variance 1 for every r; each summand u*v has fourth moment 9, so the
    excess kurtosis is 6/r and vanishes as r grows; distinct entries are
    uncorrelated."""
    m = n = 1024
    U = px.factor_matrix(31 + r, 0, m, r)
    V = px.factor_matrix(31 + r, 1, n, r)
    Z = (U @ V.T) / math.sqrt(r)
    N = Z.size
    # entries sharing a row of U or V are dependent; use loose 6-sigma bands
    # scaled by the effective sample size m (rows) for variance-type statistics
    assert abs(Z.mean()) < 6 / math.sqrt(N)
    assert abs(Z.var() - 1) < 6 * math.sqrt((2 + 6 / r) / N) + 6 * 2 / math.sqrt(r * m)
    kurt = stats.kurtosis(Z.reshape(-1))
    assert abs(kurt - 6 / r) < max(0.35 * 6 / r, 0.05)
    assert abs(np.mean(Z[:, :-1] * Z[:, 1:])) < 6 / math.sqrt(m * r) + 6 / math.sqrt(N)
    assert abs(np.mean(Z[:-1, :] * Z[1:, :])) < 6 / math.sqrt(n * r) + 6 / math.sqrt(N)


def test_bf16_rounding_matches_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40],
                                 dtype=np.float32)])
    # exact ties: 1 + 2^-8 lies half-way between two bf16 values
    ties = (1.0 + np.arange(1, 64, 2, dtype=np.float32) * 2.0**-8).astype(np.float32)
    x = np.concatenate([x, ties, -ties])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = px.round_to_bf16(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_bf16_factor_is_rounded_fp32_factor():
    a = px.factor_matrix(5, 2, 100, 8, "f32")
    b = px.factor_matrix(5, 2, 100, 8, "bf16")
    assert np.array_equal(b, px.round_to_bf16(a.astype(np.float32)).astype(np.float64))
    assert np.abs(a - b).max() <= np.abs(a).max() * 2.0**-8
