"""Pins for the oracle's random stream: Philox integers, uniforms, Box-Muller normals."""
import numpy as np
import pytest
from scipy import stats

from oracle import acc_oracle as orc
from conftest import golden_path


def _kat_rows():
    rows = []
    for line in open(golden_path("philox4x32_10_kat.txt")):
        line = line.split("#")[0].replace("->", " ").split()
        if line:
            rows.append([int(t, 16) for t in line])
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for row in rows:
        out = orc.philox4x32_10(np.array(row[0:4], np.uint32), np.array(row[4:6], np.uint32))
        assert [int(v) for v in out] == row[6:10]


def test_philox_vectorised_equals_one_by_one():
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 2**32, size=(37, 4), dtype=np.uint64).astype(np.uint32)
    key = rng.integers(0, 2**32, size=(37, 2), dtype=np.uint64).astype(np.uint32)
    batched = orc.philox4x32_10(ctr, key)
    for t in range(37):
        assert np.array_equal(batched[t], orc.philox4x32_10(ctr[t], key[t]))


def test_counter_map():
    """Entry [q, j] is the Philox call with counter (g>>2, j, 0, g>>34), key (seed lo, seed hi)."""
    seed = 0x0123456789ABCDEF
    words = orc.sketch_words(seed, 0, 50, 7)
    assert words.shape == (13, 7, 4) and words.dtype == np.uint32
    key = np.array([0x89ABCDEF, 0x01234567], np.uint32)
    for q, j in [(0, 0), (3, 5), (12, 6)]:
        want = orc.philox4x32_10(np.array([q, j, 0, 0], np.uint32), key)
        assert np.array_equal(words[q, j], want)
    # a row offset only shifts the token-group index
    shifted = orc.sketch_words(seed, 8, 42, 7)
    assert np.array_equal(shifted, words[2:])
    # token indices beyond 2^34 reach counter word 3
    big = orc.sketch_words(seed, 1 << 36, 4, 2)
    want = orc.philox4x32_10(np.array([0, 1, 0, 4], np.uint32), key)
    assert np.array_equal(big[0, 1], want)
    with pytest.raises(ValueError):
        orc.sketch_words(seed, 2, 4, 2)


def test_streams_and_seeds_differ():
    a = orc.sketch_words(1, 0, 64, 8)
    assert not np.array_equal(a, orc.sketch_words(2, 0, 64, 8))
    assert not np.array_equal(a, orc.sketch_words(1, 0, 64, 8, stream=1))
    assert not np.array_equal(a, orc.sketch_words(1 << 32, 0, 64, 8))


def test_uniform_exact_and_open_interval():
    x = np.array([0, 1, 511, 512, 0x7FFFFFFF, 0x80000000, 0xFFFFFFFF], np.uint32)
    u = orc.uniform_from_word(x)
    assert u[0] == 2.0 ** -24 and u[1] == 2.0 ** -24 and u[2] == 2.0 ** -24
    assert u[3] == 1.5 * 2.0 ** -23
    assert u[-1] == 1.0 - 2.0 ** -24
    assert np.all(u > 0) and np.all(u < 1)
    # every value is exactly representable in float32 (the GPU starts from the same real number)
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    # midpoint: x = 2^31 -> (2^22 + 0.5) 2^-23
    assert u[5] == 0.5 + 2.0 ** -24


def test_box_muller_polar_identities():
    """z_even^2 + z_odd^2 = -2 ln u_first and the angle of (z_even, z_odd) is 2 pi u_second."""
    rng = np.random.default_rng(1)
    words = rng.integers(0, 2**32, size=(1000, 4), dtype=np.uint64).astype(np.uint32)
    z = orc.normals_from_words(words)
    u = ((words >> 9).astype(np.float64) + 0.5) / 2.0 ** 23
    for a in (0, 2):
        r2 = z[:, a] ** 2 + z[:, a + 1] ** 2
        assert np.allclose(r2, -2.0 * np.log(u[:, a]), rtol=1e-12)
        ang = np.mod(np.arctan2(z[:, a + 1], z[:, a]), 2 * np.pi)
        assert np.allclose(ang, 2 * np.pi * u[:, a + 1], atol=1e-9)


def test_sketch_matrix_layout():
    """Token 4q+w, column j takes word w of call (q, j); entries are z / sqrt(r); rows >= n dropped."""
    seed, n, r = 7, 10, 3
    S = orc.sketch_matrix(seed, n, r)
    assert S.shape == (n, r)
    words = orc.sketch_words(seed, 0, n, r)
    for (i, j) in [(0, 0), (1, 2), (6, 1), (9, 2)]:
        z = orc.normals_from_words(words[i // 4, j])
        assert S[i, j] == z[i % 4] / np.sqrt(3.0)
    # global token index: a shard starting at row 4 sees rows 4.. of the global matrix
    assert np.array_equal(orc.sketch_matrix(seed, 6, r, row_offset=4), S[4:10])


def test_normal_moments_and_ks():
    r = 256
    S = orc.sketch_matrix(3, 40000, r)            # 10.24 M entries
    z = (S * np.sqrt(r)).ravel()
    n = z.size
    assert abs(z.mean()) < 4.0 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 4.0 * np.sqrt(2.0 / n)
    assert abs(stats.skew(z)) < 4.0 * np.sqrt(6.0 / n)
    assert abs(stats.kurtosis(z, fisher=False) - 3.0) < 0.01
    assert abs(np.abs(z).max()) < 5.77            # radius is capped at sqrt(-2 ln 2^-24) = 5.768
    ks = stats.kstest(z[:: 10], "norm")
    assert ks.pvalue > 1e-3
    # columns and token quadruples are uncorrelated: S^T S ~ (n/r) I, S S^T has unit mean diagonal
    G = S.T @ S
    assert np.allclose(np.diag(G), 40000 / r, rtol=0.05)
    off = G - np.diag(np.diag(G))
    assert np.abs(off).max() < 6.0 * np.sqrt(40000) / r
    Ssmall = S[:512]
    assert abs(np.mean(np.sum(Ssmall * Ssmall, axis=1)) - 1.0) < 0.02
    # neighbouring tokens of one Philox call (the sin/cos pair) are uncorrelated
    assert abs(np.mean(S[0::4] * S[1::4]) * r) < 5.0 / np.sqrt(n / 4)
