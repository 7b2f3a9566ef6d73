"""Pins for the oracle's label generator (paper Sec. 2, Eq. 1).  CPU only."""

import math
import os

import numpy as np
import pytest
import scipy.stats
import torch

from oracle import rng

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------------
# Philox4x32-10 core
# ---------------------------------------------------------------------------------
def _philox_bigint(ctr, key):
    """Second implementation with Python integers, written from the published
    round function: nothing shared with oracle/rng.py."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k[0] = (k[0] + 0x9E3779B9) % (1 << 32)
            k[1] = (k[1] + 0xBB67AE85) % (1 << 32)
        a = 0xD2511F53 * c[0]
        b = 0xCD9E8D57 * c[2]
        c = [(b >> 32) ^ c[1] ^ k[0], b % (1 << 32), (a >> 32) ^ c[3] ^ k[1], a % (1 << 32)]
    return c


def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        out = rng.philox4x32_10(*v[:6])
        assert [int(o) for o in out] == v[6:]
        assert _philox_bigint(v[:4], v[4:6]) == v[6:]
        n += 1
    assert n == 3


def test_philox_vectorised_matches_bigint():
    g = np.random.default_rng(123)
    ctr = g.integers(0, 1 << 32, size=(2000, 4), dtype=np.uint64)
    k0, k1 = 0xDEADBEEF, 0x12345678
    out = rng.philox4x32_10(ctr[:, 0], ctr[:, 1], ctr[:, 2], ctr[:, 3], k0, k1)
    out = np.stack(out, axis=1)
    for i in range(len(ctr)):
        assert _philox_bigint([int(x) for x in ctr[i]], [k0, k1]) == [int(x) for x in out[i]]


def test_label_counter_convention():
    # entry (class j, index i) is word 0 of philox(counter=(i, j, 0, 0), key=seed)
    seed = (0xABCDEF01 << 32) | 0x00000007
    T = rng.make_synthetic_labels(seed, classes=5, dim=9, dist=rng.UNIFORM01, kappa=1.0)
    for j in (0, 3, 4):
        for i in (0, 1, 8):
            r = _philox_bigint([i, j, 0, 0], [0x00000007, 0xABCDEF01])
            assert T[j, i] == np.float32((r[0] >> 8) / 2.0 ** 24)


# ---------------------------------------------------------------------------------
# exact transforms
# ---------------------------------------------------------------------------------
def test_uniform_identities_and_ranges():
    r0 = np.array([0, 255, 256, 0x7FFFFFFF, 0x80000000, 0xFFFFFFFF, 0xFFFFFF00], dtype=np.uint32)
    u = rng.uniform01_from_word(r0)
    expect = [(int(x) >> 8) / 2.0 ** 24 for x in r0]
    assert u.dtype == np.float32 and u.tolist() == expect
    assert u.min() == 0.0 and u.max() == 1.0 - 2.0 ** -24
    pm = rng.transform(rng.UNIFORM_PM1, 1.0, r0, r0)
    # 2u-1 is exact: (r0>>8 - 2^23) / 2^23
    assert pm.tolist() == [((int(x) >> 8) - (1 << 23)) / 2.0 ** 23 for x in r0]
    b = rng.transform(rng.BINARY_PM1, 1.0, r0, r0)
    assert b.tolist() == [-1, -1, -1, -1, 1, 1, 1]
    k = rng.transform(rng.UNIFORM01, 10.0, r0, r0)
    assert k.tolist() == [float(np.float32(10.0) * np.float32(e)) for e in expect]


def test_label_table_distribution_eq1():
    # Eq. 1: kappa * U(0,1): mean kappa/2, variance kappa^2/12, support [0,kappa)
    kappa = 10.0
    T = rng.make_synthetic_labels(11, classes=47, dim=60 * 400, dist=rng.UNIFORM01, kappa=kappa)
    assert T.shape == (47, 24000) and T.dtype == np.float32
    n = T.size
    assert T.min() >= 0.0 and T.max() < kappa
    assert abs(T.mean() - kappa / 2) < 5 * kappa / math.sqrt(12 * n)
    assert abs(T.var() - kappa ** 2 / 12) < 0.02
    assert scipy.stats.kstest(T.ravel()[:200000] / kappa, "uniform").pvalue > 1e-3
    B = rng.make_synthetic_labels(13, 47, 2048, rng.BINARY_PM1)
    assert set(np.unique(B)) == {-1.0, 1.0} and abs(B.mean()) < 5 / math.sqrt(B.size)
    P = rng.make_synthetic_labels(7, 47, 64, rng.UNIFORM_PM1)
    assert P.min() >= -1.0 and P.max() < 1.0


def test_prefix_stability_and_seeds():
    a = rng.make_synthetic_labels(21, 10, 33, rng.NORMAL)
    b = rng.make_synthetic_labels(21, 47, 100, rng.NORMAL)
    assert np.array_equal(a, b[:10, :33])
    c = rng.make_synthetic_labels(22, 10, 33, rng.NORMAL)
    assert not np.array_equal(a, c)
    assert np.array_equal(a, rng.make_synthetic_labels(21, 10, 33, rng.NORMAL))


# ---------------------------------------------------------------------------------
# normal transform: the fixed float32 sequence against double-precision Box-Muller
# ---------------------------------------------------------------------------------
def _box_muller_double(r0, r1):
    u1 = ((r0.astype(np.uint64) >> 8) + 1).astype(np.float64) * 2.0 ** -24
    u2 = (r1.astype(np.uint64) >> 8).astype(np.float64) * 2.0 ** -24
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def test_normal_matches_double_box_muller():
    g = np.random.default_rng(5)
    r0 = g.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    r1 = g.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    # edge words: u1 = 2^-24, u1 = 1, u1 just below 1, mantissa at the sqrt(2) split,
    # u2 on and around the quadrant boundaries and the reflection point
    edge0 = np.array([0, 0xFFFFFFFF, 0xFFFFFE00, 0x6A09E600, 0x6A09E700, 0xB504F300, 0xB504F400, 0x7FFFFF00, 0x80000000],
                     dtype=np.uint32)
    edge1 = np.array([0, 0x40000000, 0x3FFFFF00, 0x40000100, 0x80000000, 0xC0000000, 0x20000000, 0x20000100, 0xFFFFFF00],
                     dtype=np.uint32)
    e0, e1 = np.meshgrid(edge0, edge1)
    r0 = np.concatenate([r0, e0.ravel()])
    r1 = np.concatenate([r1, e1.ravel()])
    z = rng.normal_from_words(r0, r1)
    ref = _box_muller_double(r0, r1)
    assert z.dtype == np.float32 and np.all(np.isfinite(z))
    # error budget: ln u1 within ~2 ulp (halved by the square root), cosine within
    # ~2 ulp of its own value, one more rounding for the product: 4 ulp(|ref|),
    # with a floor for the exact zeros of the cosine (ref carries ~1e-16 there
    # while z is exactly 0).
    ulp = np.spacing(np.abs(ref).astype(np.float32)).astype(np.float64)
    err = np.abs(z.astype(np.float64) - ref)
    assert np.all(err <= np.maximum(4 * ulp, 1e-9))
    # hard bound of the construction: |z| <= sqrt(2 * 24 * ln 2)
    assert np.max(np.abs(z)) <= math.sqrt(48 * math.log(2)) + 1e-5


def test_normal_distribution():
    T = rng.make_synthetic_labels(31, classes=100, dim=10000, dist=rng.NORMAL)
    x = T.ravel().astype(np.float64)
    n = x.size
    assert abs(x.mean()) < 5 / math.sqrt(n)
    assert abs(x.var() - 1.0) < 5 * math.sqrt(2.0 / n)
    assert abs(scipy.stats.skew(x)) < 5 * math.sqrt(6.0 / n)
    assert abs(scipy.stats.kurtosis(x)) < 5 * math.sqrt(24.0 / n)
    assert scipy.stats.kstest(x[:300000], "norm").pvalue > 1e-3


# ---------------------------------------------------------------------------------
# inputs of interior segments, initial weights, bf16 rounding
# ---------------------------------------------------------------------------------
def test_segment_inputs_definition():
    T = rng.make_synthetic_labels(7, 47, 64, rng.UNIFORM_PM1)
    y = np.array([3, 46, 0, 3], dtype=np.int32)
    X = rng.make_segment_inputs(5, T, y, first_sample=(1 << 32) - 2, sigma=0.05)
    assert X.shape == (4, 64) and X.dtype == np.float32
    # sample n = first + row; counter = (i, n_lo, 2, n_hi)
    for row, n in enumerate([(1 << 32) - 2, (1 << 32) - 1, 1 << 32, (1 << 32) + 1]):
        for i in (0, 63):
            r = _philox_bigint([i, n % (1 << 32), 2, n >> 32], [5, 0])
            z = rng.normal_from_words(np.array([r[0]], np.uint32), np.array([r[1]], np.uint32))[0]
            assert X[row, i] == np.float32(T[y[row], i] + np.float32(0.05) * z)
    # statistically: residual / sigma is standard normal
    Xb = rng.make_segment_inputs(5, T, np.zeros(4000, np.int32), 0, 0.05)
    res = (Xb.astype(np.float64) - T[0].astype(np.float64)) / 0.05
    assert abs(res.mean()) < 0.02 and abs(res.std() - 1) < 0.02
    # window invariance: rows depend on the global sample index only
    Xc = rng.make_segment_inputs(5, T, np.zeros(10, np.int32), 100, 0.05)
    assert np.array_equal(Xb[100:110], Xc)


def test_init_weights_distribution_and_convention():
    W, b = rng.init_weights(3, layer=2, fan_out=64, fan_in=784)
    assert W.shape == (64, 784) and b.shape == (64,) and W.dtype == np.float32
    bound = 1.0 / math.sqrt(784)
    assert np.abs(W).max() <= bound and np.abs(b).max() <= bound
    assert abs(W.mean()) < 5 * bound / math.sqrt(3 * W.size)
    assert abs(W.var() - bound ** 2 / 3) < 0.05 * bound ** 2
    r = _philox_bigint([783, 5, 1, 2], [3, 0])
    bf = np.float32(1.0) / np.sqrt(np.float32(784))
    assert W[5, 783] == (np.float32(2) * np.float32((r[0] >> 8) / 2.0 ** 24) - np.float32(1)) * bf
    r = _philox_bigint([784, 5, 1, 2], [3, 0])          # bias = column fan_in
    assert b[5] == (np.float32(2) * np.float32((r[0] >> 8) / 2.0 ** 24) - np.float32(1)) * bf


def test_bf16_rounding_against_library_cast():
    g = np.random.default_rng(9)
    bits = g.integers(0, 1 << 32, size=1_000_000, dtype=np.uint64).astype(np.uint32)
    ties = np.array([0x3F808000, 0x3F818000, 0x3F80FFFF, 0x3F807FFF, 0x7F7FFFFF, 0x00008000, 0x80008000, 0x7F800000],
                    dtype=np.uint32)
    x = np.concatenate([bits, ties]).view(np.float32)
    x = x[~np.isnan(x)]
    mine = rng.round_to_bf16(x)
    lib = torch.from_numpy(x.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(mine.view(np.uint32), lib.view(np.uint32))
    assert np.isnan(rng.round_to_bf16(np.array([np.nan], np.float32))[0])
