"""Pins for the oracle's primitives: Philox, the inverse-CDF rule, the W-ary tree.

None of these tests re-types an oracle formula: each compares the oracle with a
published vector, a value printed in the paper, or a brute-force definition.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_philox_known_answers():
    rows = _rows("philox4x32_10_kat.txt")
    assert len(rows) >= 2
    for r in rows:
        v = [int(x, 16) for x in r]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_philox_counter_and_key_sensitivity():
    base = oracle.philox4x32_10([5, 0, 1, 0], [9, 0])
    seen = {tuple(base)}
    for ctr, key in [([6, 0, 1, 0], [9, 0]), ([5, 1, 1, 0], [9, 0]), ([5, 0, 2, 0], [9, 0]),
                     ([5, 0, 1, 0], [10, 0]), ([5, 0, 1, 0], [9, 1])]:
        seen.add(tuple(oracle.philox4x32_10(ctr, key)))
    assert len(seen) == 6


def test_token_uniforms_are_24bit_and_uniform():
    n = 40000
    u = np.array([oracle.token_uniforms(123, t, 3) for t in range(n)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))          # exactly representable 24-bit fractions
    for col in range(2):
        hist = np.bincount((u[:, col] * 20).astype(int), minlength=20)
        chi2 = ((hist - n / 20) ** 2 / (n / 20)).sum()
        assert chi2 < 50.0                                        # 19 dof, p ~ 1e-4
    assert abs(np.corrcoef(u[:, 0], u[:, 1])[0, 1]) < 0.03
    # the uniforms are the top 24 bits of Philox words 0 and 1 with counter (t, 0, iter, 0), key = seed
    r = oracle.philox4x32_10([77, 0, 3, 0], [123, 0])
    assert oracle.token_uniforms(123, 77, 3) == ((int(r[0]) >> 8) / 2 ** 24, (int(r[1]) >> 8) / 2 ** 24)
    big = (5 << 32) | 9                                           # 64-bit token index and seed are split lo/hi
    r = oracle.philox4x32_10([9, 5, 1, 0], [0xDEADBEEF, 0x1234])
    assert oracle.token_uniforms((0x1234 << 32) | 0xDEADBEEF, big, 1)[0] == (int(r[0]) >> 8) / 2 ** 24


def test_init_z_uniform_over_topics():
    K = 37
    z = oracle.init_z(200000, K, 99)
    assert z.min() == 0 and z.max() == K - 1
    hist = np.bincount(z, minlength=K)
    chi2 = ((hist - z.size / K) ** 2 / (z.size / K)).sum()
    assert chi2 < 90.0                                            # 36 dof
    r = oracle.philox4x32_10([1234, 0, 0, 0], [99, 0])
    assert z[1234] == (int(r[0]) * K) >> 32


def _fig2():
    rows = _rows("fig2_inverse_cdf.txt")
    p = np.array([float(x) for x in rows[0][1:]])
    draws = [(float(a), int(b)) for a, b in rows[1:]]
    return p, draws


def test_fig2_example_sparse_branch():
    """Problem 1 with A_d = (2,1,3,2) and a flat Bhat row reproduces the figure's regions."""
    p, draws = _fig2()
    K = 4
    counts = np.round(p * 8).astype(np.int32)
    assert np.allclose(counts / 8.0, p)
    phi = np.full(K, 0.125, dtype=np.float32)
    c32 = np.cumsum(phi).astype(np.float32)
    for u, k1 in draws:
        k, det = oracle.sample(np.arange(K), counts, phi, c32, Q=0.5, u0=0.0, u1=u)
        assert det.branch == 1
        assert k + 1 == k1, (u, k, k1)


def test_fig2_example_dense_branch():
    """Problem 2 (pre-processed per word) with Bhat_v = p reproduces the figure's regions."""
    p, draws = _fig2()
    phi = p.astype(np.float32)
    c32 = np.cumsum(p).astype(np.float32)
    for u, k1 in draws:
        k, det = oracle.sample([0], [1], phi, c32, Q=1e9, u0=0.5, u1=u)
        assert det.branch == 2
        assert k + 1 == k1, (u, k, k1)
        assert oracle.position_in_prefix32(c32, np.float32(u)) + 1 == k1


def test_position_in_prefix_matches_linear_scan():
    rng = np.random.default_rng(0)
    for n in [1, 2, 3, 63, 64, 65, 1000]:
        c = np.cumsum(rng.random(n).astype(np.float32) ** 4).astype(np.float32)
        xs = np.concatenate([rng.random(200).astype(np.float32) * c[-1], c[:50], [np.float32(0.0), c[-1]]])
        for x in xs:
            hit = np.nonzero(c >= np.float32(x))[0]
            expect = int(hit[0]) if hit.size else n - 1
            assert oracle.position_in_prefix32(c, x) == expect


@pytest.mark.parametrize("W", [2, 3, 64])
@pytest.mark.parametrize("n", [1, 2, 5, 9, 64, 65, 100, 4096, 4097, 10000])
def test_wary_tree_query_equals_linear_scan(W, n):
    rng = np.random.default_rng(W * 100003 + n)
    vals = rng.random(n) ** 6                       # many tiny increments, some equal prefix values
    vals[rng.random(n) < 0.1] = 0.0
    c = np.cumsum(vals).astype(np.float32)
    if c[-1] == 0:
        c[-1] = 1.0
    tree = oracle.WaryTree(c, W)
    # structure: node i of an upper level equals node (i+1)W-1 of the level below (clamped at the end)
    for l in range(1, tree.levels):
        lower, upper = tree.level(l - 1), tree.level(l)
        assert upper.size == -(-lower.size // W)
        idx = np.minimum((np.arange(upper.size) + 1) * W - 1, lower.size - 1)
        assert np.array_equal(upper, lower[idx])
    assert tree.level(tree.levels - 1).size <= W
    xs = np.concatenate([rng.random(300).astype(np.float32) * c[-1], c[:: max(1, n // 50)], [np.float32(0), c[-1]]])
    for x in xs:
        hit = np.nonzero(c >= np.float32(x))[0]
        assert tree.query(x) == int(hit[0])


def test_three_ary_example_levels():
    """A 3-ary tree as in the tree-building figure: 9 leaves -> 3 nodes -> root window."""
    p = np.array([1, 2, 3, 4, 5, 6, 7, 8, 9], dtype=np.float32)
    c = np.cumsum(p).astype(np.float32)
    tree = oracle.WaryTree(c, 3)
    assert tree.levels == 2
    assert list(tree.level(1)) == [6.0, 21.0, 45.0]
    assert tree.query(6.0) == 2 and tree.query(6.5) == 3 and tree.query(45.0) == 8 and tree.query(0.0) == 0
