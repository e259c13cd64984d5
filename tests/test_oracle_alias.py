"""Pins for the oracle's alias tables (the per-word structure Sec. 3.2.3 weighs against the tree) and for the
E-step that draws the dense term from them: hand-worked tables, the distribution every table must encode, the
measure a grid of draws induces, and the dense Eq. 1 for the whole two-branch sampler."""
import os

import numpy as np
import pytest
from scipy.stats import chi2 as chi2_dist

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "alias_sweep_examples.txt")


def golden_cases():
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        w, prob, alias = (part.split() for part in line.split("|"))
        yield np.array(w, dtype=np.float32), np.array(prob, dtype=np.float64), np.array(alias, dtype=np.int32)


def test_hand_worked_tables():
    n = 0
    for w, prob, alias in golden_cases():
        got_prob, got_alias = oracle.alias_build(w)
        assert np.allclose(got_prob, prob, rtol=0, atol=1e-6), w
        keep = prob < 1.0 - 1e-9                      # the alias of a full bucket is never used
        assert np.array_equal(got_alias[keep], alias[keep]), w
        n += 1
    assert n >= 4


@pytest.mark.parametrize("K", [1, 2, 3, 64, 65, 1000, 4097])
def test_table_encodes_the_distribution(K):
    rng = np.random.default_rng(K)
    for power in (1, 6, 30):                          # flat, skewed, a few items hold nearly all the mass
        p = (rng.random(K) ** power + 1e-12).astype(np.float32)
        prob, alias = oracle.alias_build(p)
        assert prob.min() >= 0.0 and prob.max() <= 1.0 and alias.min() >= 0 and alias.max() < K
        want = p.astype(np.float64) / p.astype(np.float64).sum()
        assert np.abs(oracle.alias_mass(prob, alias) - want).max() <= 2e-7 / K + 1e-7 * want.max()
        # a bucket that is not full hands its rest to an item that had more than a bucket's worth
        q = want * K
        part = prob < 1.0 - 1e-6
        assert np.all(q[alias[part]] > 1.0 - 1e-6)
        assert np.allclose(prob[q <= 1.0], q[q <= 1.0], rtol=1e-6, atol=1e-9)     # light items keep exactly their own mass


def test_scaling_the_weights_changes_nothing():
    rng = np.random.default_rng(3)
    p = (rng.random(200) ** 4).astype(np.float32) + np.float32(1e-6)
    a = oracle.alias_build(p)
    b = oracle.alias_build(p * np.float32(8.0))       # exact in binary32
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_draws_on_a_grid_induce_the_table():
    rng = np.random.default_rng(4)
    K = 6
    p = (rng.random(K) ** 3 + 0.01).astype(np.float32)
    prob, alias = oracle.alias_build(p)
    n = 1 << 16
    hist = np.zeros(K)
    for i in range(n):
        k, _ = oracle.alias_draw(prob, alias, i << 8)           # u = i / n
        hist[k] += 1
    assert np.abs(hist / n - oracle.alias_mass(prob, alias)).max() <= K / n
    # the bucket is floor(u K) and the fraction decides: spelled out for a few draws
    for bits in (0, 1, (1 << 24) - 1, 5_000_000, 12_345_678):
        b = (bits * K) >> 24
        frac = np.float32((bits * K) & 0xFFFFFF) * np.float32(2.0 ** -24)
        k, margin = oracle.alias_draw(prob, alias, bits)
        assert k == (b if frac < prob[b] else alias[b])
        assert margin == pytest.approx(abs(float(frac) - float(prob[b])) / K)


def test_alias_estep_chi_square_against_eq1():
    """Many tokens with the same (d, w): the two-branch sampler with an alias table for the dense term follows
    Eq. 1 (alpha included), and takes the dense branch as often as S / (S + Q) says."""
    K, V, L = 10, 3, 120000
    rng = np.random.default_rng(10)
    topics = np.array([1, 4, 5, 8], dtype=np.int32); counts = np.array([3, 1, 7, 2], dtype=np.int32)
    phi = (rng.random((V, K)) * 0.02 + 1e-4).astype(np.float32)
    _, s64 = oracle.build_prefix(phi)
    prob = np.empty((V, K), dtype=np.float32); alias = np.empty((V, K), dtype=np.int32)
    for v in range(V):
        prob[v], alias[v] = oracle.alias_build(phi[v])
    doc_ptr = np.array([0, L], dtype=np.int64); w = 2
    word_ids = np.full(L, w, dtype=np.int32)
    alpha = np.float32(0.7)
    z = np.empty(L, dtype=np.int32); br = np.empty(L, dtype=np.int8); mg = np.empty(L)
    oracle.lib().orc_estep_alias(1, doc_ptr.ctypes.data, word_ids.ctypes.data, K, alpha,
                                 np.array([0, 4], dtype=np.int64).ctypes.data, topics.ctypes.data, counts.ctypes.data,
                                 phi.ctypes.data, s64.ctypes.data, prob.ctypes.data, alias.ctypes.data, 42, 1,
                                 z.ctypes.data, br.ctypes.data, mg.ctypes.data, 2)
    a = np.full(K, float(alpha)); a[topics] += counts
    p = a * phi[w].astype(np.float64); p /= p.sum()
    hist = np.bincount(z, minlength=K)
    assert ((hist - L * p) ** 2 / (L * p)).sum() < chi2_dist.ppf(1 - 1e-4, K - 1)
    S = (counts * phi[w, topics].astype(np.float64)).sum(); Q = float(alpha) * s64[w]
    assert abs((br == 2).mean() - Q / (S + Q)) < 5e-3
    # the sparse-branch tokens are the ones the tree variant draws, with the same result
    c32, _ = oracle.build_prefix(phi)
    z_tree = np.empty(L, dtype=np.int32); br_tree = np.empty(L, dtype=np.int8)
    oracle.lib().orc_estep(1, doc_ptr.ctypes.data, word_ids.ctypes.data, K, alpha,
                           np.array([0, 4], dtype=np.int64).ctypes.data, topics.ctypes.data, counts.ctypes.data,
                           phi.ctypes.data, c32.ctypes.data, s64.ctypes.data, 42, 1, z_tree.ctypes.data,
                           None, None, br_tree.ctypes.data, None, 1)
    assert np.array_equal(br, br_tree) and np.array_equal(z[br == 1], z_tree[br_tree == 1])
    assert (z[br == 2] != z_tree[br == 2]).any()                 # another map from u to the topic, same distribution


def test_a_planted_mistake_is_caught():
    """The mass check fails for a table whose alias points one item too far (an off-by-one in the pairing)."""
    rng = np.random.default_rng(5)
    p = (rng.random(50) ** 5 + 1e-6).astype(np.float32)
    prob, alias = oracle.alias_build(p)
    want = p.astype(np.float64) / p.astype(np.float64).sum()
    wrong = (alias + 1) % p.size
    assert np.abs(oracle.alias_mass(prob, wrong) - want).max() > 1e-3
    assert np.abs(oracle.alias_mass(1.0 - prob, alias) - want).max() > 1e-3    # kept and handed-over parts swapped
