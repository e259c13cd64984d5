"""Pins for the oracle's M-step, split sampler, whole iteration and log-likelihood.

Each check compares the oracle with a definition written out independently here
(dense numpy histograms, the dense Eq. 1, closed forms for K=1), with values the
paper states, or with statistical properties of the generative process.
"""
import numpy as np
import pytest
from scipy.optimize import linear_sum_assignment
from scipy.stats import chi2 as chi2_dist

import corpusgen
import oracle


def small_corpus(seed=3, D=60, V=90, K=12, mean_len=25.0):
    c = corpusgen.tiny(seed, D, V, K, mean_len)
    return c


# ------------------------------------------------------------------------------- counts
def test_prose_example_counts():
    """Sec. 2.1: D=3, T=8, V=5, K=3; both tokens of document 1 carry topic 3, so A_13 = 2."""
    doc_ptr = np.array([0, 2, 5, 8], dtype=np.int64)
    word_ids = np.array([3, 4, 0, 1, 4, 0, 2, 2], dtype=np.int32)
    z = np.array([2, 2, 0, 0, 2, 1, 1, 1], dtype=np.int32)           # 0-based topics
    cd_ptr, topic, count = oracle.count_by_dz(doc_ptr, z, 3)
    assert list(cd_ptr) == [0, 1, 3, 4]
    assert list(topic) == [2, 0, 2, 1] and list(count) == [2, 2, 1, 3]   # A_13 = 2 (1-based)
    cwk, ck = oracle.count_by_vz(word_ids, z, 5, 3)
    assert cwk.sum() == 8 and list(ck) == [2, 3, 3]
    assert cwk[4, 2] == 2 and cwk[2, 1] == 2 and cwk[0, 0] == 1 and cwk[0, 1] == 1


def test_counts_match_dense_histograms_and_invariants():
    c = small_corpus()
    K, V = 12, c.spec.V
    rng = np.random.default_rng(1)
    z = rng.integers(0, K, c.T).astype(np.int32)
    cd_ptr, topic, count = oracle.count_by_dz(c.doc_ptr, z, K)
    cwk, ck = oracle.count_by_vz(c.word_ids, z, V, K)
    doc_of = np.repeat(np.arange(c.spec.D), np.diff(c.doc_ptr))
    dense_A = np.zeros((c.spec.D, K), dtype=np.int64)
    np.add.at(dense_A, (doc_of, z), 1)
    dense_B = np.zeros((V, K), dtype=np.int64)
    np.add.at(dense_B, (c.word_ids, z), 1)
    assert np.array_equal(cwk, dense_B)
    assert np.array_equal(ck, dense_B.sum(0)) and np.array_equal(ck, dense_A.sum(0))
    assert cwk.sum() == c.T
    for d in range(c.spec.D):
        a, b = cd_ptr[d], cd_ptr[d + 1]
        nz = np.nonzero(dense_A[d])[0]
        assert np.array_equal(topic[a:b], nz)                        # ascending topic order, no zeros stored
        assert np.array_equal(count[a:b], dense_A[d, nz])
        assert count[a:b].sum() == c.doc_ptr[d + 1] - c.doc_ptr[d]
    # equals the naive rebuild: sort tokens by (d, k), then scan runs (Sec. 3.3)
    order = np.lexsort((z, doc_of))
    pairs = np.stack([doc_of[order], z[order]], 1)
    uniq, cnt = np.unique(pairs, axis=0, return_counts=True)
    assert np.array_equal(uniq[:, 1], topic) and np.array_equal(cnt, count)


def test_count_by_dz_rejects_bad_topic():
    with pytest.raises(ValueError):
        oracle.count_by_dz(np.array([0, 2]), np.array([0, 5], dtype=np.int32), 3)


# ------------------------------------------------------------------------------- Bhat (Eq. 2)
def test_phi_columns_sum_to_one_and_k1_closed_form():
    c = small_corpus(seed=5, V=200)
    V, K, beta = c.spec.V, 7, 0.01
    z = np.random.default_rng(2).integers(0, K, c.T).astype(np.int32)
    cwk, ck = oracle.count_by_vz(c.word_ids, z, V, K)
    phi = oracle.preprocess(cwk, ck, beta)
    assert phi.dtype == np.float32 and phi.min() > 0
    assert np.allclose(phi.astype(np.float64).sum(0), 1.0, rtol=0, atol=2e-6)   # each column sums to 1
    # K = 1: Bhat_v = (n_v + beta) / (T + V beta)
    cwk1, ck1 = oracle.count_by_vz(c.word_ids, np.zeros(c.T, dtype=np.int32), V, 1)
    phi1 = oracle.preprocess(cwk1, ck1, beta)[:, 0].astype(np.float64)
    n_v = np.bincount(c.word_ids, minlength=V)
    assert np.allclose(phi1, (n_v + beta) / (c.T + V * beta), rtol=3e-7)
    # empty topic: Bhat = 1/V
    cwk0 = np.zeros((V, 2), dtype=np.int32); cwk0[:, 0] = cwk1[:, 0]
    phi0 = oracle.preprocess(cwk0, np.array([c.T, 0]), beta)
    assert np.allclose(phi0[:, 1], 1.0 / V, rtol=3e-7)


def test_phi_is_single_rounded_binary32():
    """Each operation of Eq. 2 is one IEEE binary32 operation (numpy float32 arithmetic is the same)."""
    rng = np.random.default_rng(4)
    V, K = 50, 9
    cwk = rng.integers(0, 40_000_000, (V, K)).astype(np.int32)       # above 2^24: conversion must round
    ck = cwk.astype(np.int64).sum(0)
    beta = np.float32(0.01)
    phi = oracle.preprocess(cwk, ck, beta)
    denom = ck.astype(np.float32) + np.float32(V) * beta
    expect = (cwk.astype(np.float32) + beta) / denom[None, :]
    assert expect.dtype == np.float32 and np.array_equal(phi, expect)


def test_prefix_table_against_exact_sums():
    rng = np.random.default_rng(6)
    phi = (rng.random((5, 3000)) ** 8).astype(np.float32) + np.float32(1e-9)
    c32, sum64 = oracle.build_prefix(phi)
    from fractions import Fraction
    for v in [0, 4]:
        exact = np.cumsum([Fraction(float(x)) for x in phi[v]])
        approx = np.array([float(x) for x in exact])
        assert np.allclose(c32[v], approx.astype(np.float32), rtol=1.2e-7, atol=0)   # within one rounding
        assert abs(sum64[v] - float(exact[-1])) <= 1e-12 * float(exact[-1])
    assert np.all(np.diff(c32.astype(np.float64), axis=1) >= 0)


# ------------------------------------------------------------------------------- split sampler (Alg. 2)
def dense_eq1(topics, counts, phi_w, alpha):
    """Eq. 1 evaluated densely: p(k) = (A_dk + alpha) Bhat_vk / sum."""
    A = np.zeros(phi_w.size)
    A[topics] = counts
    p = (A + alpha) * phi_w.astype(np.float64)
    return p / p.sum()


def toy_token(seed, K=9, nnz=4):
    rng = np.random.default_rng(seed)
    topics = np.sort(rng.choice(K, nnz, replace=False)).astype(np.int32)
    counts = rng.integers(1, 6, nnz).astype(np.int32)
    phi_w = (rng.random(K) ** 2 * 0.01 + 1e-5).astype(np.float32)
    c32, s64 = oracle.build_prefix(phi_w[None, :])
    return topics, counts, phi_w, c32[0], float(s64[0])


@pytest.mark.parametrize("seed,alpha", [(0, 0.5), (1, 5.0), (2, 0.05)])
def test_split_sampler_induced_measure(seed, alpha):
    """Sweep (u0,u1) over a fine grid: the area mapped to each k must equal Eq. 1."""
    topics, counts, phi_w, c32, s64 = toy_token(seed)
    p = dense_eq1(topics, counts, phi_w, alpha)
    n0, n1 = 300, 400
    area = np.zeros(phi_w.size)
    branch1 = 0
    for i in range(n0):
        for j in range(n1):
            k, det = oracle.sample(topics, counts, phi_w, c32, alpha * s64, (i + 0.5) / n0, (j + 0.5) / n1)
            area[k] += 1
            branch1 += det.branch == 1
    area /= n0 * n1
    assert np.abs(area - p).max() < 6e-3
    S = (counts * phi_w[topics].astype(np.float64)).sum()
    assert abs(branch1 / (n0 * n1) - S / (S + alpha * s64)) < 4e-3


def test_all_topics_present_reduces_to_vanilla_on_sparse_branch():
    """With K_d = K and alpha -> 0 the sparse branch alone is the vanilla sampler of Sec. 2.3."""
    rng = np.random.default_rng(8)
    K = 7
    counts = rng.integers(1, 9, K).astype(np.int32)
    phi_w = (rng.random(K) * 0.1 + 0.01).astype(np.float32)
    c32, s64 = oracle.build_prefix(phi_w[None, :])
    p = counts * phi_w.astype(np.float64)
    c = np.cumsum(p)
    for u in rng.random(500):
        k, det = oracle.sample(np.arange(K), counts, phi_w, c32[0], 1e-30, 0.5, u)
        assert det.branch == 1 and k == int(np.nonzero(c >= u * c[-1])[0][0])


def test_estep_chi_square_against_eq1():
    """Many tokens with the same (d, w): Philox-driven draws follow Eq. 1 (alpha included)."""
    K, V, L = 10, 3, 120000
    rng = np.random.default_rng(10)
    topics = np.array([1, 4, 5, 8], dtype=np.int32); counts = np.array([3, 1, 7, 2], dtype=np.int32)
    phi = (rng.random((V, K)) * 0.02 + 1e-4).astype(np.float32)
    c32, s64 = oracle.build_prefix(phi)
    doc_ptr = np.array([0, L], dtype=np.int64); w = 2
    word_ids = np.full(L, w, dtype=np.int32)
    alpha = np.float32(0.7)
    z = np.empty(L, dtype=np.int32); br = np.empty(L, dtype=np.int8)
    oracle.lib().orc_estep(1, doc_ptr.ctypes.data, word_ids.ctypes.data, K, alpha,
                           np.array([0, 4], dtype=np.int64).ctypes.data, topics.ctypes.data, counts.ctypes.data,
                           phi.ctypes.data, c32.ctypes.data, s64.ctypes.data, 42, 1, z.ctypes.data,
                           None, None, br.ctypes.data, None, 1)
    p = dense_eq1(topics, counts, phi[w], float(alpha))
    hist = np.bincount(z, minlength=K)
    stat = ((hist - L * p) ** 2 / (L * p)).sum()
    assert stat < chi2_dist.ppf(1 - 1e-4, K - 1)
    # a sampler that dropped alpha would never emit topics outside the document's row
    assert hist[[0, 2, 3, 6, 7, 9]].sum() > 0
    S = (counts * phi[w, topics].astype(np.float64)).sum()
    frac = (br == 1).mean(); pb = S / (S + float(alpha) * s64[w])
    assert abs(frac - pb) < 5 * np.sqrt(pb * (1 - pb) / L)


def test_margin_reports_distance_to_boundary():
    topics, counts, phi_w, c32, s64 = toy_token(3)
    Q = 0.3 * s64
    S = (counts * phi_w[topics].astype(np.float64)).sum()
    thr = S / (S + Q)
    k, det = oracle.sample(topics, counts, phi_w, c32, Q, thr - 1e-7, 0.5)
    assert det.branch == 1 and det.margin <= 1.0000001e-7
    k, det = oracle.sample(topics, counts, phi_w, c32, Q, thr + 1e-7, 0.5)
    assert det.branch == 2 and det.margin <= 1.0000001e-7
    cp = np.cumsum(counts * phi_w[topics].astype(np.float64)) / S
    k, det = oracle.sample(topics, counts, phi_w, c32, Q, 0.0, cp[1] + 1e-9)
    assert k == topics[2] and det.margin < 2e-9


# ------------------------------------------------------------------------------- whole iteration (Alg. 1)
def test_iteration_determinism_threads_and_invariants():
    c = small_corpus(seed=7, D=80, V=150, K=20, mean_len=40.0)
    args = (c.doc_ptr, c.word_ids, c.spec.V, 20, 2.5, 0.01, 17)
    m1, m2 = oracle.Model(*args), oracle.Model(*args)
    assert np.array_equal(m1.z, oracle.init_z(c.T, 20, 17))
    m1.iterate(3, nthreads=1); m2.iterate(3, nthreads=4)
    assert np.array_equal(m1.z, m2.z) and m1.iter == 3
    assert np.array_equal(m1.cwk, m2.cwk)
    cd_ptr, topic, count = m1.cd
    assert count.sum() == c.T and m1.cwk.sum() == c.T and np.array_equal(m1.ck, m1.cwk.sum(0))
    lens = np.diff(c.doc_ptr)
    assert np.array_equal(np.add.reduceat(np.r_[count, 0], cd_ptr[:-1]) * (np.diff(cd_ptr) > 0), lens * (lens > 0))
    m3 = oracle.Model(c.doc_ptr, c.word_ids, c.spec.V, 20, 2.5, 0.01, 18)
    m3.iterate(3)
    assert not np.array_equal(m1.z, m3.z)                              # the seed matters
    # E-step reads frozen counts: re-sampling from the same state gives the same answer (BSP, Sec. 2.4)
    za = m1.estep_detail()[0]; zb = m1.estep_detail(nthreads=3)[0]
    assert np.array_equal(za, zb)


def test_single_topic_stays_put():
    c = small_corpus(seed=9)
    m = oracle.Model(c.doc_ptr, c.word_ids, c.spec.V, 1, 50.0, 0.01, 1)
    m.iterate(2)
    assert not m.z.any()
    n_v = np.bincount(c.word_ids, minlength=c.spec.V)
    V, T, beta = c.spec.V, c.T, np.float64(np.float32(0.01))
    # K = 1: every token's predictive likelihood is Bhat_w, so LL = mean ln((n_w+beta)/(T+V beta))
    expect = np.log((n_v[c.word_ids] + beta) / (T + V * beta)).mean()
    assert abs(m.loglik() - expect) < 1e-6 * abs(expect)


def test_loglik_equals_dense_predictive_likelihood():
    c = small_corpus(seed=11, D=40, V=70, K=8, mean_len=30.0)
    K, alpha = 8, np.float32(6.25)
    m = oracle.Model(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 5)
    m.iterate(2)
    doc_of = np.repeat(np.arange(c.spec.D), np.diff(c.doc_ptr))
    A = np.zeros((c.spec.D, K)); np.add.at(A, (doc_of, m.z), 1)
    lens = np.diff(c.doc_ptr).astype(np.float64)
    theta = (A + float(alpha)) / (lens[:, None] + K * float(alpha))
    phi = m.phi.astype(np.float64)
    ll = np.log((theta[doc_of] * phi[c.word_ids]).sum(1)).mean()
    assert abs(m.loglik() - ll) < 1e-9 * abs(ll)


def test_planted_topics_are_recovered():
    """Data drawn from the LDA process with 10 well separated topics: LL rises to the level of the
    planted assignment and the fitted topic-word columns match the planted ones."""
    spec = corpusgen.CorpusSpec("rec", 600, 800, 48000, "poisson", 80.0, 0.0, 10, 1.1, 0.02, 0.1, 10, 1, 11)
    c = corpusgen.generate(spec, nthreads=2)
    m = oracle.Model(c.doc_ptr, c.word_ids, spec.V, 10, 0.1, 0.01, 5)
    ll = [m.loglik()]
    for _ in range(4):
        m.iterate(30); ll.append(m.loglik())
    assert all(b > a for a, b in zip(ll, ll[1:]))
    truth = oracle.Model(c.doc_ptr, c.word_ids, spec.V, 10, 0.1, 0.01, 5)
    truth.set_z(c.true_topic)
    assert ll[0] < truth.loglik() - 0.4 and abs(ll[-1] - truth.loglik()) < 0.06
    unit = lambda a: a / np.linalg.norm(a, axis=0, keepdims=True)
    sim = unit(m.phi.astype(np.float64)).T @ unit(truth.phi.astype(np.float64))
    r, cidx = linear_sum_assignment(-sim)
    assert (sim[r, cidx] > 0.9).sum() >= 8


def test_config1_likelihood_rises():
    c = corpusgen.generate(corpusgen.SPECS["C1"], nthreads=2)
    s = c.spec
    assert 95_000 < c.T < 105_000 and c.doc_ptr.size == 1001 and c.word_ids.max() < 5000
    m = oracle.Model(c.doc_ptr, c.word_ids, s.V, s.K, s.alpha, s.beta, s.seed)
    ll0 = m.loglik(); m.iterate(10); ll10 = m.loglik()
    assert ll10 > ll0 + 0.05


def test_sample_tokens_is_the_estep_restricted_to_a_list():
    c = small_corpus(seed=13, D=50, V=80, K=10, mean_len=30.0)
    m = oracle.Model(c.doc_ptr, c.word_ids, c.spec.V, 10, 0.7, 0.01, 3)
    m.iterate(1)
    z, S, p, br, mg = m.estep_detail()
    tok = np.random.default_rng(0).choice(c.T, 200, replace=False)
    z2, S2, p2, br2, mg2 = m.sample_tokens(tok)
    assert np.array_equal(z2, z[tok]) and np.array_equal(S2, S[tok]) and np.array_equal(mg2, mg[tok])
    assert np.array_equal(br2, br[tok]) and np.array_equal(p2, p[tok])
