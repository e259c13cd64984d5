"""Pins for the oracle's holdout log-likelihood (document completion; the metric Sec. 4 names without a formula).

Everything here is checked against something other than the oracle's own arithmetic: closed forms, a dense numpy
evaluation from the returned assignments, count invariants, and the expected behaviour on a planted corpus."""
import numpy as np

import corpusgen
import oracle


def split_mask(doc_ptr, rng=None):
    """Even positions of every document are observed, odd ones scored (or a random half)."""
    T = int(doc_ptr[-1])
    pos = np.arange(T) - np.repeat(doc_ptr[:-1], np.diff(doc_ptr))
    if rng is None:
        return (pos % 2 == 0).astype(np.uint8)
    return (rng.random(T) < 0.5).astype(np.uint8)


def dense_score(model, doc_ptr, word_ids, observed, z_obs, K, alpha):
    """sum_k theta_dk Bhat_wk written out densely: theta from the histogram of the observed assignments."""
    phi = model.phi.astype(np.float64)                      # [V, K]
    D = doc_ptr.size - 1
    doc_of = np.repeat(np.arange(D), np.diff(doc_ptr))
    obs = observed.astype(bool)
    A = np.zeros((D, K)); np.add.at(A, (doc_of[obs], z_obs), 1.0)
    L_obs = A.sum(1)
    assert np.array_equal(L_obs, np.bincount(doc_of[obs], minlength=D))
    a = float(np.float32(alpha))
    theta = (A + a) / (L_obs[:, None] + K * a)
    sc = ~obs
    p = np.einsum("tk,tk->t", theta[doc_of[sc]], phi[word_ids[sc]])
    return float(np.log(p).mean()), int(sc.sum())


def trained(seed=3, D=120, V=150, K_true=6, K=8, iters=15):
    c = corpusgen.tiny(seed, D, V, K_true, 60.0)
    m = oracle.Model(c.doc_ptr, c.word_ids, V, K, 0.3, 0.01, 11)
    m.iterate(iters, nthreads=2)
    return c, m


def test_dense_evaluation_and_fold_in_bookkeeping():
    c, m = trained()
    h = corpusgen.tiny(77, 40, 150, 6, 50.0)               # held-out documents from the same planted model family
    mask = split_mask(h.doc_ptr)
    cwk_before = m.cwk.copy(); phi_before = m.phi.copy()
    for n_fold in (0, 1, 5):
        ll, scored, z_obs = m.holdout_loglik(h.doc_ptr, h.word_ids, mask, n_fold, 5)
        assert z_obs.size == int(mask.sum()) and z_obs.min() >= 0 and z_obs.max() < m.K
        ref, n_ref = dense_score(m, h.doc_ptr, h.word_ids, mask, z_obs, m.K, 0.3)
        assert scored == n_ref == int((mask == 0).sum())
        assert abs(ll - ref) < 1e-12 * abs(ref)
    assert np.array_equal(m.cwk, cwk_before) and np.array_equal(m.phi, phi_before)     # the model stays frozen


def test_initial_assignment_and_supplied_state():
    c, m = trained()
    h = corpusgen.tiny(78, 30, 150, 6, 40.0)
    mask = split_mask(h.doc_ptr, np.random.default_rng(1))
    n_obs = int(mask.sum())
    _, _, z0 = m.holdout_loglik(h.doc_ptr, h.word_ids, mask, 0, 99)
    assert np.array_equal(z0, oracle.init_z(n_obs, m.K, 99))       # Philox iteration 0 over the observed tokens
    z_mine = np.random.default_rng(2).integers(0, m.K, n_obs).astype(np.int32)
    ll, _, z_back = m.holdout_loglik(h.doc_ptr, h.word_ids, mask, 0, 99, z_init=z_mine)
    assert np.array_equal(z_back, z_mine)
    ref, _ = dense_score(m, h.doc_ptr, h.word_ids, mask, z_mine, m.K, 0.3)
    assert abs(ll - ref) < 1e-12 * abs(ref)
    # the draws are keyed by (seed, position among the observed tokens, iteration): the thread count is immaterial
    a = m.holdout_loglik(h.doc_ptr, h.word_ids, mask, 3, 7)
    b = m.holdout_loglik(h.doc_ptr, h.word_ids, mask, 3, 7, nthreads=3)
    assert a[0] == b[0] and np.array_equal(a[2], b[2])


def test_closed_forms():
    # K = 1: theta = 1, so the score is the mean of ln Bhat_w = ln((n_w + beta) / (T + V beta)) over scored tokens
    c = corpusgen.tiny(5, 60, 40, 3, 30.0)
    m = oracle.Model(c.doc_ptr, c.word_ids, 40, 1, 0.5, 0.01, 1)
    h = corpusgen.tiny(6, 25, 40, 3, 30.0)
    mask = split_mask(h.doc_ptr)
    ll, scored, _ = m.holdout_loglik(h.doc_ptr, h.word_ids, mask, 4, 3)
    n_w = np.bincount(c.word_ids, minlength=40).astype(np.float64)
    ref = np.log((n_w + 0.01) / (c.T + 40 * 0.01))[h.word_ids[mask == 0]].mean()
    assert abs(ll - ref) < 1e-6 * abs(ref)                          # Bhat itself is binary32
    # nothing observed: theta is uniform, the score is the mean of ln((1/K) sum_k Bhat_wk)
    c2, m2 = trained()
    h2 = corpusgen.tiny(9, 25, 150, 6, 30.0)
    none = np.zeros(h2.word_ids.size, dtype=np.uint8)
    ll2, scored2, z2 = m2.holdout_loglik(h2.doc_ptr, h2.word_ids, none, 3, 3)
    assert scored2 == h2.T and z2.size == 0
    ref2 = np.log(m2.phi.astype(np.float64).sum(1) / m2.K)[h2.word_ids].mean()
    assert abs(ll2 - ref2) < 1e-9 * abs(ref2)
    # everything observed: nothing to score
    allobs = np.ones(h2.word_ids.size, dtype=np.uint8)
    ll3, scored3, z3 = m2.holdout_loglik(h2.doc_ptr, h2.word_ids, allobs, 2, 3)
    assert scored3 == 0 and ll3 == 0.0 and z3.size == h2.T


def test_fold_in_helps_on_a_planted_corpus():
    """Held-out documents drawn from the same planted topics: folding in the observed half must beat the
    uniform-theta score by a clear margin, and more iterations must not hurt."""
    spec = corpusgen.CorpusSpec("plant", 400, 300, 400 * 80, "poisson", 80.0, 0.0, 8, 1.1, 0.05, 0.2, 8, 1, 21)
    full = corpusgen.generate(spec, nthreads=2)
    D_train = 300
    cut = int(full.doc_ptr[D_train])
    m = oracle.Model(full.doc_ptr[:D_train + 1], full.word_ids[:cut], 300, 8, 0.2, 0.01, 4)
    m.iterate(40, nthreads=4)
    hp = full.doc_ptr[D_train:] - cut; hw = full.word_ids[cut:]
    mask = split_mask(hp)
    ll0 = m.holdout_loglik(hp, hw, np.zeros_like(mask), 0, 1)[0]          # uniform theta, all tokens scored
    ll = [m.holdout_loglik(hp, hw, mask, n, 1, nthreads=4)[0] for n in (0, 2, 20)]
    assert ll[2] > ll[1] > ll[0]
    assert ll[2] > ll0 + 0.2
    assert ll[2] < 0.0 and ll[2] < m.loglik() + 0.5
