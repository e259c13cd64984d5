"""GPU parity of the holdout log-likelihood (document completion) against the oracle.

Both sides score held-out documents on the same frozen model: the GPU model is trained a few iterations and the
oracle is given its assignments, so Bhat and the prefix tables are identical.  Fold-in steps are compared one at
a time from identical assignments, as for training (a single boundary flip legitimately separates two chains)."""
import numpy as np
import pytest

import corpusgen
import oracle

pytestmark = pytest.mark.gpu


def saber():
    import paper_1610_02496_amd as pk
    return pk


def split_mask(doc_ptr, seed=None):
    T = int(doc_ptr[-1])
    if seed is None:
        pos = np.arange(T) - np.repeat(doc_ptr[:-1], np.diff(doc_ptr))
        return (pos % 2 == 0).astype(np.uint8)
    return (np.random.default_rng(seed).random(T) < 0.6).astype(np.uint8)


def trained_pair(K, seed=61, D=300, V=700, iters=4, **opts):
    c = corpusgen.tiny(seed, D, V, 20, 70.0)
    pk = saber()
    alpha = 50.0 / K
    g = pk.Saber(c.doc_ptr, c.word_ids, V, K, alpha, 0.01, 5, **opts)
    g.iterate(iters)
    o = oracle.Model(c.doc_ptr, c.word_ids, V, K, alpha, 0.01, 5)
    o.set_z(g.get_z(), it=g.get_iteration())
    phi, _ = g.get_phi(np.arange(0, V, 37, dtype=np.int32))
    assert np.array_equal(phi, o.phi[::37])                      # same frozen model on both sides
    return c, g, o


def margins(o, optr, ow, z_prev, tok, seed, it):
    """Oracle's distance from a decision boundary for the listed observed tokens (one fold-in step from z_prev)."""
    cd_ptr, cd_topic, cd_count = oracle.count_by_dz(optr, z_prev, o.K)
    doc_of = np.searchsorted(optr, tok, side="right") - 1
    out = np.empty(tok.size); zs = np.empty(tok.size, dtype=np.int64)
    for i, (t, d) in enumerate(zip(tok, doc_of)):
        a, b = cd_ptr[d], cd_ptr[d + 1]
        w = ow[t]
        u0, u1 = oracle.token_uniforms(seed, int(t), it)
        k, det = oracle.sample(cd_topic[a:b], cd_count[a:b], o.phi[w], o.c32[w], o.alpha * o.sum64[w], u0, u1)
        out[i] = det.margin; zs[i] = k
    return zs, out


@pytest.mark.parametrize("K,opts", [(100, {}), (1000, {}), (1000, {"light_word_tokens": -1}),
                                    (1000, {"light_word_tokens": 1 << 20}), (5000, {"block_threads": 256})])
def test_holdout_parity(K, opts):
    c, g, o = trained_pair(K, **opts)
    h = corpusgen.tiny(62, 120, 700, 20, 60.0)
    for mask in (split_mask(h.doc_ptr), split_mask(h.doc_ptr, seed=3)):
        obs = mask.astype(bool)
        optr = np.r_[0, np.cumsum(np.add.reduceat(mask.astype(np.int64), h.doc_ptr[:-1]) * (np.diff(h.doc_ptr) > 0))]
        optr = np.zeros(h.doc_ptr.size, dtype=np.int64)
        np.cumsum(np.bincount(np.repeat(np.arange(h.doc_ptr.size - 1), np.diff(h.doc_ptr))[obs],
                              minlength=h.doc_ptr.size - 1), out=optr[1:])
        ow = h.word_ids[obs]
        seed = 1234
        # no fold-in: identical state by construction
        ll_g, n_g, z_g = g.holdout_loglik(h.doc_ptr, h.word_ids, mask, 0, seed)
        ll_o, n_o, z_o = o.holdout_loglik(h.doc_ptr, h.word_ids, mask, 0, seed)
        assert n_g == n_o == int((~obs).sum()) and np.array_equal(z_g, z_o)
        assert abs(ll_g - ll_o) <= 1e-6 * abs(ll_o)
        # fold-in, one step at a time from identical assignments
        z_prev = z_o
        for step in range(3):
            ll_g, _, z_g = g.holdout_loglik(h.doc_ptr, h.word_ids, mask, 1, seed, z_init=z_prev)
            _, _, z_o = o.holdout_loglik(h.doc_ptr, h.word_ids, mask, 1, seed, z_init=z_prev, nthreads=4)
            bad = np.nonzero(z_g != z_o)[0]
            assert bad.size <= 1e-3 * z_o.size
            if bad.size:
                zs, mg = margins(o, optr, ow, z_prev, bad, seed, 1)
                assert np.array_equal(zs, z_o[bad]) and np.all(mg < 1e-5)
            # the score on the GPU's own assignments, re-evaluated by the oracle from exactly that state
            ll_ref, _, _ = o.holdout_loglik(h.doc_ptr, h.word_ids, mask, 0, seed, z_init=z_g)
            assert abs(ll_g - ll_ref) <= 1e-6 * abs(ll_ref)
            z_prev = z_g
        # free-running fold-in
        a = g.holdout_loglik(h.doc_ptr, h.word_ids, mask, 5, seed)[0]
        b = o.holdout_loglik(h.doc_ptr, h.word_ids, mask, 5, seed, nthreads=4)[0]
        assert abs(a - b) <= 1e-4 * abs(b)
    g.close(); o.close()


def test_holdout_leaves_the_model_alone_and_edge_cases():
    c, g, o = trained_pair(200)
    pk = saber()
    twin = pk.Saber(c.doc_ptr, c.word_ids, 700, 200, 50.0 / 200, 0.01, 5)
    twin.iterate(4)
    h = corpusgen.tiny(63, 50, 700, 20, 40.0)                       # Poisson lengths: contains short documents
    mask = split_mask(h.doc_ptr)
    z_before = g.get_z(); ll_before = g.loglik()
    g.holdout_loglik(h.doc_ptr, h.word_ids, mask, 3, 9)
    assert np.array_equal(g.get_z(), z_before) and g.loglik() == ll_before and g.get_iteration() == 4
    g.iterate(2); twin.iterate(2)
    assert np.array_equal(g.get_z(), twin.get_z())
    o.set_z(g.get_z(), it=g.get_iteration())
    # everything observed / nothing observed / empty documents / no documents
    ones = np.ones_like(mask); zeros = np.zeros_like(mask)
    ll, n, z = g.holdout_loglik(h.doc_ptr, h.word_ids, ones, 2, 9)
    assert n == 0 and ll == 0.0 and z.size == h.T
    ll, n, z = g.holdout_loglik(h.doc_ptr, h.word_ids, zeros, 2, 9)
    ref = o.holdout_loglik(h.doc_ptr, h.word_ids, zeros, 2, 9)
    assert n == h.T and z.size == 0 and abs(ll - ref[0]) <= 1e-6 * abs(ref[0])
    dp = np.array([0, 0, 3, 3, 4], dtype=np.int64); w = np.array([5, 5, 9, 650], dtype=np.int32)
    m = np.array([1, 0, 0, 0], dtype=np.uint8)
    got = g.holdout_loglik(dp, w, m, 2, 4); ref = o.holdout_loglik(dp, w, m, 2, 4)
    assert got[1] == ref[1] == 3 and np.array_equal(got[2], ref[2]) and abs(got[0] - ref[0]) <= 1e-6 * abs(ref[0])
    ll, n, z = g.holdout_loglik(np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint8), 1, 1)
    assert n == 0 and ll == 0.0
    with pytest.raises(pk.SaberError):
        g.holdout_loglik(dp, np.array([5, 5, 9, 700], dtype=np.int32), m, 1, 1)      # word id outside [0, V)
    with pytest.raises(pk.SaberError):
        g.holdout_loglik(dp, w, m, 0, 1, z_init=np.array([200], dtype=np.int32))      # topic outside [0, K)
    g.close(); twin.close(); o.close()
