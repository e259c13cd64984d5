"""GPU parity at the benchmark's full size and launch configuration (library defaults, as bench.py uses).

Corpus: the 100M-token NYTimes-shaped synthetic corpus (D=300K, V=100K), fitted with K=1,000 and K=10,000.
What the oracle can afford is compared in full (initial assignment, A, C_k, B for K=1,000); the E-step is
compared on a random sample of tokens the oracle evaluates one by one, plus invariants that hold at any size.
"""
import sys
import time

import numpy as np
import pytest

import corpusgen
import oracle

pytestmark = pytest.mark.gpu

N_SAMPLE = 200_000


def say(*a):
    print(*a, file=sys.stderr, flush=True)


_CORPORA = {}


def corpus_for(name):
    """C3: the benchmark corpus (100M tokens).  C4p: the first million documents of the PubMed-shaped
    workload (short documents, 90M tokens, V=141K), fitted with its K=5,000.  C5p: the first 820,000 documents of
    the ClueWeb12-subset-shaped workload (long, heavy-tailed documents, 300M tokens), fitted with its K=10,000:
    the library cuts it into four document chunks by itself (Sec. 3.1.2), as it cuts the full workload into 85."""
    if name not in _CORPORA:
        _CORPORA.clear()                       # one large corpus in memory at a time
        t = time.time()
        spec = {"C3": corpusgen.SPECS["C3"], "C4p": corpusgen.scaled(corpusgen.SPECS["C4"], 1_000_000),
                "C5p": corpusgen.scaled(corpusgen.SPECS["C5"], 820_000)}[name]
        c = corpusgen.generate(spec, with_topics=False)
        say("[fullsize] corpus %s T=%d generated in %.1fs" % (spec.name, c.T, time.time() - t))
        if name == "C3":
            assert c.T == 100_000_000 and c.spec.D == 300_000 and c.spec.V == 100_000
        _CORPORA[name] = c
    return _CORPORA[name]


@pytest.mark.parametrize("name,K", [("C4p", 5000), ("C5p", 10000), ("C3", 1000), ("C3", 10000)])
def test_full_size_parity(name, K):
    import paper_1610_02496_amd as pk
    c = corpus_for(name)
    s = c.spec
    alpha, beta, seed = 50.0 / K, s.beta, s.seed
    t = time.time()
    g = pk.Saber(c.doc_ptr, c.word_ids, s.V, K, alpha, beta, seed)       # default options = bench configuration
    say("[fullsize] %s K=%d gpu init %.1fs, %d chunks" % (name, K, time.time() - t, g.get_stats()["chunks"])); t = time.time()
    if name == "C5p":
        assert g.get_stats()["chunks"] >= 3 and g.get_stats()["stream_workers"] == 0   # the automatic, resident layout
    o = oracle.Model(c.doc_ptr, c.word_ids, s.V, K, alpha, beta, seed)
    say("[fullsize] K=%d oracle init + M-step %.1fs" % (K, time.time() - t)); t = time.time()

    # ---- iteration 0: assignment and counts, in full ----
    assert np.array_equal(g.get_z(), o.z)
    cd_ptr, topic, count, _, ck = g.counts(want_cwk=False)
    o_ptr, o_topic, o_count = o.cd
    assert np.array_equal(cd_ptr, o_ptr) and np.array_equal(topic, o_topic) and np.array_equal(count, o_count)
    assert np.array_equal(ck, o.ck) and int(ck.sum()) == c.T
    del cd_ptr, topic, count
    if K <= 1000:
        cwk = g.counts(want_cd=False, want_ck=False)[3]
        assert np.array_equal(cwk, o.cwk)
        del cwk
    rng = np.random.default_rng(K)
    words = np.unique(np.r_[0, 1, s.V - 1, rng.integers(0, s.V, 100)]).astype(np.int32)
    phi, prefix = g.get_phi(words)
    assert np.array_equal(phi, o.phi[words])
    ref = o.c32[words]; diff = prefix != ref
    assert diff.mean() < 1e-5
    assert np.all(np.abs(prefix[diff].astype(np.float64) - ref[diff]) <= np.spacing(ref[diff]).astype(np.float64))
    say("[fullsize] K=%d iteration-0 state equal (%.1fs)" % (K, time.time() - t)); t = time.time()

    # ---- one E-step from the identical state: a sample of tokens, one by one ----
    tok = np.sort(rng.choice(c.T, N_SAMPLE, replace=False)).astype(np.int64)
    # add every token of three documents, the longest one included
    lens = np.diff(c.doc_ptr)
    for d in (int(lens.argmax()), 17, s.D - 1):
        tok = np.r_[tok, np.arange(c.doc_ptr[d], c.doc_ptr[d + 1])]
    tok = np.unique(tok)
    S, Q, p = g.token_probs(tok)
    z_ref, S_ref, p_ref, br, margin = o.sample_tokens(tok)
    assert np.allclose(S, S_ref, rtol=1e-5, atol=0)
    assert np.allclose(p, p_ref, rtol=1e-5, atol=0)
    assert np.allclose(Q, np.float64(np.float32(alpha)) * o.sum64[c.word_ids[tok]], rtol=1e-5, atol=0)
    g.iterate(1)
    z = g.get_z()
    bad = np.nonzero(z[tok] != z_ref)[0]
    say("[fullsize] K=%d E-step: %d of %d sampled tokens differ; dense-branch share %.3f (%.1fs)"
        % (K, bad.size, tok.size, (br == 2).mean(), time.time() - t)); t = time.time()
    assert bad.size <= 1e-3 * tok.size
    assert np.all(margin[bad] < 1e-5)
    assert (br == 1).any() and (br == 2).any()

    # ---- invariants after the iteration, at full size ----
    assert z.min() >= 0 and z.max() < K
    cd_ptr, topic, count, _, ck = g.counts(want_cwk=False)
    assert int(count.sum()) == c.T and int(ck.sum()) == c.T
    assert np.array_equal(np.bincount(z, minlength=K), ck)
    rows = np.repeat(np.arange(s.D), np.diff(cd_ptr))
    assert np.array_equal(np.bincount(rows, weights=count, minlength=s.D).astype(np.int64), lens)
    inner = np.ones(topic.size, dtype=bool); inner[cd_ptr[:-1][np.diff(cd_ptr) > 0]] = False
    assert np.all(np.diff(topic)[inner[1:]] > 0)                     # ascending topics inside every row
    # A is bit-exact given the same z: the oracle's CountByDZ on the GPU's assignment
    o_ptr, o_topic, o_count = oracle.count_by_dz(c.doc_ptr, z, K)
    assert np.array_equal(cd_ptr, o_ptr) and np.array_equal(topic, o_topic) and np.array_equal(count, o_count)
    st = g.get_stats()
    assert st["sum_tokens"] == c.T and st["nnz_cd"] == o_ptr[-1]
    ll = g.loglik()
    assert np.isfinite(ll) and -12.0 < ll < -3.0
    say("[fullsize] K=%d invariants and A after iteration 1 ok, loglik %.4f (%.1fs)" % (K, ll, time.time() - t))
    g.close(); o.close()
    if name == "C5p":
        # the same corpus with its token lists streamed from pinned host memory (the billion-token workload's
        # configuration: three workers, chunks as the library cuts them): assignments equal bit for bit
        t = time.time()
        g = pk.Saber(c.doc_ptr, c.word_ids, s.V, K, alpha, beta, seed, stream_workers=3)
        assert g.get_stats()["chunks"] >= 3 and g.get_stats()["stream_workers"] == 3
        g.iterate(1)
        assert np.array_equal(g.get_z(), z)
        assert g.loglik() == ll
        say("[fullsize] %s host streaming, 3 workers: z and log-likelihood equal to the resident path (%.1fs)" % (name, time.time() - t))
        g.close()


def test_full_size_streaming_and_variants_equal_default():
    """At the benchmark's size: host streaming (the configuration bench.py times: 3 workers, 2 chunks; and others) and the two
    ablation variants give the assignments of the default path bit for bit, which the test above holds against the
    oracle; the chains are compared after two iterations."""
    import paper_1610_02496_amd as pk
    c = corpus_for("C3")
    s = c.spec
    K = 10000
    args = (c.doc_ptr, c.word_ids, s.V, K, 50.0 / K, s.beta, s.seed)
    g = pk.Saber(*args)
    g.iterate(2)
    z_ref, ll_ref = g.get_z(), g.loglik()
    ck_ref = g.counts(want_cd=False, want_cwk=False)[4]
    g.close()
    for label, opts in [("streaming 3x2", {"stream_workers": 3, "n_chunks": 2}), ("streaming 3x4", {"stream_workers": 3, "n_chunks": 4}),
                        ("streaming 2x7", {"stream_workers": 2, "n_chunks": 7}),
                        ("A by sorting", {"ablation": 2}), ("document order", {"ablation": 1})]:
        t = time.time()
        g = pk.Saber(*args, **opts)
        g.iterate(2)
        z = g.get_z()
        assert np.array_equal(z, z_ref), label
        assert np.array_equal(g.counts(want_cd=False, want_cwk=False)[4], ck_ref), label
        assert abs(g.loglik() - ll_ref) <= 1e-9 * abs(ll_ref), label
        say("[fullsize] %s: z, topic totals and log-likelihood equal to the default path (%.1fs)" % (label, time.time() - t))
        g.close()
