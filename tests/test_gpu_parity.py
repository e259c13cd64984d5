"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars (from the benchmark spec of tolerances):
  * counts (A, B, C_k) bit-exact given the same assignments z;
  * Bhat bit-exact (each operation of Eq. 2 is one binary32 rounding on both sides);
  * prefix tables equal except for isolated entries one binary32 ulp apart (both sides round a
    binary64 running sum to binary32; the summation order differs);
  * S, Q, p_sparse within 1e-5 relative;
  * one E-step from identical z: >= 99.9 % of tokens agree, and every disagreement has a uniform draw
    within 1e-5 of a decision boundary (the oracle reports that distance as ``margin``);
  * per-token log-likelihood within 1e-4 relative after 10 free-running iterations.
"""
import numpy as np
import pytest

import corpusgen
import oracle

pytestmark = pytest.mark.gpu


def saber():
    import paper_1610_02496_amd as pk
    return pk


def make_pair(c, K, alpha, beta, seed, **opts):
    pk = saber()
    g = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, beta, seed, **opts)
    o = oracle.Model(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, beta, seed)
    return g, o


def assert_counts_equal(g, o, words=None):
    cd_ptr, topic, count, cwk, ck = g.counts()
    o_ptr, o_topic, o_count = o.cd
    assert np.array_equal(cd_ptr, o_ptr)
    assert np.array_equal(topic, o_topic)
    assert np.array_equal(count, o_count)
    assert np.array_equal(cwk, o.cwk)
    assert np.array_equal(ck, o.ck)
    assert g.counts_nnz() == o_ptr[-1]


def assert_phi_equal(g, o, nwords=64, seed=0):
    V = o.V
    words = np.unique(np.r_[0, V - 1, np.random.default_rng(seed).integers(0, V, min(nwords, V))]).astype(np.int32)
    phi, prefix = g.get_phi(words)
    assert np.array_equal(phi, o.phi[words])                       # bit-exact
    ref = o.c32[words]
    diff = prefix != ref
    if diff.any():
        assert diff.mean() < 1e-5
        assert np.all(np.abs(prefix[diff].astype(np.float64) - ref[diff]) <= np.spacing(ref[diff]).astype(np.float64))


def assert_estep_parity(g, o, min_agree=0.999):
    """Both sides hold the same z and iteration counter; advance the GPU one iteration and compare."""
    assert g.get_iteration() == o.iter
    tok = np.arange(o.T, dtype=np.int64)
    if o.T:
        S, Q, p = g.token_probs(tok)
    z_ref, S_ref, p_ref, br, margin = o.estep_detail(nthreads=4)
    if o.T:
        w = o.word_ids
        Q_ref = np.float64(np.float32(o.alpha)) * o.sum64[w]
        assert np.allclose(S, S_ref, rtol=1e-5, atol=0)
        assert np.allclose(Q, Q_ref, rtol=1e-5, atol=0)
        assert np.allclose(p, p_ref, rtol=1e-5, atol=0)
    g.iterate(1)
    z = g.get_z()
    bad = np.nonzero(z != z_ref)[0]
    if o.T:
        assert 1.0 - bad.size / o.T >= min_agree, "only %.5f of tokens agree" % (1.0 - bad.size / o.T)
    assert np.all(margin[bad] < 1e-5), "disagreement away from any boundary: tokens %s" % bad[margin[bad] >= 1e-5][:10]
    # counts are bit-exact given the same z: hand the GPU's z to the oracle's M-step
    o.set_z(z, it=g.get_iteration())
    assert_counts_equal(g, o)
    assert_phi_equal(g, o)
    return bad.size


# ------------------------------------------------------------------------------------------- init
def test_init_state_matches_oracle():
    c = corpusgen.tiny(21, 300, 700, 20, 60.0)
    g, o = make_pair(c, 50, 1.0, 0.01, 1234)
    assert np.array_equal(g.get_z(), o.z)                           # Philox init, bit-exact
    assert_counts_equal(g, o)
    assert_phi_equal(g, o, nwords=700)
    assert abs(g.loglik() - o.loglik()) < 1e-6 * abs(o.loglik())
    st = g.get_stats()
    assert st["nnz_cd"] == o.cd[0][-1] and st["tokens"] == c.T
    lens = np.diff(c.doc_ptr)
    assert st["next_row_entries"] == int((np.diff(o.cd[0]) * lens).sum())
    # what the sampler has to fetch: a row once per (word, document) pair, i.e. K_d times the distinct words of d
    U = np.array([np.unique(c.word_ids[a:b]).size for a, b in zip(c.doc_ptr[:-1], c.doc_ptr[1:])])
    assert st["next_row_fetch"] == int((np.diff(o.cd[0]) * U).sum())
    # words with fewer than K/2 tokens keep their row of B sparse
    n_v = np.bincount(c.word_ids, minlength=c.spec.V)
    light = n_v < 50 // 2
    assert st["light_tokens"] == int(n_v[light].sum()) and st["light_words_present"] == int((n_v[light] > 0).sum())
    assert st["next_light_entries"] == int(np.count_nonzero(o.cwk[light]))


def test_philox_seed_and_64bit_seed():
    c = corpusgen.tiny(22, 50, 100, 5, 30.0)
    seed = (0xABCDEF12 << 32) | 0x13572468
    g, o = make_pair(c, 33, 0.5, 0.01, seed)
    assert np.array_equal(g.get_z(), o.z)
    assert_estep_parity(g, o)


# ------------------------------------------------------------------------------------------- one E-step
@pytest.mark.parametrize("K,opts", [
    (100, {}),                                   # config-1 shape: K < 128, two tree levels
    (64, {}), (65, {}), (1, {}), (2, {}),        # edges of the 64-wide tiles
    (1000, {"n_chunks": 3, "tile_tokens": 100}), # several chunks, heavy words split into many tiles
    (1000, {"stage_phi": 0}),                    # Bhat gathered from global memory instead of LDS
    (5000, {"block_threads": 512}),              # three tree levels (K > 4096)
    (5000, {"block_threads": 64, "tile_tokens": 64}),
    (1000, {"light_word_tokens": -1}),           # every word keeps a dense row of B
    (1000, {"light_word_tokens": 1 << 20}),      # every word keeps a sparse row of B
    (1000, {"light_word_tokens": 40, "n_chunks": 3, "tile_tokens": 16, "long_doc_tokens": 16, "dz_lds_entries": 8}),
    (130, {"light_word_tokens": 1 << 20}),
    (20000, {}),                                 # Bhat row of 80 KB in LDS: two workgroups per CU
    (37000, {"light_word_tokens": 300}),         # 148 KB: one workgroup per CU; above that the row stays in global memory
    (40000, {}),                                 # not staged
])
def test_one_estep_from_random_state(K, opts):
    c = corpusgen.tiny(30 + K % 7, 400, 900, 25, 70.0)
    g, o = make_pair(c, K, 50.0 / K, 0.01, 99, **opts)
    assert_estep_parity(g, o)
    assert_estep_parity(g, o)                    # a second step from the state the GPU produced


def test_one_estep_from_planted_state():
    """Sparse, converged-like rows: z set to the planted topics of the generator."""
    c = corpusgen.tiny(41, 500, 1200, 40, 90.0)
    g, o = make_pair(c, 40, 0.1, 0.01, 5)
    g.set_z(c.true_topic, 7); o.set_z(c.true_topic, 7)
    assert_counts_equal(g, o)
    assert_estep_parity(g, o)


def test_wide_topic_ids_use_int32_z():
    """K > 65536: assignments are stored as int32 and Bhat is gathered from global memory."""
    c = corpusgen.tiny(43, 120, 40, 6, 50.0)
    g, o = make_pair(c, 70000, 0.01, 0.01, 8)
    assert_estep_parity(g, o)


def test_largest_topic_count():
    c = corpusgen.tiny(44, 60, 12, 4, 40.0)
    g, o = make_pair(c, 262144, 0.01, 0.01, 3)
    assert_estep_parity(g, o)


def test_long_documents_and_global_row_fallback():
    """Documents above the long-document threshold, and rows larger than the LDS row buffer."""
    spec = corpusgen.CorpusSpec("long", 12, 300, 12 * 3000, "poisson", 3000.0, 0.0, 30, 1.1, 0.05, 0.5, 2000, 1, 9)
    c = corpusgen.generate(spec, nthreads=2)
    g, o = make_pair(c, 2000, 0.05, 0.01, 17, long_doc_tokens=256, dz_lds_entries=128)
    assert np.diff(o.cd[0]).max() > 128
    assert_counts_equal(g, o)
    assert_estep_parity(g, o)


def test_mixed_row_lengths_in_one_tile():
    """Lognormal lengths from a few tokens to a few thousand: rows of at most 128 entries (taken two at a time),
    rows that fill one 256-entry block and rows of several blocks meet inside the same tiles."""
    spec = corpusgen.CorpusSpec("mixed", 400, 600, 400 * 300, "lognormal", 300.0, 1.2, 30, 1.1, 0.05, 0.5, 3000, 1, 13)
    c = corpusgen.generate(spec, nthreads=2)
    g, o = make_pair(c, 3000, 50.0 / 3000, 0.01, 23)
    kd = np.diff(o.cd[0])
    assert (kd <= 128).sum() > 20 and ((kd > 128) & (kd <= 256)).sum() > 20 and (kd > 256).sum() > 20
    assert_estep_parity(g, o)
    assert_estep_parity(g, o)


@pytest.mark.parametrize("V", [3, 40, 900])
def test_short_rows_share_a_wavefront(V):
    """Rows of at most 64 entries are sampled four at a time (one per 16 lanes), rows of at most 128 entries two at
    a time, longer ones with all 64 lanes.  Documents of 1 to 700 tokens over a vocabulary of V words: with V = 3
    a (word, document) run holds up to a few hundred tokens, far more than the 16 or 32 a group of lanes collects in
    one piece; with V = 900 nearly every run is a single token.  Every way of dividing the rows among the three
    layouts must give the assignments of the plain one-run-per-wavefront layout, which is held against the oracle."""
    rng = np.random.default_rng(V)
    lens = np.r_[rng.integers(1, 60, 150), rng.integers(60, 130, 150), rng.integers(130, 260, 60), rng.integers(260, 700, 25)]
    rng.shuffle(lens)
    doc_ptr = np.r_[0, np.cumsum(lens)].astype(np.int64)
    word_ids = np.minimum((V * rng.random(int(doc_ptr[-1])) ** 1.5).astype(np.int32), V - 1)
    K, alpha, beta, seed = 2000, 0.02, 0.01, 5
    pk = saber()
    g = pk.Saber(doc_ptr, word_ids, V, K, alpha, beta, seed, quarter_row_entries=-1, half_row_entries=-1)
    o = oracle.Model(doc_ptr, word_ids, V, K, alpha, beta, seed)
    kd = np.diff(o.cd[0])
    assert (kd <= 64).sum() > 50 and ((kd > 64) & (kd <= 128)).sum() > 50 and (kd > 128).sum() > 50
    assert_estep_parity(g, o)
    assert_estep_parity(g, o)
    z_ref, ll_ref = g.get_z(), g.loglik()
    S_ref = g.token_probs(np.arange(o.T, dtype=np.int64))[0]
    g.close()
    for opts in [{}, {"half_row_entries": -1}, {"quarter_row_entries": -1}, {"quarter_row_entries": 20, "half_row_entries": 70},
                 {"quarter_row_entries": 64, "half_row_entries": 64}, {"tile_tokens": 64}, {"n_chunks": 3, "stream_workers": 2},
                 {"block_threads": 64, "light_word_tokens": -1}]:
        g = pk.Saber(doc_ptr, word_ids, V, K, alpha, beta, seed, **opts)
        g.iterate(2)
        assert np.array_equal(g.get_z(), z_ref), opts
        if set(opts) <= {"quarter_row_entries", "half_row_entries"}:
            assert g.loglik() == ll_ref, opts                                      # same sums in the same order
        else:
            assert abs(g.loglik() - ll_ref) <= 1e-12 * abs(ll_ref), opts           # tiles and chunks regroup the sum
        assert np.array_equal(g.token_probs(np.arange(o.T, dtype=np.int64))[0], S_ref), opts
        g.close()
    o.close()


def test_large_counts_in_a_row():
    """Few topics and documents of 6,000 to 30,000 tokens: single entries of A with counts of many thousands next
    to ordinary rows (16/16 packing is used up to its limit of 65,535 tokens per document)."""
    rng = np.random.default_rng(5)
    lens = np.r_[rng.integers(6000, 30000, 6), rng.integers(50, 300, 40)]
    doc_ptr = np.r_[0, np.cumsum(lens)].astype(np.int64)
    word_ids = rng.integers(0, 50, int(doc_ptr[-1])).astype(np.int32)
    pk = saber()
    for K in (3, 8):
        g = pk.Saber(doc_ptr, word_ids, 50, K, 0.5, 0.01, 9)
        o = oracle.Model(doc_ptr, word_ids, 50, K, 0.5, 0.01, 9)
        assert o.cd[2].max() > 2048 and (o.cd[2] <= 2048).any()
        assert_counts_equal(g, o)
        assert_estep_parity(g, o)
        assert_estep_parity(g, o)
        assert abs(g.loglik() - o.loglik()) <= 1e-6 * abs(o.loglik())
        g.close(); o.close()


def test_document_longer_than_16_bit_counts():
    """A document of 65,536 tokens or more no longer fits 16-bit counts: entries of A are then packed with just
    enough topic bits for K and the rest for the count, and the kernels take the shifts at run time.  K = 50 keeps
    every word dense, K = 1000 makes about half of the words light (sparse rows of B with the same packing)."""
    rng = np.random.default_rng(6)
    lens = np.r_[70000, rng.integers(40, 400, 30), 66000, rng.integers(40, 400, 30)]
    doc_ptr = np.r_[0, np.cumsum(lens)].astype(np.int64)
    word_ids = rng.integers(0, 300, int(doc_ptr[-1])).astype(np.int32)
    word_ids[:70000] = rng.integers(0, 12, 70000)          # the long document leans on a few words: large counts
    pk = saber()
    for K in (50, 1000):
        g = pk.Saber(doc_ptr, word_ids, 300, K, 0.5, 0.01, 4)
        o = oracle.Model(doc_ptr, word_ids, 300, K, 0.5, 0.01, 4)
        assert (g.get_stats()["light_words_present"] > 0) == (K == 1000)
        assert_counts_equal(g, o)
        assert_estep_parity(g, o)
        # concentrate the long documents on two topics: single counts above 65,535 would not fit 16 bits
        z = o.z.copy(); z[:70000] = np.where(np.arange(70000) % 16 == 0, 1, 0)
        g.set_z(z, 1); o.set_z(z, 1)
        assert o.cd[2].max() > 65535
        assert_counts_equal(g, o)
        assert_estep_parity(g, o)
        assert abs(g.loglik() - o.loglik()) <= 1e-6 * abs(o.loglik())
        g.close(); o.close()


def test_empty_documents_and_single_tokens():
    doc_ptr = np.array([0, 0, 1, 1, 4, 4, 4, 9, 9], dtype=np.int64)
    word_ids = np.array([3, 0, 0, 2, 1, 1, 1, 3, 0], dtype=np.int32)
    pk = saber()
    g = pk.Saber(doc_ptr, word_ids, 5, 7, 0.3, 0.01, 11)
    o = oracle.Model(doc_ptr, word_ids, 5, 7, 0.3, 0.01, 11)
    assert np.array_equal(g.get_z(), o.z)
    assert_counts_equal(g, o)
    for _ in range(3):
        assert_estep_parity(g, o, min_agree=0.0)


@pytest.mark.parametrize("K", [7, 300, 70000])
def test_short_segments_counted_in_registers(K):
    """Segments of at most 64 and of 65 to 128 assignments are sorted and counted in a wavefront's registers, longer
    ones with the LDS bitmap: documents and (light) words on both sides of each limit, with planted assignments that
    make every key different (rows of 64 and 128 entries), all keys equal, and two keys alternating; K = 70,000 takes
    the 32-bit assignments.  CountByDZ and CountByVZ (Alg. 1, Sec. 3.3) must equal the oracle's bit for bit."""
    lens = [1, 2, 3, 63, 64, 65, 66, 127, 128, 129, 130, 200, 64, 128, 64, 128, 64, 128, 100, 0, 5]
    doc_ptr = np.r_[0, np.cumsum(lens)].astype(np.int64)
    T = int(doc_ptr[-1])
    rng = np.random.default_rng(K)
    V = 40
    # word lengths (segments of z_wm) hit the same limits: words 0..5 get 64, 65, 128, 129, 1, 2 tokens
    want = [64, 65, 128, 129, 1, 2]
    word_ids = rng.integers(len(want), V, T).astype(np.int32)
    free = rng.permutation(T)
    at = 0
    for w, n in enumerate(want):
        word_ids[free[at:at + n]] = w; at += n
    pk = saber()
    g = pk.Saber(doc_ptr, word_ids, V, K, 0.2, 0.01, 3)
    o = oracle.Model(doc_ptr, word_ids, V, K, 0.2, 0.01, 3)
    assert np.array_equal(g.get_z(), o.z)
    assert_counts_equal(g, o)
    z = rng.integers(0, K, T).astype(np.int32)
    for d, kind in ((12, "distinct"), (13, "distinct"), (14, "equal"), (15, "equal"), (16, "two"), (17, "two"), (11, "distinct")):
        b, e = int(doc_ptr[d]), int(doc_ptr[d + 1])
        if kind == "distinct" and K >= e - b:
            z[b:e] = rng.permutation(K)[: e - b]
        elif kind == "equal":
            z[b:e] = K - 1
        elif kind == "two":
            z[b:e] = np.where(np.arange(e - b) % 2 == 0, K - 1, 0)
    g.set_z(z, 1); o.set_z(z, 1)
    if K >= 200:
        assert np.diff(o.cd[0])[[12, 13]].tolist() == [64, 128]
    assert_counts_equal(g, o)
    for _ in range(2):
        assert_estep_parity(g, o, min_agree=0.0)
    g.close(); o.close()


def test_empty_corpus():
    pk = saber()
    g = pk.Saber(np.zeros(4, dtype=np.int64), np.zeros(0, dtype=np.int32), 3, 4, 0.1, 0.01, 1)
    g.iterate(2)
    cd_ptr, topic, count, cwk, ck = g.counts()
    assert not cd_ptr.any() and topic.size == 0 and not cwk.any() and not ck.any()
    assert g.loglik() == 0.0
    g0 = pk.Saber(np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), 3, 4, 0.1, 0.01, 1)
    g0.iterate(1)


# ------------------------------------------------------------------------------------------- whole runs
def test_config1_ten_iterations_loglik():
    """Config 1 (D=1000, V=5000, K=100, ~100K tokens): free-running chains, LL within 1e-4 relative."""
    c = corpusgen.generate(corpusgen.SPECS["C1"], nthreads=4)
    s = c.spec
    g, o = make_pair(c, s.K, s.alpha, s.beta, s.seed)
    ll = []
    for it in range(10):
        g.iterate(1); o.iterate(1, nthreads=4)
        ll.append((g.loglik(), o.loglik()))
    assert abs(ll[-1][0] - ll[-1][1]) <= 1e-4 * abs(ll[-1][1])
    assert ll[-1][0] > ll[0][0]
    # the two chains separate only where a draw sat on a decision boundary, but every such flip perturbs
    # its document's row and the chains then drift apart: z itself is compared one E-step at a time
    assert (g.get_z() == o.z).mean() > 0.5
    # the same check with the oracle re-seeded from the GPU's z: exact same state, LL to rounding
    o.set_z(g.get_z(), it=g.get_iteration())
    assert abs(g.loglik() - o.loglik()) <= 1e-6 * abs(o.loglik())
    assert_counts_equal(g, o)
    assert_estep_parity(g, o)


def test_results_do_not_depend_on_layout_options():
    c = corpusgen.tiny(51, 300, 500, 15, 80.0)
    pk = saber()
    ref = None
    for opts in [{}, {"n_chunks": 4}, {"tile_tokens": 64, "block_threads": 128}, {"stage_phi": 0},
                 {"long_doc_tokens": 16, "dz_lds_entries": 8}, {"stage_min_tokens": 65, "light_block_threads": 128},
                 {"stage_min_tokens": 100000}, {"light_word_tokens": -1}, {"light_word_tokens": 1 << 20},
                 {"light_word_tokens": 30, "n_chunks": 2}, {"quarter_row_entries": -1}, {"half_row_entries": 40},
                 {"quarter_row_entries": 10, "half_row_entries": -1}]:
        g = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, 300, 0.2, 0.01, 77, **opts)
        g.iterate(3)
        z = g.get_z()
        if ref is None:
            ref = z
        assert np.array_equal(z, ref), opts


@pytest.mark.parametrize("K", [300, 70000])
def test_host_streaming_matches_oracle_and_resident_path(K):
    """Token arrays kept in pinned host memory and streamed chunk by chunk (Sec. 3.1.2), with 1, 2 and 3 buffers in
    flight and more chunks than buffers: same parity with the oracle, and z, counts and log-likelihood identical
    to the resident path at every step; set_z and get_z go through the host copy."""
    c = corpusgen.tiny(53, 300, 500, 15, 80.0) if K == 300 else corpusgen.tiny(54, 120, 60, 6, 50.0)
    pk = saber()
    alpha = 0.2 if K == 300 else 0.01
    ref = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 77)
    z0 = ref.get_z()
    ref.iterate(3)
    z3, ll3 = ref.get_z(), ref.loglik()
    held = corpusgen.tiny(55, 40, c.spec.V, 15, 60.0)          # held-out documents over the same vocabulary
    observed = (np.arange(held.T) % 2 == 0).astype(np.uint8)
    hold3 = ref.holdout_loglik(held.doc_ptr, held.word_ids, observed, 3, 5)
    for workers, chunks in [(1, 1), (1, 4), (2, 5), (3, 7), (8, 3)]:
        g = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 77, stream_workers=workers, n_chunks=chunks)
        o = oracle.Model(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 77)
        assert np.array_equal(g.get_z(), z0), (workers, chunks)
        assert_counts_equal(g, o)
        assert_estep_parity(g, o)
        g.set_z(z0, 0)
        g.iterate(3)
        assert np.array_equal(g.get_z(), z3), (workers, chunks)
        # per-tile sums added in a fixed order: the same bits for the same chunking, rounding apart otherwise
        assert g.loglik() == ll3 if chunks == 1 else abs(g.loglik() - ll3) <= 1e-12 * abs(ll3)
        o.set_z(z3, 3)
        assert_counts_equal(g, o)
        # held-out documents are scored on the model only: same model, same bits
        h = g.holdout_loglik(held.doc_ptr, held.word_ids, observed, 3, 5)
        assert h[0] == hold3[0] and h[1] == hold3[1] and np.array_equal(h[2], hold3[2])
        g.close(); o.close()
    with pytest.raises(pk.SaberError):
        pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 77, stream_workers=9)


@pytest.mark.parametrize("ablation", [1, 2, 3])
def test_ablation_variants_match_oracle_and_default_path(ablation):
    """The measurement variants of Sec. 4.2's decomposition (bit 0: tokens sampled in document order, bit 1: A rebuilt
    by sorting all (document, topic) pairs) compute what the regular kernels compute: oracle parity step by step,
    and z bit-identical to the default path after several iterations.  Rows of one, two and more 256-entry blocks,
    empty documents, both widths of z."""
    pk = saber()
    spec = corpusgen.CorpusSpec("mixed", 300, 600, 300 * 300, "lognormal", 300.0, 1.2, 30, 1.1, 0.05, 0.5, 3000, 1, 14)
    cases = [(corpusgen.tiny(56, 300, 500, 15, 80.0), 300, 0.2),
             (corpusgen.generate(spec, nthreads=2), 3000, 50.0 / 3000),
             (corpusgen.tiny(57, 120, 60, 6, 50.0), 70000, 0.01)]
    for c, K, alpha in cases:
        ref = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 21, light_word_tokens=-1)
        ref.iterate(3)
        g, o = make_pair(c, K, alpha, 0.01, 21, ablation=ablation)
        assert_counts_equal(g, o)
        assert_estep_parity(g, o)
        assert_estep_parity(g, o)
        g2 = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 21, ablation=ablation)
        g2.iterate(3)
        assert np.array_equal(g2.get_z(), ref.get_z()), (K, ablation)
        assert g2.get_stats()["sum_tokens_dense"] == ref.get_stats()["sum_tokens_dense"]
        for x in (ref, g, g2): x.close()
        o.close()
    dp = np.array([0, 0, 1, 1, 4, 4, 4, 9, 9], dtype=np.int64)
    w = np.array([3, 0, 0, 2, 1, 1, 1, 3, 0], dtype=np.int32)
    g = pk.Saber(dp, w, 5, 7, 0.3, 0.01, 11, ablation=ablation)
    o = oracle.Model(dp, w, 5, 7, 0.3, 0.01, 11)
    assert_counts_equal(g, o)
    for _ in range(3):
        assert_estep_parity(g, o, min_agree=0.0)
    with pytest.raises(pk.SaberError):
        pk.Saber(dp, w, 5, 7, 0.3, 0.01, 11, ablation=ablation, stream_workers=2)


@pytest.mark.parametrize("K,ablation", [(300, 4), (64, 4), (1000, 6), (5000, 4)])
def test_alias_variant_matches_the_oracles_alias_mode(K, ablation):
    """The dense term drawn from per-word alias tables (Sec. 3.2.3's alternative to the tree): the tables, built by
    one workgroup per word from prefix sums, against the oracle's sweep construction, and the E-step against the
    oracle's alias mode, which draws from the oracle's own tables.  The sparse branch and every count are those of
    the default path."""
    c = corpusgen.tiny(80 + K % 9, 300, 500, 20, 70.0)
    alpha = 50.0 / K
    g, o = make_pair(c, K, alpha, 0.01, 31, ablation=ablation)
    assert np.array_equal(g.get_z(), o.z)
    assert_counts_equal(g, o)
    words = np.arange(c.spec.V, dtype=np.int32)
    for step in range(2):
        prob_o, alias_o = o.alias_tables()
        prob, alias = g.get_alias(words)
        # the same construction in another order of additions: probabilities within a binary32 ulp, partners equal
        # wherever a bucket hands over a share that matters
        assert np.all(np.abs(prob.astype(np.float64) - prob_o) <= np.spacing(np.maximum(prob_o, np.float32(1e-30))).astype(np.float64))
        assert (prob != prob_o).mean() < 1e-3
        share = 1.0 - prob_o.astype(np.float64) > 1e-6
        assert np.array_equal(alias[share], alias_o[share])
        for v in (0, 1, c.spec.V - 1):
            want = o.phi[v].astype(np.float64) / o.phi[v].astype(np.float64).sum()
            assert np.abs(oracle.alias_mass(prob[v], alias[v]) - want).max() < 1e-7
        tok = np.arange(o.T, dtype=np.int64)
        S, Q, p = g.token_probs(tok)
        _, S_ref, p_ref, _, _ = o.estep_detail(nthreads=4)
        assert np.allclose(S, S_ref, rtol=1e-5, atol=0) and np.allclose(p, p_ref, rtol=1e-5, atol=0)
        z_ref, br, margin = o.estep_alias(prob_o, alias_o, nthreads=4)
        assert (br == 1).any() and (br == 2).any()
        g.iterate(1)
        z = g.get_z()
        bad = np.nonzero(z != z_ref)[0]
        assert bad.size <= 1e-3 * o.T and np.all(margin[bad] < 1e-5)
        o.set_z(z, it=g.get_iteration())
        assert_counts_equal(g, o)
        assert_phi_equal(g, o)
    # the same chain with the tree: other assignments (another map from the uniform draw to the topic) ...
    t = saber().Saber(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 31)
    t.iterate(1)
    o2 = oracle.Model(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 31)
    a = saber().Saber(c.doc_ptr, c.word_ids, c.spec.V, K, alpha, 0.01, 31, ablation=ablation)
    a.iterate(1)
    _, _, _, br_tree, _ = o2.estep_detail(nthreads=4)
    za, zt = a.get_z(), t.get_z()
    assert np.array_equal(za[br_tree == 1], zt[br_tree == 1])        # ... on the dense branch only
    assert (za[br_tree == 2] != zt[br_tree == 2]).any()
    # ... with the same distribution: topic totals of the dense-branch tokens, alias against tree, chi-square on the
    # topics that hold enough of them
    ha = np.bincount(za[br_tree == 2], minlength=K).astype(np.float64); ht = np.bincount(zt[br_tree == 2], minlength=K).astype(np.float64)
    if K <= 300:
        big = (ha + ht) >= 20
        stat = (((ha - ht) ** 2) / (ha + ht))[big].sum()
        from scipy.stats import chi2 as chi2_dist
        assert stat < chi2_dist.ppf(1 - 1e-4, int(big.sum()))


def test_alias_variant_argument_checks():
    pk = saber()
    c = corpusgen.tiny(90, 30, 60, 5, 20.0)
    with pytest.raises(pk.SaberError) as e:
        pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, 50, 0.5, 0.01, 1, ablation=5)
    assert e.value.code == pk.binding.SABER_EINVAL
    with pytest.raises(pk.SaberError) as e:
        pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, 14000, 0.5, 0.01, 1, ablation=4)
    assert e.value.code == pk.binding.SABER_ERANGE
    g = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, 50, 0.5, 0.01, 1)
    with pytest.raises(pk.SaberError) as e:
        g.get_alias([0])
    assert e.value.code == pk.binding.SABER_ESTATE


def test_alias_tables_encode_the_word_distributions():
    """The alias-table build (measurement aid for Sec. 3.2.3): any valid table is accepted, what is checked is the
    distribution it encodes, bucket by bucket in binary64, against the oracle's Bhat rows: p_k = Bhat_vk / sum."""
    pk = saber()
    for c, K in [(corpusgen.tiny(58, 300, 500, 15, 80.0), 300), (corpusgen.tiny(59, 200, 90, 8, 120.0), 3000)]:
        g, o = make_pair(c, K, 50.0 / K, 0.01, 31, light_word_tokens=-1)
        g.iterate(2); o.set_z(g.get_z(), 2)
        words = np.unique(np.r_[0, c.spec.V - 1, np.random.default_rng(1).integers(0, c.spec.V, 24)]).astype(np.int32)
        ms, rows, prob, alias = g.alias_build_probe(words)
        assert rows == c.spec.V and ms > 0.0
        assert prob.min() >= 0.0 and prob.max() <= 1.0 and alias.min() >= 0 and alias.max() < K
        for i, w in enumerate(words):
            phi = o.phi[w].astype(np.float64)
            want = phi / phi.sum()
            got = prob[i].astype(np.float64)
            np.add.at(got, alias[i], 1.0 - prob[i].astype(np.float64))
            assert np.allclose(got / K, want, rtol=1e-5, atol=1e-12), w
        g.close(); o.close()
    # words that keep a sparse row have no dense Bhat row to build from
    c = corpusgen.tiny(58, 300, 500, 15, 80.0)
    g = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, 300, 0.2, 0.01, 31)
    light = int(np.argmin(np.bincount(c.word_ids, minlength=c.spec.V)))
    with pytest.raises(pk.SaberError):
        g.alias_build_probe([light])
    ms, rows, _, _ = g.alias_build_probe([])
    assert rows < c.spec.V


@pytest.mark.parametrize("test_seed", [20240607, 7, 99])
def test_random_shapes_and_options(test_seed):
    """Sixty corpora per seed of random shape (documents of 0 to a few hundred tokens, vocabularies of 1 to 400 words, K from
    2 to 4,000 including values next to multiples of 64 and of 256) under random hyper-parameters and random
    layout options, each checked against the oracle for two E-steps and the counts that follow."""
    rng = np.random.default_rng(test_seed)
    pk = saber()
    k_pool = [2, 3, 5, 63, 64, 65, 100, 255, 256, 257, 300, 511, 512, 513, 1000, 1023, 1025, 2000, 4000]
    for case in range(60):
        D = int(rng.integers(1, 120))
        V = int(rng.choice([1, 2, 7, 50, 400]))
        K = int(rng.choice(k_pool))
        mean_len = float(rng.choice([0.5, 3.0, 40.0, 90.0, 300.0]))
        lens = rng.poisson(mean_len, D) * (rng.random(D) > 0.1)
        if rng.random() < 0.3:
            lens[int(rng.integers(0, D))] += int(rng.integers(600, 3000))      # one long document
        doc_ptr = np.r_[0, np.cumsum(lens)].astype(np.int64)
        T = int(doc_ptr[-1])
        # Zipf-like word choice so that frequent and rare words meet
        w = np.minimum((V * rng.random(T) ** 2.5).astype(np.int32), V - 1)
        alpha = float(rng.choice([0.01, 0.1, 1.0, 50.0 / K]))
        beta = float(rng.choice([0.001, 0.01, 0.5]))
        seed = int(rng.integers(0, 2 ** 63))
        opts = {}
        if rng.random() < 0.5: opts["n_chunks"] = int(rng.integers(1, 6))
        if rng.random() < 0.4: opts["tile_tokens"] = int(rng.choice([64, 100, 1000]))
        if rng.random() < 0.4: opts["block_threads"] = int(rng.choice([64, 128, 256, 512, 1024]))
        if rng.random() < 0.4: opts["light_word_tokens"] = int(rng.choice([-1, 1, 5, 1 << 20]))
        if rng.random() < 0.3: opts["long_doc_tokens"] = int(rng.choice([8, 64]))
        if rng.random() < 0.3: opts["dz_lds_entries"] = int(rng.choice([4, 64]))
        if rng.random() < 0.2: opts["stage_phi"] = 0
        if rng.random() < 0.3: opts["quarter_row_entries"] = int(rng.choice([-1, 4, 30, 64]))
        if rng.random() < 0.3: opts["half_row_entries"] = int(rng.choice([-1, 8, 100, 128]))
        mode = rng.random()
        if mode < 0.25: opts["stream_workers"] = int(rng.integers(1, 5))
        elif mode < 0.45: opts["ablation"] = int(rng.integers(1, 4))
        label = (case, D, V, K, T, alpha, beta, opts)
        g = pk.Saber(doc_ptr, w, V, K, alpha, beta, seed, **opts)
        o = oracle.Model(doc_ptr, w, V, K, alpha, beta, seed)
        try:
            assert np.array_equal(g.get_z(), o.z), label
            assert_counts_equal(g, o)
            for _ in range(2):
                assert_estep_parity(g, o, min_agree=0.999 if T >= 5000 else 0.0)
            # a binary32 S + Q carries a relative error of 1e-6 at most: the same absolute error in its logarithm
            assert abs(g.loglik() - o.loglik()) <= 1e-6 * abs(o.loglik()) + 1e-6, label
        except AssertionError as e:
            raise AssertionError("%s: %s" % (label, e))
        g.close(); o.close()


def test_streaming_is_chosen_when_the_device_memory_does_not_suffice():
    """stream_workers = 0 plans with the free device memory (here: with a stated limit): resident when the estimate
    fits, three streaming buffers when only that fits, an error when neither does; results do not depend on it."""
    rng = np.random.default_rng(3)
    lens = rng.integers(50, 150, 5000)
    doc_ptr = np.r_[0, np.cumsum(lens)].astype(np.int64)
    w = rng.integers(0, 50, int(doc_ptr[-1])).astype(np.int32)
    pk = saber()
    res = pk.Saber(doc_ptr, w, 50, 16, 0.5, 0.01, 8, n_chunks=8, device_mem_limit_mb=1000)
    assert res.get_stats()["stream_workers"] == 0
    auto = pk.Saber(doc_ptr, w, 50, 16, 0.5, 0.01, 8, n_chunks=8, device_mem_limit_mb=40)
    assert auto.get_stats()["stream_workers"] == 3
    never = pk.Saber(doc_ptr, w, 50, 16, 0.5, 0.01, 8, n_chunks=8, device_mem_limit_mb=40, stream_workers=-1)
    assert never.get_stats()["stream_workers"] == 0
    for g in (res, auto, never):
        g.iterate(3)
    assert np.array_equal(res.get_z(), auto.get_z()) and np.array_equal(res.get_z(), never.get_z())
    with pytest.raises(pk.SaberError) as e:
        pk.Saber(doc_ptr, w, 50, 16, 0.5, 0.01, 8, n_chunks=8, device_mem_limit_mb=33)
    assert e.value.code == pk.binding.SABER_ENOMEM and "streamed" in str(e.value)


def test_set_z_roundtrip_and_determinism():
    c = corpusgen.tiny(52, 200, 300, 10, 50.0)
    pk = saber()
    a = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, 128, 0.4, 0.01, 5)
    a.iterate(2)
    b = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, 128, 0.4, 0.01, 5)
    b.set_z(a.get_z(), a.get_iteration())
    a.iterate(2); b.iterate(2)
    assert np.array_equal(a.get_z(), b.get_z()) and a.get_iteration() == 4
    assert a.loglik() == b.loglik()


# ------------------------------------------------------------------------------------------- errors
def test_error_paths():
    pk = saber()
    dp = np.array([0, 2], dtype=np.int64); w = np.array([0, 1], dtype=np.int32)
    for args, code in [((dp, w, 2, 0, 0.1, 0.01, 1), pk.binding.SABER_EINVAL),
                       ((dp, w, 2, 3, 0.0, 0.01, 1), pk.binding.SABER_EINVAL),
                       ((dp, w, 2, 3, 0.1, -1.0, 1), pk.binding.SABER_EINVAL),
                       ((dp, w, 2, 300000, 0.1, 0.01, 1), pk.binding.SABER_ERANGE),
                       ((np.array([0, 2, 1]), w, 2, 3, 0.1, 0.01, 1), pk.binding.SABER_EINVAL),
                       ((np.array([1, 2]), w, 2, 3, 0.1, 0.01, 1), pk.binding.SABER_EINVAL),
                       ((dp, np.array([0, 2], dtype=np.int32), 2, 3, 0.1, 0.01, 1), pk.binding.SABER_EINVAL)]:
        with pytest.raises(pk.SaberError) as e:
            pk.Saber(*args)
        assert e.value.code == code
    g = pk.Saber(dp, w, 2, 3, 0.1, 0.01, 1)
    with pytest.raises(pk.SaberError):
        g.iterate(-1)
    with pytest.raises(pk.SaberError):
        g.set_z(np.array([0, 3]))
    with pytest.raises(pk.SaberError):
        g.token_probs(np.array([2]))
    with pytest.raises(pk.SaberError):
        pk.Saber(dp, w, 2, 3, 0.1, 0.01, 1, block_threads=100)


# ------------------------------------------------------------------------------------------- does it learn
def test_gpu_chain_recovers_planted_topics_and_generalises():
    """The GPU path on its own (free-running, 120 iterations) on data drawn from the LDA process with 10 well
    separated topics: the log-likelihood rises to the level of the planted assignment, the fitted topic-word
    columns match the planted ones, and folding in half of each held-out document predicts the other half much
    better than a uniform mixture does."""
    from scipy.optimize import linear_sum_assignment
    spec = corpusgen.CorpusSpec("rec", 800, 800, 64000, "poisson", 80.0, 0.0, 10, 1.1, 0.02, 0.1, 10, 1, 11)
    full = corpusgen.generate(spec, nthreads=2)
    D_train = 600
    cut = int(full.doc_ptr[D_train])
    dp, w = full.doc_ptr[:D_train + 1], full.word_ids[:cut]
    pk = saber()
    g = pk.Saber(dp, w, spec.V, 10, 0.1, 0.01, 5)
    ll = [g.loglik()]
    for _ in range(4):
        g.iterate(30); ll.append(g.loglik())
    assert all(b > a for a, b in zip(ll, ll[1:]))
    truth = oracle.Model(dp, w, spec.V, 10, 0.1, 0.01, 5)
    truth.set_z(full.true_topic[:cut])
    assert ll[0] < truth.loglik() - 0.4 and abs(ll[-1] - truth.loglik()) < 0.06
    phi, _ = g.get_phi(np.arange(spec.V, dtype=np.int32))
    unit = lambda a: a / np.linalg.norm(a, axis=0, keepdims=True)
    sim = unit(phi.astype(np.float64)).T @ unit(truth.phi.astype(np.float64))
    r, cidx = linear_sum_assignment(-sim)
    assert (sim[r, cidx] > 0.9).sum() >= 8
    # held-out documents of the same planted model
    hp = full.doc_ptr[D_train:] - cut; hw = full.word_ids[cut:]
    pos = np.arange(hw.size) - np.repeat(hp[:-1], np.diff(hp))
    mask = (pos % 2 == 0).astype(np.uint8)
    uniform = g.holdout_loglik(hp, hw, np.zeros_like(mask), 0, 1)[0]
    folded = [g.holdout_loglik(hp, hw, mask, n, 1)[0] for n in (0, 2, 20)]
    assert folded[2] > folded[1] > folded[0] and folded[2] > uniform + 0.3
    assert folded[2] < ll[-1] + 0.3
    g.close(); truth.close()
