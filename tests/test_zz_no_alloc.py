"""saber_loglik_static: the log-likelihood reduction for callers that must not allocate (its work space is a static
device array) against saber_loglik, through the C ABI, on two calls in a row, the second on a smaller corpus."""
import ctypes

import numpy as np
import pytest

import corpusgen

pytestmark = pytest.mark.gpu


def test_static_work_space_matches_the_allocating_entry_point():
    import torch
    import paper_1610_02496_amd as pk
    L = pk.load_library()
    out = torch.full((2,), float("nan"), dtype=torch.float64, device="cuda")
    # first a corpus with several chunks and a few thousand sampling workgroups, then a much smaller one: the second
    # call finds the first call's partial sums in the work space and must not read them
    for seed, docs, V, K, opts in ((71, 600, 1500, 200, {"n_chunks": 3}), (72, 40, 90, 48, {})):
        c = corpusgen.tiny(seed, docs, V, 20, 60.0)
        g = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, K, 0.2, 0.01, seed, **opts)
        g.iterate(2)
        want = g.loglik()
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        rc = L.saber_loglik_static(g._h, ctypes.c_void_p(out.data_ptr()))
        assert rc == 0, L.saber_last_error()
        got = out.cpu().numpy()
        assert got[0] == want, (got[0], want)          # same kernels, same order of additions: bit-identical
        assert np.isnan(got[1])                        # nothing is written past the one result
        assert g.loglik_static() == want
        g.close()


def test_static_work_space_limits_and_empty_corpus():
    import torch
    import paper_1610_02496_amd as pk
    L = pk.load_library()
    out = torch.full((1,), 5.0, dtype=torch.float64, device="cuda")
    g = pk.Saber(np.zeros(3, dtype=np.int64), np.zeros(0, dtype=np.int32), 4, 8, 0.5, 0.01, 1)
    assert L.saber_loglik_static(g._h, ctypes.c_void_p(out.data_ptr())) == 0
    assert float(out.cpu()[0]) == 0.0
    assert L.saber_loglik_static(g._h, None) == pk.binding.SABER_EINVAL
    g.close()
