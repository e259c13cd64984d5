"""saber_set_hooks: device memory from the caller's allocator and kernels on the caller's stream (PyTorch's caching
allocator and a torch stream), called through the C ABI.  Results must not depend on where the memory comes from."""
import numpy as np
import pytest

import corpusgen
import oracle

pytestmark = pytest.mark.gpu


def run(pk, c, K, **opts):
    g = pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, K, 0.3, 0.01, 77, **opts)
    z0 = g.get_z()
    g.iterate(3)
    out = (z0, g.get_z(), g.counts(), g.loglik(), g.get_stream())
    return g, out


@pytest.mark.parametrize("opts", [{}, {"n_chunks": 3, "stream_workers": 2}])
def test_torch_allocator_and_stream_give_the_same_results(opts):
    import torch
    import paper_1610_02496_amd as pk
    c = corpusgen.tiny(61, 400, 900, 25, 70.0)
    K = 300
    g, ref = run(pk, c, K, **opts)
    g.close()
    stream = torch.cuda.Stream()
    # dirty the cache first: the library must not rely on fresh (zeroed) memory
    junk = torch.full((64 << 20,), 0x7F, dtype=torch.uint8, device="cuda")
    del junk
    before = torch.cuda.memory_allocated()
    pk.set_torch_hooks(stream)
    try:
        g, got = run(pk, c, K, **opts)
        held = torch.cuda.memory_allocated() - before
        assert held > c.T * 8, "the context's device arrays did not come from torch's allocator (%d bytes)" % held
        assert got[4] == stream.cuda_stream, "kernels are not on the caller's stream"
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
        for a, b in zip(got[2], ref[2]):
            assert np.array_equal(a, b)
        assert got[3] == ref[3]                       # the reduction order is fixed: bit-identical
        # and against the oracle from the same state
        o = oracle.Model(c.doc_ptr, c.word_ids, c.spec.V, K, 0.3, 0.01, 77)
        o.set_z(got[1], it=3)
        assert abs(got[3] - o.loglik()) <= 1e-6 * abs(o.loglik())
        S, Q, p = g.token_probs(np.arange(c.T, dtype=np.int64))
        _, S_ref, p_ref, _, _ = o.estep_detail(nthreads=4)
        assert np.allclose(S, S_ref, rtol=1e-5, atol=0) and np.allclose(p, p_ref, rtol=1e-5, atol=0)
        g.close()
        assert torch.cuda.memory_allocated() == before, "saber_free did not hand the memory back"
    finally:
        pk.clear_hooks()
    # back on hipMalloc and a stream of the library's own
    g, again = run(pk, c, K, **opts)
    assert again[4] != stream.cuda_stream and np.array_equal(again[1], ref[1])
    g.close()


def test_hooks_must_come_in_pairs():
    import ctypes
    import paper_1610_02496_amd as pk
    L = pk.load_library()
    cb = pk.binding.ALLOC_FN(lambda n: None)
    assert L.saber_set_hooks(ctypes.cast(cb, ctypes.c_void_p), None, None) == pk.binding.SABER_EINVAL
    assert b"together" in L.saber_last_error()
    pk.clear_hooks()


def test_allocator_failure_is_reported():
    import paper_1610_02496_amd as pk
    c = corpusgen.tiny(62, 30, 60, 5, 20.0)
    calls = []

    def alloc(n):
        calls.append(n)
        return None

    pk.set_hooks(alloc, lambda p: None, 0)
    try:
        with pytest.raises(pk.SaberError) as e:
            pk.Saber(c.doc_ptr, c.word_ids, c.spec.V, 16, 0.3, 0.01, 1)
        assert e.value.code == pk.binding.SABER_ENOMEM and calls
    finally:
        pk.clear_hooks()
