"""ctypes binding of the C ABI in ``include/saber.h``: argument marshalling only.

Every step of the path runs in the HIP kernels of ``libsaber.so``.  There is no
CPU fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

SABER_OK, SABER_EINVAL, SABER_ENOMEM, SABER_EDEVICE, SABER_ESTATE, SABER_ERANGE = 0, -1, -2, -3, -4, -5
_STATUS = {0: "SABER_OK", -1: "SABER_EINVAL", -2: "SABER_ENOMEM", -3: "SABER_EDEVICE", -4: "SABER_ESTATE",
           -5: "SABER_ERANGE"}

# every symbol include/saber.h declares
EXPORTS = ["saber_set_hooks", "saber_options_default", "saber_init_ex", "saber_init", "saber_iterate", "saber_counts_nnz",
           "saber_counts", "saber_loglik", "saber_loglik_static", "saber_holdout_loglik", "saber_free", "saber_last_error", "saber_get_z", "saber_set_z",
           "saber_get_iteration", "saber_token_probs", "saber_get_phi", "saber_get_stats", "saber_reset_stats",
           "saber_get_stream", "saber_bandwidth_probe", "saber_alias_build_probe", "saber_get_alias"]


class SaberError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("%s: %s" % (_STATUS.get(code, str(code)), msg))
        self.code = code


class Options(ctypes.Structure):
    _fields_ = [("n_chunks", ctypes.c_int32), ("block_threads", ctypes.c_int32), ("tile_tokens", ctypes.c_int32),
                ("stage_phi", ctypes.c_int32), ("profile", ctypes.c_int32), ("long_doc_tokens", ctypes.c_int32),
                ("dz_lds_entries", ctypes.c_int32), ("stage_min_tokens", ctypes.c_int32),
                ("light_block_threads", ctypes.c_int32), ("light_word_tokens", ctypes.c_int32),
                ("stream_workers", ctypes.c_int32), ("ablation", ctypes.c_int32), ("device_mem_limit_mb", ctypes.c_int32),
                ("quarter_row_entries", ctypes.c_int32), ("half_row_entries", ctypes.c_int32), ("reserved", ctypes.c_int32 * 1)]


class Stats(ctypes.Structure):
    _fields_ = [("iterations", ctypes.c_int64), ("ms_sample", ctypes.c_double), ("ms_count_dz", ctypes.c_double),
                ("ms_ck", ctypes.c_double), ("ms_phi", ctypes.c_double), ("ms_total", ctypes.c_double),
                ("sample_launches", ctypes.c_int64), ("sum_tokens", ctypes.c_int64),
                ("sum_tokens_dense", ctypes.c_int64), ("sum_row_entries", ctypes.c_int64),
                ("nnz_cd", ctypes.c_int64), ("next_row_entries", ctypes.c_int64), ("tokens", ctypes.c_int64),
                ("words_present", ctypes.c_int64), ("tiles", ctypes.c_int64), ("sum_row_fetch", ctypes.c_int64),
                ("next_row_fetch", ctypes.c_int64), ("light_words_present", ctypes.c_int64),
                ("light_tokens", ctypes.c_int64), ("sum_light_entries", ctypes.c_int64),
                ("next_light_entries", ctypes.c_int64), ("stream_workers", ctypes.c_int64), ("chunks", ctypes.c_int64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_ if n != "reserved"}


_lib = None


def library_path() -> str:
    return _build.LIB


def load_library():
    """Load libsaber.so (building it first only if it does not exist) and declare the signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    L = ctypes.CDLL(_build.LIB)
    vp, i32, i64, u32, u64, f32 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32,
                                   ctypes.c_uint64, ctypes.c_float)
    sig = {
        "saber_set_hooks": (ctypes.c_int, [vp, vp, vp]),
        "saber_options_default": (None, [vp]),
        "saber_init_ex": (ctypes.c_int, [vp, vp, vp, i64, i32, i32, f32, f32, u64, vp]),
        "saber_init": (ctypes.c_int, [vp, vp, vp, i64, i32, i32, f32, f32, u64]),
        "saber_iterate": (ctypes.c_int, [vp, i32]),
        "saber_counts_nnz": (ctypes.c_int, [vp, vp]),
        "saber_counts": (ctypes.c_int, [vp, vp, vp, vp, vp, vp]),
        "saber_loglik": (ctypes.c_int, [vp, vp]),
        "saber_loglik_static": (ctypes.c_int, [vp, vp]),
        "saber_holdout_loglik": (ctypes.c_int, [vp, vp, vp, vp, i64, i32, u64, vp, vp, vp, vp]),
        "saber_free": (None, [vp]),
        "saber_last_error": (ctypes.c_char_p, []),
        "saber_get_z": (ctypes.c_int, [vp, vp]),
        "saber_set_z": (ctypes.c_int, [vp, vp, u32]),
        "saber_get_iteration": (ctypes.c_int, [vp, vp]),
        "saber_token_probs": (ctypes.c_int, [vp, vp, i64, vp, vp, vp]),
        "saber_get_phi": (ctypes.c_int, [vp, vp, i32, vp, vp]),
        "saber_get_stats": (ctypes.c_int, [vp, vp]),
        "saber_reset_stats": (ctypes.c_int, [vp]),
        "saber_get_stream": (ctypes.c_int, [vp, vp]),
        "saber_bandwidth_probe": (ctypes.c_int, [i64, i32, vp]),
        "saber_alias_build_probe": (ctypes.c_int, [vp, vp, i32, vp, vp, vp, vp]),
        "saber_get_alias": (ctypes.c_int, [vp, vp, i32, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def _check(rc):
    if rc != SABER_OK:
        raise SaberError(rc, load_library().saber_last_error().decode("utf-8", "replace"))


def _ptr(a):
    return None if a is None else a.ctypes.data


ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t)
DEALLOC_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p)
_hook_refs = None   # the callbacks in force: ctypes function objects must outlive their use by the library


def set_hooks(alloc=None, dealloc=None, hip_stream=0):
    """saber_set_hooks: ``alloc(bytes) -> device address`` / ``dealloc(address)`` (Python callables or None for
    hipMalloc / hipFree) and the hipStream_t (an integer; 0: every context creates its own) used by contexts created
    from now on."""
    global _hook_refs
    a = ALLOC_FN(alloc) if alloc is not None else None
    d = DEALLOC_FN(dealloc) if dealloc is not None else None
    _check(load_library().saber_set_hooks(ctypes.cast(a, ctypes.c_void_p) if a else None,
                                          ctypes.cast(d, ctypes.c_void_p) if d else None,
                                          ctypes.c_void_p(int(hip_stream)) if hip_stream else None))
    _hook_refs = (_hook_refs or []) + [(a, d)]   # earlier contexts may still hold earlier callbacks


def set_torch_hooks(stream=None):
    """Device memory from PyTorch's caching allocator and kernels on a torch stream (default: the current one).
    PyTorch serves as plumbing only: it hands out device memory and the stream."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    dev = torch.cuda.current_device()

    def alloc(nbytes):
        try:
            return torch.cuda.caching_allocator_alloc(int(nbytes), dev, st)
        except Exception:   # out of memory: the library reports SABER_ENOMEM
            return None

    def dealloc(ptr):
        torch.cuda.caching_allocator_delete(ptr)

    set_hooks(alloc, dealloc, st.cuda_stream)


def clear_hooks():
    """Back to hipMalloc / hipFree and a library-owned stream per context."""
    set_hooks(None, None, 0)


def options_default() -> Options:
    o = Options()
    load_library().saber_options_default(ctypes.addressof(o))
    return o


def bandwidth_probe(nbytes=1 << 30, reps=10) -> float:
    """Read+write GB/s of a plain device-to-device copy kernel."""
    v = ctypes.c_double()
    _check(load_library().saber_bandwidth_probe(int(nbytes), int(reps), ctypes.addressof(v)))
    return v.value


class Saber:
    """One sampler context.  Method names follow the C ABI (saber_init -> constructor)."""

    def __init__(self, doc_ptr, word_ids, V, K, alpha, beta, seed, **opts):
        L = load_library()
        self._doc_ptr = np.ascontiguousarray(doc_ptr, dtype=np.int64)
        self._word_ids = np.ascontiguousarray(word_ids, dtype=np.int32)
        self.D = int(self._doc_ptr.size - 1); self.V = int(V); self.K = int(K)
        self.T = int(self._doc_ptr[-1]) if self._doc_ptr.size else 0
        o = options_default()
        for k, v in opts.items():
            if not hasattr(o, k):
                raise TypeError("unknown option %r" % k)
            setattr(o, k, int(v))
        h = ctypes.c_void_p()
        self._h = None
        _check(L.saber_init_ex(ctypes.addressof(h), _ptr(self._doc_ptr), _ptr(self._word_ids), self.D, self.V, self.K,
                               np.float32(alpha), np.float32(beta), int(seed), ctypes.addressof(o)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            load_library().saber_free(self._h); self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def iterate(self, n=1):
        _check(load_library().saber_iterate(self._h, int(n)))

    def counts_nnz(self) -> int:
        n = ctypes.c_int64()
        _check(load_library().saber_counts_nnz(self._h, ctypes.addressof(n)))
        return n.value

    def counts(self, want_cd=True, want_cwk=True, want_ck=True):
        """Returns (cd_row_ptr, cd_topic, cd_count, cwk[V,K], ck[K]); skipped parts are None."""
        cd_ptr = topic = count = cwk = ck = None
        if want_cd:
            nnz = self.counts_nnz()
            cd_ptr = np.zeros(self.D + 1, dtype=np.int64)
            topic = np.zeros(nnz, dtype=np.int32); count = np.zeros(nnz, dtype=np.int32)
        if want_cwk:
            cwk = np.zeros((self.V, self.K), dtype=np.int32)
        if want_ck:
            ck = np.zeros(self.K, dtype=np.int64)
        _check(load_library().saber_counts(self._h, _ptr(cd_ptr), _ptr(topic), _ptr(count), _ptr(cwk), _ptr(ck)))
        return cd_ptr, topic, count, cwk, ck

    def loglik(self) -> float:
        v = ctypes.c_double()
        _check(load_library().saber_loglik(self._h, ctypes.addressof(v)))
        return v.value

    def loglik_static(self) -> float:
        """saber_loglik_static: the same number through the entry point that allocates nothing; the result lands in
        device memory of the caller (a torch tensor here) and is read back."""
        import torch
        out = torch.zeros(1, dtype=torch.float64, device="cuda")
        _check(load_library().saber_loglik_static(self._h, ctypes.c_void_p(out.data_ptr())))
        return float(out.cpu()[0])

    def holdout_loglik(self, doc_ptr, word_ids, observed, n_foldin, seed, z_init=None):
        """Document-completion log-likelihood of held-out documents; returns (ll per scored token, scored tokens,
        final assignments of the observed tokens)."""
        doc_ptr = np.ascontiguousarray(doc_ptr, dtype=np.int64)
        word_ids = np.ascontiguousarray(word_ids, dtype=np.int32)
        observed = np.ascontiguousarray(observed, dtype=np.uint8)
        if observed.size != word_ids.size or word_ids.size != int(doc_ptr[-1]):
            raise ValueError("doc_ptr, word_ids and observed do not describe the same token list")
        n_obs = int(np.count_nonzero(observed))
        if z_init is not None:
            z_init = np.ascontiguousarray(z_init, dtype=np.int32)
            if z_init.size != n_obs:
                raise ValueError("z_init must hold one assignment per observed token")
        z_out = np.zeros(max(n_obs, 1), dtype=np.int32)
        ll = ctypes.c_double(); scored = ctypes.c_int64()
        _check(load_library().saber_holdout_loglik(self._h, _ptr(doc_ptr), _ptr(word_ids), _ptr(observed),
                                                   doc_ptr.size - 1, n_foldin, seed,
                                                   None if z_init is None else _ptr(z_init), _ptr(z_out),
                                                   ctypes.addressof(ll), ctypes.addressof(scored)))
        return ll.value, scored.value, z_out[:n_obs]

    def alias_build_probe(self, words=()):
        """Builds alias tables for all dense rows; returns (ms, rows built, prob[m][K], alias[m][K]) for `words`."""
        words = np.ascontiguousarray(words, dtype=np.int32)
        m = int(words.size)
        prob = np.zeros((max(m, 1), self.K), dtype=np.float32)
        alias = np.zeros((max(m, 1), self.K), dtype=np.int32)
        ms = ctypes.c_double(); rows = ctypes.c_int32()
        _check(load_library().saber_alias_build_probe(self._h, _ptr(words) if m else None, m, _ptr(prob), _ptr(alias),
                                                      ctypes.addressof(ms), ctypes.addressof(rows)))
        return ms.value, rows.value, prob[:m], alias[:m]

    def get_alias(self, words):
        """Alias tables (prob[m][K], alias[m][K]) of the listed words; needs ablation bit 2."""
        words = np.ascontiguousarray(words, dtype=np.int32)
        prob = np.zeros((words.size, self.K), dtype=np.float32); alias = np.zeros((words.size, self.K), dtype=np.int32)
        _check(load_library().saber_get_alias(self._h, _ptr(words), words.size, _ptr(prob), _ptr(alias)))
        return prob, alias

    def get_z(self):
        z = np.zeros(self.T, dtype=np.int32)
        _check(load_library().saber_get_z(self._h, _ptr(z)))
        return z

    def set_z(self, z, iteration=0):
        z = np.ascontiguousarray(z, dtype=np.int32)
        if z.size != self.T:
            raise ValueError("z must hold T values")
        _check(load_library().saber_set_z(self._h, _ptr(z), int(iteration)))

    def get_iteration(self) -> int:
        v = ctypes.c_uint32()
        _check(load_library().saber_get_iteration(self._h, ctypes.addressof(v)))
        return v.value

    def token_probs(self, tok):
        tok = np.ascontiguousarray(tok, dtype=np.int64)
        S = np.zeros(tok.size, dtype=np.float32); Q = np.zeros_like(S); p = np.zeros_like(S)
        _check(load_library().saber_token_probs(self._h, _ptr(tok), tok.size, _ptr(S), _ptr(Q), _ptr(p)))
        return S, Q, p

    def get_phi(self, words):
        words = np.ascontiguousarray(words, dtype=np.int32)
        phi = np.zeros((words.size, self.K), dtype=np.float32); prefix = np.zeros_like(phi)
        _check(load_library().saber_get_phi(self._h, _ptr(words), words.size, _ptr(phi), _ptr(prefix)))
        return phi, prefix

    def get_stats(self) -> dict:
        s = Stats()
        _check(load_library().saber_get_stats(self._h, ctypes.addressof(s)))
        return s.as_dict()

    def reset_stats(self):
        _check(load_library().saber_reset_stats(self._h))

    def get_stream(self) -> int:
        v = ctypes.c_void_p()
        _check(load_library().saber_get_stream(self._h, ctypes.addressof(v)))
        return v.value or 0
