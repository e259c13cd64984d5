"""ctypes front end of the CPU oracle (``saber_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The GPU package never imports this module and
this module never imports the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "saber_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

c_void_p, c_i32, c_i64, c_u32, c_u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint64
c_f32, c_f64, c_int = ctypes.c_float, ctypes.c_double, ctypes.c_int


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (about a second).  Without ``force`` the library is rebuilt only when it is
    missing or older than the C source, so that an edited oracle is never judged through a stale binary."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class Detail(ctypes.Structure):
    _fields_ = [("S", c_f64), ("Q", c_f64), ("p_sparse", c_f64), ("branch", c_i32), ("pad", c_i32),
                ("margin", c_f64)]


def lib():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    sig = {
        "orc_philox4x32_10": (None, [c_void_p, c_void_p, c_void_p]),
        "orc_token_uniforms": (None, [c_u64, c_u64, c_u32, c_void_p, c_void_p]),
        "orc_init_z": (None, [c_i64, c_i32, c_u64, c_void_p]),
        "orc_count_by_dz": (c_int, [c_i64, c_void_p, c_void_p, c_i32, c_void_p, c_void_p, c_void_p]),
        "orc_count_by_vz": (None, [c_i64, c_void_p, c_void_p, c_i32, c_i32, c_void_p, c_void_p]),
        "orc_preprocess": (c_int, [c_void_p, c_void_p, c_i32, c_i32, c_f32, c_void_p]),
        "orc_build_prefix": (None, [c_void_p, c_i32, c_i32, c_void_p, c_void_p]),
        "orc_wary_build": (c_int, [c_void_p, c_i32, c_i32, c_void_p, c_i64, c_void_p, c_void_p, c_int]),
        "orc_wary_query": (c_i32, [c_void_p, c_void_p, c_void_p, c_int, c_i32, c_f32]),
        "orc_position_in_prefix32": (c_i32, [c_void_p, c_i32, c_f32]),
        "orc_sample": (c_i32, [c_i32, c_void_p, c_void_p, c_void_p, c_void_p, c_i32, c_f64, c_f64, c_f64, c_void_p]),
        "orc_estep": (None, [c_i64, c_void_p, c_void_p, c_i32, c_f32, c_void_p, c_void_p, c_void_p, c_void_p,
                             c_void_p, c_void_p, c_u64, c_u32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int]),
        "orc_alias_build": (None, [c_void_p, c_i32, c_void_p, c_void_p]),
        "orc_alias_draw": (c_i32, [c_void_p, c_void_p, c_i32, c_u32, c_void_p]),
        "orc_estep_alias": (None, [c_i64, c_void_p, c_void_p, c_i32, c_f32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                   c_void_p, c_void_p, c_u64, c_u32, c_void_p, c_void_p, c_void_p, c_int]),
        "orc_loglik": (c_f64, [c_i64, c_void_p, c_void_p, c_i32, c_f32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
        "orc_model_create": (c_void_p, [c_void_p, c_void_p, c_i64, c_i32, c_i32, c_f32, c_f32, c_u64]),
        "orc_model_free": (None, [c_void_p]),
        "orc_model_set_z": (c_int, [c_void_p, c_void_p, c_u32]),
        "orc_model_iterate": (c_int, [c_void_p, c_i32, c_int]),
        "orc_model_estep_detail": (None, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int]),
        "orc_model_sample_tokens": (None, [c_void_p, c_void_p, c_i64, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
        "orc_model_loglik": (c_f64, [c_void_p]),
        "orc_model_iter": (c_u32, [c_void_p]),
        "orc_holdout_loglik": (c_int, [c_void_p, c_i64, c_void_p, c_void_p, c_void_p, c_i32, c_u64, c_void_p, c_int,
                                       c_void_p, c_void_p, c_void_p]),
    }
    for name in ("z", "cd_ptr", "cd_topic", "cd_count", "cwk", "ck", "phi", "c32", "sum64"):
        sig["orc_model_" + name] = (c_void_p, [c_void_p])
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def _p(a):
    return None if a is None else a.ctypes.data


def _view(ptr, shape, dtype):
    n = int(np.prod(shape))
    if n == 0:
        return np.zeros(shape, dtype=dtype)
    buf = (ctypes.c_char * (n * np.dtype(dtype).itemsize)).from_address(ptr)
    return np.frombuffer(buf, dtype=dtype).reshape(shape)


# ----------------------------------------------------------------------------- primitives
def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32); k = np.asarray(key, dtype=np.uint32); out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def token_uniforms(seed, t, it):
    u0, u1 = c_f64(), c_f64()
    lib().orc_token_uniforms(seed, t, it, ctypes.addressof(u0), ctypes.addressof(u1))
    return u0.value, u1.value


def init_z(T, K, seed):
    z = np.empty(T, dtype=np.int32)
    lib().orc_init_z(T, K, seed, _p(z))
    return z


def count_by_dz(doc_ptr, z, K):
    doc_ptr = np.ascontiguousarray(doc_ptr, dtype=np.int64); z = np.ascontiguousarray(z, dtype=np.int32)
    D = doc_ptr.size - 1; T = int(doc_ptr[-1])
    cd_ptr = np.zeros(D + 1, dtype=np.int64); topic = np.zeros(max(T, 1), dtype=np.int32); count = np.zeros(max(T, 1), dtype=np.int32)
    rc = lib().orc_count_by_dz(D, _p(doc_ptr), _p(z), K, _p(cd_ptr), _p(topic), _p(count))
    if rc:
        raise ValueError("orc_count_by_dz: %d" % rc)
    n = int(cd_ptr[-1])
    return cd_ptr, topic[:n].copy(), count[:n].copy()


def count_by_vz(word_ids, z, V, K):
    word_ids = np.ascontiguousarray(word_ids, dtype=np.int32); z = np.ascontiguousarray(z, dtype=np.int32)
    cwk = np.zeros((V, K), dtype=np.int32); ck = np.zeros(K, dtype=np.int64)
    lib().orc_count_by_vz(word_ids.size, _p(word_ids), _p(z), V, K, _p(cwk), _p(ck))
    return cwk, ck


def preprocess(cwk, ck, beta):
    cwk = np.ascontiguousarray(cwk, dtype=np.int32); ck = np.ascontiguousarray(ck, dtype=np.int64)
    V, K = cwk.shape
    phi = np.empty((V, K), dtype=np.float32)
    rc = lib().orc_preprocess(_p(cwk), _p(ck), V, K, np.float32(beta), _p(phi))
    assert rc == 0
    return phi


def build_prefix(phi):
    phi = np.ascontiguousarray(phi, dtype=np.float32)
    V, K = phi.shape
    c32 = np.empty((V, K), dtype=np.float32); sum64 = np.empty(V, dtype=np.float64)
    lib().orc_build_prefix(_p(phi), V, K, _p(c32), _p(sum64))
    return c32, sum64


class WaryTree:
    """Generic W-ary tree over a non-decreasing array (Sec. 3.2.4)."""

    def __init__(self, bottom, W):
        bottom = np.ascontiguousarray(bottom, dtype=np.float32)
        self.W = W
        cap = 2 * bottom.size + 64
        self.tree = np.zeros(cap, dtype=np.float32)
        self.off = np.zeros(40, dtype=np.int64); self.len = np.zeros(40, dtype=np.int32)
        self.levels = lib().orc_wary_build(_p(bottom), bottom.size, W, _p(self.tree), cap, _p(self.off), _p(self.len), 40)
        if self.levels < 1:
            raise ValueError("orc_wary_build failed")

    def level(self, l):
        return self.tree[self.off[l]: self.off[l] + self.len[l]]

    def query(self, x):
        return lib().orc_wary_query(_p(self.tree), _p(self.off), _p(self.len), self.levels, self.W, np.float32(x))


def position_in_prefix32(c, x):
    c = np.ascontiguousarray(c, dtype=np.float32)
    return lib().orc_position_in_prefix32(_p(c), c.size, np.float32(x))


def sample(topic, count, phi_w, c32_w, Q, u0, u1):
    """Alg. 2 for one token. Returns (k, Detail)."""
    topic = np.ascontiguousarray(topic, dtype=np.int32); count = np.ascontiguousarray(count, dtype=np.int32)
    phi_w = np.ascontiguousarray(phi_w, dtype=np.float32); c32_w = np.ascontiguousarray(c32_w, dtype=np.float32)
    det = Detail()
    k = lib().orc_sample(topic.size, _p(topic), _p(count), _p(phi_w), _p(c32_w), phi_w.size, Q, u0, u1,
                         ctypes.addressof(det))
    return k, det


def alias_build(p):
    """Alias table (Walker's method, sweep construction) of one weight vector: (prob float32[K], alias int32[K])."""
    p = np.ascontiguousarray(p, dtype=np.float32)
    prob = np.empty(p.size, dtype=np.float32); alias = np.empty(p.size, dtype=np.int32)
    lib().orc_alias_build(_p(p), p.size, _p(prob), _p(alias))
    return prob, alias


def alias_draw(prob, alias, bits24):
    """Walker's draw for the uniform bits24 * 2^-24; returns (item, margin)."""
    prob = np.ascontiguousarray(prob, dtype=np.float32); alias = np.ascontiguousarray(alias, dtype=np.int32)
    m = c_f64()
    k = lib().orc_alias_draw(_p(prob), _p(alias), prob.size, int(bits24), ctypes.addressof(m))
    return k, m.value


def alias_mass(prob, alias):
    """The distribution a table encodes: (prob[k] + sum of (1 - prob[b]) over buckets b whose alias is k) / K."""
    prob = np.asarray(prob, dtype=np.float64)
    mass = prob.copy()
    np.add.at(mass, np.asarray(alias), 1.0 - prob)
    return mass / prob.size


# ----------------------------------------------------------------------------- whole model
class Model:
    """Alg. 1 as a stateful object: iteration 0 = Philox-initialised z and a first M-step."""

    def __init__(self, doc_ptr, word_ids, V, K, alpha, beta, seed):
        self.doc_ptr = np.ascontiguousarray(doc_ptr, dtype=np.int64)
        self.word_ids = np.ascontiguousarray(word_ids, dtype=np.int32)
        self.D = self.doc_ptr.size - 1; self.T = int(self.doc_ptr[-1]); self.V = V; self.K = K
        self.alpha = float(np.float32(alpha)); self.beta = float(np.float32(beta)); self.seed = seed
        self._h = lib().orc_model_create(_p(self.doc_ptr), _p(self.word_ids), self.D, V, K,
                                         np.float32(alpha), np.float32(beta), seed)
        if not self._h:
            raise MemoryError("orc_model_create failed")

    def close(self):
        if self._h:
            lib().orc_model_free(self._h); self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def iterate(self, n=1, nthreads=1):
        rc = lib().orc_model_iterate(self._h, n, nthreads)
        if rc:
            raise RuntimeError("orc_model_iterate: %d" % rc)

    def set_z(self, z, it=0):
        z = np.ascontiguousarray(z, dtype=np.int32); assert z.size == self.T
        rc = lib().orc_model_set_z(self._h, _p(z), it)
        if rc:
            raise ValueError("orc_model_set_z: %d" % rc)

    def estep_detail(self, nthreads=1):
        """One E-step from the current state (iteration iter+1) without changing it."""
        T = self.T
        z = np.empty(T, dtype=np.int32); S = np.empty(T); p = np.empty(T)
        br = np.empty(T, dtype=np.int8); mg = np.empty(T)
        lib().orc_model_estep_detail(self._h, _p(z), _p(S), _p(p), _p(br), _p(mg), nthreads)
        return z, S, p, br, mg

    def sample_tokens(self, tok):
        """Alg. 2 for the listed tokens only (iteration iter+1), from the current state."""
        tok = np.ascontiguousarray(tok, dtype=np.int64); n = tok.size
        z = np.empty(n, dtype=np.int32); S = np.empty(n); p = np.empty(n); br = np.empty(n, dtype=np.int8); mg = np.empty(n)
        lib().orc_model_sample_tokens(self._h, _p(tok), n, _p(z), _p(S), _p(p), _p(br), _p(mg))
        return z, S, p, br, mg

    def loglik(self):
        return lib().orc_model_loglik(self._h)

    def alias_tables(self):
        """Alias tables of all V rows of the current Bhat: (prob float32[V,K], alias int32[V,K])."""
        phi = self.phi
        prob = np.empty((self.V, self.K), dtype=np.float32); alias = np.empty((self.V, self.K), dtype=np.int32)
        for v in range(self.V):
            lib().orc_alias_build(phi[v].ctypes.data, self.K, prob[v].ctypes.data, alias[v].ctypes.data)
        return prob, alias

    def estep_alias(self, prob, alias, nthreads=1):
        """One E-step from the current state (iteration iter+1) with the dense term drawn from the given alias tables;
        the state is not changed.  Returns (z, branch, margin)."""
        prob = np.ascontiguousarray(prob, dtype=np.float32); alias = np.ascontiguousarray(alias, dtype=np.int32)
        assert prob.shape == (self.V, self.K) and alias.shape == (self.V, self.K)
        z = np.empty(self.T, dtype=np.int32); br = np.empty(self.T, dtype=np.int8); mg = np.empty(self.T)
        cd_ptr, cd_topic, cd_count = self.cd
        cd_topic = np.ascontiguousarray(cd_topic); cd_count = np.ascontiguousarray(cd_count)
        lib().orc_estep_alias(self.D, _p(self.doc_ptr), _p(self.word_ids), self.K, np.float32(self.alpha), _p(cd_ptr),
                              _p(cd_topic), _p(cd_count), _p(self.phi), _p(self.sum64), _p(prob), _p(alias),
                              self.seed, self.iter + 1, _p(z), _p(br), _p(mg), nthreads)
        return z, br, mg

    def holdout_loglik(self, doc_ptr, word_ids, observed, n_fold, seed, z_init=None, nthreads=1):
        """Document-completion log-likelihood of held-out documents under this model's frozen Bhat: fold in the
        observed tokens for ``n_fold`` iterations, score the others.  Returns (ll per scored token, scored tokens,
        final assignments of the observed tokens)."""
        doc_ptr = np.ascontiguousarray(doc_ptr, dtype=np.int64)
        word_ids = np.ascontiguousarray(word_ids, dtype=np.int32)
        observed = np.ascontiguousarray(observed, dtype=np.uint8)
        assert observed.size == word_ids.size == int(doc_ptr[-1])
        n_obs = int(np.count_nonzero(observed))
        if z_init is not None:
            z_init = np.ascontiguousarray(z_init, dtype=np.int32); assert z_init.size == n_obs
        z_out = np.empty(max(n_obs, 1), dtype=np.int32)
        ll = c_f64(); scored = c_i64()
        rc = lib().orc_holdout_loglik(self._h, doc_ptr.size - 1, _p(doc_ptr), _p(word_ids), _p(observed), n_fold, seed,
                                      _p(z_init), nthreads, ctypes.addressof(ll), ctypes.addressof(scored), _p(z_out))
        if rc:
            raise ValueError("orc_holdout_loglik: %d" % rc)
        return ll.value, scored.value, z_out[:n_obs]

    @property
    def iter(self):
        return lib().orc_model_iter(self._h)

    @property
    def z(self):
        return _view(lib().orc_model_z(self._h), (self.T,), np.int32)

    @property
    def cd(self):
        cd_ptr = _view(lib().orc_model_cd_ptr(self._h), (self.D + 1,), np.int64)
        n = int(cd_ptr[-1])
        return cd_ptr, _view(lib().orc_model_cd_topic(self._h), (max(self.T, 1),), np.int32)[:n], \
            _view(lib().orc_model_cd_count(self._h), (max(self.T, 1),), np.int32)[:n]

    @property
    def cwk(self):
        return _view(lib().orc_model_cwk(self._h), (self.V, self.K), np.int32)

    @property
    def ck(self):
        return _view(lib().orc_model_ck(self._h), (self.K,), np.int64)

    @property
    def phi(self):
        return _view(lib().orc_model_phi(self._h), (self.V, self.K), np.float32)

    @property
    def c32(self):
        return _view(lib().orc_model_c32(self._h), (self.V, self.K), np.float32)

    @property
    def sum64(self):
        return _view(lib().orc_model_sum64(self._h), (self.V,), np.float64)
