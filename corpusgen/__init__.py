"""Seeded synthetic LDA corpora (inputs for tests and benchmarks only).

The corpora stand in for the datasets of Table 3 (NYTimes, PubMed, a ClueWeb12
subset): same D, V, T and T/D, drawn from the LDA generative process with
planted topics.  Nothing here belongs to the sampler: the module only produces
``doc_ptr`` (int64, D+1), ``word_ids`` (int32, T, doc-major) and the planted
topic of every token.  The CPU oracle and the GPU path both read these arrays;
neither imports the other.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lda_corpus.c")
_LIB = os.path.join(_HERE, "libldacorpus.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the generator with gcc (about a second).  Without ``force`` the library is rebuilt only when it is
    missing or older than the C source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.lda_corpus_lengths.restype = ctypes.c_int64
        lib.lda_corpus_lengths.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int, ctypes.c_double,
                                           ctypes.c_double, ctypes.c_int64, ctypes.c_void_p]
        lib.lda_corpus_fill.restype = ctypes.c_int
        lib.lda_corpus_fill.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        _lib = lib
    return _lib


@dataclass(frozen=True)
class CorpusSpec:
    """Recipe of one synthetic corpus plus the sampler settings it is fitted with."""
    name: str
    D: int
    V: int
    T: int                 # target token count (exact for lognormal lengths, approximate for Poisson)
    length_kind: str       # "poisson" | "lognormal"
    length_mean: float
    length_sigma: float    # sigma of log-length (lognormal only)
    K_true: int            # planted topics
    zipf_s: float
    topic_conc: float      # mean per-word Dirichlet concentration of a planted topic
    doc_conc: float        # symmetric Dirichlet concentration of document mixtures
    K: int                 # fitted topics
    iters: int
    seed: int
    beta: float = 0.01

    @property
    def alpha(self) -> float:
        return 50.0 / self.K


# The five workloads of the benchmark definition; "C2"/"C3" share one corpus.
SPECS = {
    "C1": CorpusSpec("C1", 1_000, 5_000, 100_000, "poisson", 100.0, 0.0, 100, 1.1, 0.01, 0.1, 100, 10, 0),
    "C2": CorpusSpec("C2", 300_000, 100_000, 100_000_000, "lognormal", 330.0, 0.8, 1_000, 1.07, 0.01, 0.05, 1_000, 50, 1),
    "C3": CorpusSpec("C3", 300_000, 100_000, 100_000_000, "lognormal", 330.0, 0.8, 1_000, 1.07, 0.01, 0.05, 10_000, 50, 1),
    "C4": CorpusSpec("C4", 8_200_000, 141_000, 738_000_000, "lognormal", 90.0, 0.6, 2_000, 1.05, 0.01, 0.05, 5_000, 20, 2),
    "C5": CorpusSpec("C5", 19_400_000, 100_000, 7_100_000_000, "lognormal", 366.0, 1.0, 5_000, 1.05, 0.01, 0.03, 10_000, 10, 3),
}


def scaled(spec: CorpusSpec, docs: int) -> CorpusSpec:
    """The same per-document shape on a document prefix of ``docs`` documents."""
    docs = min(docs, spec.D)
    T = int(round(spec.T * docs / spec.D))
    return replace(spec, name=f"{spec.name}[:{docs}]", D=docs, T=T)


@dataclass
class Corpus:
    spec: CorpusSpec
    doc_ptr: np.ndarray     # int64 [D+1]
    word_ids: np.ndarray    # int32 [T]
    true_topic: np.ndarray  # int32 [T]

    @property
    def T(self) -> int:
        return int(self.doc_ptr[-1])


def generate(spec: CorpusSpec, nthreads: int | None = None, with_topics: bool = True) -> Corpus:
    lib = _load()
    if nthreads is None:
        nthreads = max(1, min(16, os.cpu_count() or 1))
    doc_ptr = np.zeros(spec.D + 1, dtype=np.int64)
    kind = {"poisson": 0, "lognormal": 1}[spec.length_kind]
    T = lib.lda_corpus_lengths(spec.seed, spec.D, kind, spec.length_mean, spec.length_sigma, spec.T,
                               doc_ptr.ctypes.data)
    if T < 0:
        raise RuntimeError("lda_corpus_lengths failed: %d" % T)
    word_ids = np.empty(T, dtype=np.int32)
    true_topic = np.empty(T if with_topics else 0, dtype=np.int32)
    rc = lib.lda_corpus_fill(spec.seed, spec.D, spec.V, spec.K_true, spec.zipf_s, spec.topic_conc,
                             spec.doc_conc, doc_ptr.ctypes.data, word_ids.ctypes.data,
                             true_topic.ctypes.data if with_topics else None, nthreads)
    if rc != 0:
        raise RuntimeError("lda_corpus_fill failed: %d" % rc)
    return Corpus(spec, doc_ptr, word_ids, true_topic)


def tiny(seed: int, D: int, V: int, K_true: int, mean_len: float, K: int | None = None) -> Corpus:
    """A small corpus for unit tests (Poisson lengths; may contain empty documents)."""
    spec = CorpusSpec(f"tiny{seed}", D, V, int(D * mean_len), "poisson", mean_len, 0.0, K_true, 1.1, 0.05, 0.2,
                      K if K is not None else K_true, 1, seed)
    return generate(spec, nthreads=2)
