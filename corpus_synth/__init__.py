"""Seeded synthetic LDA corpora shaped like the paper's workloads.

Input generation only: nothing here knows how a topic is resampled.  Both the
CPU oracle's tests and the GPU library's tests/benchmark draw their inputs from
this module; it imports neither of them.

The five named configurations follow the sizes of the paper's two corpora
(Table 3: a news-article collection with T=99.5M, D=300K, V=102K and a
biomedical-abstract collection with T=738M, D=8.2M, V=141K; mean document
lengths 332 and 92, Section 7.1) plus two small cases and a high-K case.
The collections themselves are not reproduced: only their shapes are used.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "corpus_gen.c")
_LIB = os.path.join(_HERE, "libcorpus_gen.so")

CORPUS_SEED = 1803
SAMPLER_SEED = 4631


@dataclass(frozen=True)
class CorpusConfig:
    name: str
    D: int
    V: int
    K: int
    length_law: str          # "poisson" or "lognormal"
    mean_len: float
    sigma: float             # lognormal log-sd (unused for poisson)
    zipf_s: float
    alpha_gen: float
    beta_gen: float
    iters: int

    @property
    def alpha(self) -> float:        # training hyper-parameters, Section 7: alpha = 50/K
        return 50.0 / self.K

    @property
    def beta(self) -> float:
        return 0.01


CONFIGS = {
    "C1": CorpusConfig("C1", 1_000, 5_000, 32, "poisson", 100.0, 0.0, 1.1, 0.1, 0.01, 10),
    "C2": CorpusConfig("C2", 20_000, 30_000, 128, "poisson", 50.0, 0.0, 1.1, 0.1, 0.01, 50),
    "C3": CorpusConfig("C3", 300_000, 102_000, 1_000, "lognormal", 330.0, 0.5, 1.05, 0.05, 0.01, 100),
    "C4": CorpusConfig("C4", 8_200_000, 141_000, 1_000, "lognormal", 90.0, 0.4, 1.05, 0.05, 0.01, 100),
    "C5": CorpusConfig("C5", 300_000, 102_000, 10_000, "lognormal", 330.0, 0.5, 1.05, 0.05, 0.01, 50),
}


def build(force: bool = False) -> str:
    """Compile the generator with gcc; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, u64, dbl = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_double
        ptr = ctypes.c_void_p
        lib.corpus_doc_lengths.restype = i64
        lib.corpus_doc_lengths.argtypes = [i64, ctypes.c_int, dbl, dbl, u64, ptr]
        lib.corpus_fill.restype = ctypes.c_int
        lib.corpus_fill.argtypes = [i64, ptr, i32, i32, dbl, dbl, dbl, u64, ptr, ptr, ctypes.c_int]
        lib.corpus_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclass
class Corpus:
    config: CorpusConfig
    doc_ptr: np.ndarray      # int64 [D+1]
    word_ids: np.ndarray     # int32 [T], document-major
    z_true: np.ndarray       # uint16 [T], topics the generative process used

    @property
    def T(self) -> int:
        return int(self.doc_ptr[-1])


def generate(config: CorpusConfig | str, seed: int = CORPUS_SEED, threads: int = 0,
             scale: float = 1.0) -> Corpus:
    """Generate a corpus.  `scale` < 1 shrinks the number of documents only
    (same V, K and length law): used for bounded samples of a large workload."""
    cfg = CONFIGS[config] if isinstance(config, str) else config
    lib = _load()
    D = max(1, int(round(cfg.D * scale)))
    doc_ptr = np.zeros(D + 1, dtype=np.int64)
    if cfg.length_law == "poisson":
        law, p1, p2 = 0, cfg.mean_len, 0.0
    elif cfg.length_law == "lognormal":
        law, p1, p2 = 1, math.log(cfg.mean_len) - 0.5 * cfg.sigma ** 2, cfg.sigma
    else:
        raise ValueError(cfg.length_law)
    T = lib.corpus_doc_lengths(D, law, p1, p2, seed, doc_ptr.ctypes.data)
    word_ids = np.empty(T, dtype=np.int32)
    z_true = np.empty(T, dtype=np.uint16)
    rc = lib.corpus_fill(D, doc_ptr.ctypes.data, cfg.V, cfg.K, cfg.alpha_gen, cfg.beta_gen,
                         cfg.zipf_s, seed, word_ids.ctypes.data, z_true.ctypes.data, threads)
    if rc != 0:
        raise RuntimeError("corpus_fill failed")
    return Corpus(cfg, doc_ptr, word_ids, z_true)


def tiny(D: int, V: int, K: int, mean_len: float, seed: int = 7, name: str = "tiny",
         alpha_gen: float = 0.1, beta_gen: float = 0.01, zipf_s: float = 1.1) -> Corpus:
    """A small Poisson-length corpus with free dimensions (unit tests, edge cases)."""
    return generate(CorpusConfig(name, D, V, K, "poisson", mean_len, 0.0, zipf_s,
                                 alpha_gen, beta_gen, 1), seed=seed)
