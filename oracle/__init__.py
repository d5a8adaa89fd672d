"""CPU oracle for the LDA collapsed-Gibbs iteration (TEST INFRASTRUCTURE ONLY).

Thin ctypes access to `lda_oracle.c`, the plain fp64 statement of what the GPU
library computes (paper Eq. 1, Eq. 6-8, Algorithm 2).  Only tests, the smoke
check and the benchmark's CPU-baseline leg may import this package; the
product package never does, and this package never imports the product.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lda_oracle.c")
_LIB = os.path.join(_HERE, "liblda_oracle.so")

# -ffp-contract=off: no fused multiply-adds, so every product and sum rounds as written.
_CFLAGS = ["-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math"]


def build(force: bool = False) -> str:
    # The mutation test binds deliberately broken builds in subprocesses of its own: the
    # override counts only together with the marker that test sets, so that no other
    # environment can swap the checker under the parity tests.
    override = os.environ.get("LDA_ORACLE_LIB")
    if override and os.environ.get("LDA_ORACLE_MUTATION_TEST") == "1":
        return override
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *_CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = bind(build())
    return _lib


def bind(path: str):
    """Load an oracle library from `path` and declare its signatures (the mutation test
    binds deliberately broken builds this way)."""
    lib = ctypes.CDLL(path)
    i64, i32, u64, u32, dbl = (ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                               ctypes.c_uint32, ctypes.c_double)
    p = ctypes.c_void_p
    lib.oracle_philox4x32_10.restype = None
    lib.oracle_philox4x32_10.argtypes = [p, p, p]
    lib.oracle_uniform.restype = dbl
    lib.oracle_uniform.argtypes = [u64, u32, u64]
    lib.oracle_uniforms.restype = None
    lib.oracle_uniforms.argtypes = [u64, u32, u64, i64, p]
    lib.oracle_init_topics.restype = None
    lib.oracle_init_topics.argtypes = [i64, i32, u64, p]
    lib.oracle_count_word_topic.restype = None
    lib.oracle_count_word_topic.argtypes = [i64, p, p, i32, i32, p, p]
    lib.oracle_doc_topic_csr.restype = i64
    lib.oracle_doc_topic_csr.argtypes = [i64, p, p, i32, p, p, p]
    lib.oracle_resample_token.restype = i32
    lib.oracle_resample_token.argtypes = [i32, i32, dbl, dbl, p, p, p, i32, dbl, p, p, p]
    lib.oracle_iteration.restype = None
    lib.oracle_iteration.argtypes = [i64, p, p, p, i32, i32, dbl, dbl, u64, u32, p, p, p,
                                     ctypes.c_int]
    lib.oracle_resample_listed.restype = None
    lib.oracle_resample_listed.argtypes = [i64, p, p, p, p, p, i32, i32, dbl, dbl, u64, u32,
                                           p, p, p]
    lib.oracle_loglik.restype = dbl
    lib.oracle_loglik.argtypes = [i64, p, p, i32, i32, dbl, dbl, p, p]
    lib.oracle_max_threads.restype = ctypes.c_int
    return lib


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def philox4x32_10(ctr, key) -> np.ndarray:
    ctr = _c(ctr, np.uint32); key = _c(key, np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(ctr.ctypes.data, key.ctypes.data, out.ctypes.data)
    return out


def uniform(seed: int, it: int, token: int) -> float:
    return _load().oracle_uniform(seed, it, token)


def uniforms(seed: int, it: int, token0: int, n: int) -> np.ndarray:
    u = np.empty(n, dtype=np.float64)
    _load().oracle_uniforms(seed, it, token0, n, u.ctypes.data)
    return u


def init_topics(T: int, K: int, seed: int) -> np.ndarray:
    z = np.empty(T, dtype=np.uint16)
    _load().oracle_init_topics(T, K, seed, z.ctypes.data)
    return z


def count_word_topic(word_ids, z, V: int, K: int):
    word_ids = _c(word_ids, np.int32); z = _c(z, np.uint16)
    n_wk = np.empty((V, K), dtype=np.int32)
    n_k = np.empty(K, dtype=np.int32)
    _load().oracle_count_word_topic(len(z), word_ids.ctypes.data, z.ctypes.data, V, K,
                                    n_wk.ctypes.data, n_k.ctypes.data)
    return n_wk, n_k


def doc_topic_csr(doc_ptr, z, K: int):
    doc_ptr = _c(doc_ptr, np.int64); z = _c(z, np.uint16)
    D = len(doc_ptr) - 1
    row_ptr = np.empty(D + 1, dtype=np.int64)
    nnz = _load().oracle_doc_topic_csr(D, doc_ptr.ctypes.data, z.ctypes.data, K,
                                       row_ptr.ctypes.data, None, None)
    topics = np.empty(nnz, dtype=np.uint16)
    counts = np.empty(nnz, dtype=np.int32)
    _load().oracle_doc_topic_csr(D, doc_ptr.ctypes.data, z.ctypes.data, K,
                                 row_ptr.ctypes.data, topics.ctypes.data, counts.ctypes.data)
    return row_ptr, topics, counts


def resample_token(K: int, V: int, alpha: float, beta: float, n_d, n_w, n_k, o: int, u: float):
    """Returns (new topic, S, Q) for one token given its frozen dense count rows."""
    n_d = _c(n_d, np.int32); n_w = _c(n_w, np.int32); n_k = _c(n_k, np.int32)
    work = np.empty(2 * K, dtype=np.float64)
    S = ctypes.c_double(); Q = ctypes.c_double()
    k = _load().oracle_resample_token(K, V, alpha, beta, n_d.ctypes.data, n_w.ctypes.data,
                                      n_k.ctypes.data, o, u, work.ctypes.data,
                                      ctypes.addressof(S), ctypes.addressof(Q))
    return k, S.value, Q.value


def iteration(doc_ptr, word_ids, z, V: int, K: int, alpha: float, beta: float, seed: int,
              it: int, n_wk=None, n_k=None, threads: int = 0) -> np.ndarray:
    """One full pass from the counts of z; returns the new assignments."""
    doc_ptr = _c(doc_ptr, np.int64); word_ids = _c(word_ids, np.int32); z = _c(z, np.uint16)
    if n_wk is None or n_k is None:
        n_wk, n_k = count_word_topic(word_ids, z, V, K)
    n_wk = _c(n_wk, np.int32); n_k = _c(n_k, np.int32)
    z_new = np.empty_like(z)
    _load().oracle_iteration(len(doc_ptr) - 1, doc_ptr.ctypes.data, word_ids.ctypes.data,
                             z.ctypes.data, V, K, alpha, beta, seed, it, n_wk.ctypes.data,
                             n_k.ctypes.data, z_new.ctypes.data, threads)
    return z_new


def resample_listed(tokens, doc_ptr, word_ids, z, V: int, K: int, alpha: float, beta: float,
                    seed: int, it: int, n_wk, n_k) -> np.ndarray:
    """New topics of the listed tokens only (document-major token indices)."""
    doc_ptr = _c(doc_ptr, np.int64); word_ids = _c(word_ids, np.int32); z = _c(z, np.uint16)
    tokens = _c(tokens, np.int64)
    docs = (np.searchsorted(doc_ptr, tokens, side="right") - 1).astype(np.int64)
    n_wk = _c(n_wk, np.int32); n_k = _c(n_k, np.int32)
    out = np.empty(len(tokens), dtype=np.uint16)
    _load().oracle_resample_listed(len(tokens), tokens.ctypes.data, docs.ctypes.data,
                                   doc_ptr.ctypes.data, word_ids.ctypes.data, z.ctypes.data,
                                   V, K, alpha, beta, seed, it, n_wk.ctypes.data,
                                   n_k.ctypes.data, out.ctypes.data)
    return out


def loglik(doc_ptr, z, V: int, K: int, alpha: float, beta: float, n_wk, n_k) -> float:
    doc_ptr = _c(doc_ptr, np.int64); z = _c(z, np.uint16)
    n_wk = _c(n_wk, np.int32); n_k = _c(n_k, np.int32)
    return _load().oracle_loglik(len(doc_ptr) - 1, doc_ptr.ctypes.data, z.ctypes.data, V, K,
                                 alpha, beta, n_wk.ctypes.data, n_k.ctypes.data)


def max_threads() -> int:
    return _load().oracle_max_threads()
