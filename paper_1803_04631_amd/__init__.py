"""Collapsed Gibbs sampling for LDA on one AMD MI355X: Python binding of libmlda.so.

Argument marshalling only: every step of an iteration (sampling, rebuild of phi, n_k
and theta, log-likelihood) runs in the library's HIP kernels.  PyTorch supplies the
device workspace and the stream.  There is no CPU fallback: without the built
library, or without a GPU, construction raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from ._build import LIB_PATH, build  # noqa: F401  (re-exported)

STEP_LOGLIK = 1
STATIC_WORKSPACE_BYTES = 64 << 20     # MLDA_STATIC_WORKSPACE_BYTES of include/mlda.h

_lib = None


class MldaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"mlda error {code}: {message}")
        self.code = code


def load_library() -> ctypes.CDLL:
    """Load the built libmlda.so (never builds implicitly on a GPU machine: build first)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                          "g.build()'` (hipcc, gfx950) first")
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, u64, u32, dbl = (ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint32,
                               ctypes.c_double)
    p, sz = ctypes.c_void_p, ctypes.c_size_t
    sig = {
        "mlda_workspace_bytes": [i64, i64, i32, i32, p],
        "mlda_create": [p, p, p, i64, i32, i32, dbl, dbl, u64, p, sz, p],
        "mlda_workspace_bytes_streamed": [p, i64, i32, i32, i32, p],
        "mlda_create_streamed": [p, p, p, i64, i32, i32, dbl, dbl, u64, i32, p, sz, p],
        "mlda_create_static": [p, p, p, i64, i32, i32, dbl, dbl, u64, p],
        "mlda_init_random": [p],
        "mlda_set_assignments": [p, p, i32],
        "mlda_step": [p, i32, u32],
        "mlda_iteration": [p, p],
        "mlda_get_assignments": [p, p],
        "mlda_get_word_topic": [p, p],
        "mlda_get_topic_totals": [p, p],
        "mlda_get_doc_topic_nnz": [p, p],
        "mlda_get_doc_topic_csr": [p, p, p, p],
        "mlda_get_loglik": [p, p],
        "mlda_get_timing": [p, p, i32, p],
        "mlda_get_sampler_bytes": [p, p, i32, p],
        "mlda_philox_uniform": [u64, u32, u64, i64, p, p],
    }
    for name, argtypes in sig.items():
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = argtypes
    lib.mlda_destroy.restype = None
    lib.mlda_destroy.argtypes = [p]
    lib.mlda_strerror.restype = ctypes.c_char_p
    lib.mlda_strerror.argtypes = [ctypes.c_int]
    lib.mlda_last_error.restype = ctypes.c_char_p
    lib.mlda_last_error.argtypes = []
    _lib = lib
    return lib


EXPORTED = ["mlda_workspace_bytes", "mlda_create", "mlda_workspace_bytes_streamed",
            "mlda_create_streamed", "mlda_create_static", "mlda_init_random", "mlda_set_assignments",
            "mlda_step", "mlda_iteration", "mlda_get_assignments", "mlda_get_word_topic",
            "mlda_get_topic_totals", "mlda_get_doc_topic_nnz", "mlda_get_doc_topic_csr",
            "mlda_get_loglik", "mlda_get_timing", "mlda_get_sampler_bytes", "mlda_destroy",
            "mlda_philox_uniform", "mlda_strerror", "mlda_last_error"]


def _check(rc: int):
    if rc != 0:
        raise MldaError(rc, load_library().mlda_last_error().decode())


def workspace_bytes(D: int, T: int, V: int, K: int) -> int:
    n = ctypes.c_size_t()
    _check(load_library().mlda_workspace_bytes(D, T, V, K, ctypes.addressof(n)))
    return n.value


def philox_uniform(seed: int, it: int, token0: int, n: int):
    """n uniforms as a CUDA float64 tensor (the library's generator, for checks)."""
    import torch
    out = torch.empty(n, dtype=torch.float64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    _check(load_library().mlda_philox_uniform(seed, it, token0, n, out.data_ptr(), stream))
    torch.cuda.current_stream().synchronize()
    return out


class Mlda:
    """One corpus on the GPU: resident (Algorithm 1, WorkSchedule1 with a single chunk), or with
    chunks > 1 cut by document into that many chunks that are streamed through the GPU every
    iteration (WorkSchedule2).  static_workspace: no device memory is allocated, the context
    works in the library's own static array (mlda_create_static; small corpora only)."""

    def __init__(self, doc_ptr, word_ids, V: int, K: int, alpha: float, beta: float, seed: int,
                 device: str = "cuda:0", chunks: int = 1, static_workspace: bool = False):
        import torch
        self.doc_ptr = np.ascontiguousarray(doc_ptr, dtype=np.int64)
        word_ids = np.ascontiguousarray(word_ids, dtype=np.int32)
        if len(self.doc_ptr) < 1 or self.doc_ptr[0] != 0 or int(self.doc_ptr[-1]) != len(word_ids):
            raise ValueError("doc_ptr must start at 0 and end at len(word_ids): the library reads "
                             "word_ids[0 .. doc_ptr[D])")
        self._lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("mlda needs a GPU: there is no CPU path")
        self._torch = torch
        self.D, self.T, self.V, self.K = len(self.doc_ptr) - 1, int(self.doc_ptr[-1]), int(V), int(K)
        self.alpha, self.beta, self.seed = float(alpha), float(beta), int(seed)
        self.device = torch.device(device)
        self.chunks = int(chunks)
        with torch.cuda.device(self.device):
            self.stream = torch.cuda.current_stream(self.device)
            ctx = ctypes.c_void_p()
            if static_workspace:
                if self.chunks != 1:
                    raise ValueError("the static workspace holds a resident corpus only")
                self.workspace = None
                _check(self._lib.mlda_create_static(ctypes.addressof(ctx), self.doc_ptr.ctypes.data,
                                                    word_ids.ctypes.data, self.D, self.V, self.K,
                                                    self.alpha, self.beta, self.seed,
                                                    self.stream.cuda_stream))
            elif self.chunks == 1:
                need = workspace_bytes(self.D, self.T, self.V, self.K)
                self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
                _check(self._lib.mlda_create(ctypes.addressof(ctx), self.doc_ptr.ctypes.data,
                                             word_ids.ctypes.data, self.D, self.V, self.K, self.alpha,
                                             self.beta, self.seed, self.workspace.data_ptr(), need,
                                             self.stream.cuda_stream))
            else:
                n = ctypes.c_size_t()
                _check(self._lib.mlda_workspace_bytes_streamed(self.doc_ptr.ctypes.data, self.D, self.V,
                                                               self.K, self.chunks, ctypes.addressof(n)))
                need = n.value
                self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
                _check(self._lib.mlda_create_streamed(ctypes.addressof(ctx), self.doc_ptr.ctypes.data,
                                                      word_ids.ctypes.data, self.D, self.V, self.K,
                                                      self.alpha, self.beta, self.seed, self.chunks,
                                                      self.workspace.data_ptr(), need,
                                                      self.stream.cuda_stream))
        self._ctx = ctx

    # -- state
    def init_random(self):
        _check(self._lib.mlda_init_random(self._ctx))

    def set_assignments(self, z, it: int = 0):
        z = np.ascontiguousarray(z, dtype=np.uint16)
        if len(z) != self.T:
            raise ValueError("z must have one entry per token")
        _check(self._lib.mlda_set_assignments(self._ctx, z.ctypes.data, it))

    def step(self, n_iters: int = 1, loglik: bool = False):
        _check(self._lib.mlda_step(self._ctx, n_iters, STEP_LOGLIK if loglik else 0))

    def synchronize(self):
        self.stream.synchronize()

    # -- getters
    @property
    def iteration(self) -> int:
        it = ctypes.c_int32()
        _check(self._lib.mlda_iteration(self._ctx, ctypes.addressof(it)))
        return it.value

    def assignments(self) -> np.ndarray:
        z = np.empty(self.T, dtype=np.uint16)
        _check(self._lib.mlda_get_assignments(self._ctx, z.ctypes.data))
        return z

    def word_topic(self) -> np.ndarray:
        n_wk = np.empty((self.V, self.K), dtype=np.int32)
        _check(self._lib.mlda_get_word_topic(self._ctx, n_wk.ctypes.data))
        return n_wk

    def topic_totals(self) -> np.ndarray:
        n_k = np.empty(self.K, dtype=np.int32)
        _check(self._lib.mlda_get_topic_totals(self._ctx, n_k.ctypes.data))
        return n_k

    def doc_topic_nnz(self) -> int:
        n = ctypes.c_int64()
        _check(self._lib.mlda_get_doc_topic_nnz(self._ctx, ctypes.addressof(n)))
        return n.value

    def doc_topic_csr(self):
        nnz = self.doc_topic_nnz()
        row_ptr = np.empty(self.D + 1, dtype=np.int64)
        topics = np.empty(nnz, dtype=np.uint16)
        counts = np.empty(nnz, dtype=np.int32)
        _check(self._lib.mlda_get_doc_topic_csr(self._ctx, row_ptr.ctypes.data, topics.ctypes.data,
                                                counts.ctypes.data))
        return row_ptr, topics, counts

    def loglik(self) -> float:
        ll = ctypes.c_double()
        _check(self._lib.mlda_get_loglik(self._ctx, ctypes.addressof(ll)))
        return ll.value

    def timing(self, capacity: int = 1024) -> np.ndarray:
        """[n_iters, 4] ms of the last step: sampling, rebuild phi+n_k, rebuild theta, loglik."""
        ms = np.zeros((capacity, 4), dtype=np.float64)
        n = ctypes.c_int32()
        _check(self._lib.mlda_get_timing(self._ctx, ms.ctypes.data, capacity, ctypes.addressof(n)))
        return ms[:n.value]

    def sampler_bytes(self, capacity: int = 1024) -> np.ndarray:
        """Algorithmic bytes of each sampling launch of the last step (same rows as timing)."""
        b = np.zeros(capacity, dtype=np.float64)
        n = ctypes.c_int32()
        _check(self._lib.mlda_get_sampler_bytes(self._ctx, b.ctypes.data, capacity,
                                                ctypes.addressof(n)))
        return b[:n.value]

    def close(self):
        if getattr(self, "_ctx", None):
            self._lib.mlda_destroy(self._ctx)
            self._ctx = None
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
