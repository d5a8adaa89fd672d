"""Host-side checks that need no GPU: the library loads, exports what the header
declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1803_04631_amd as mlda

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mlda.LIB_PATH):
        mlda.build()
    return mlda.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "mlda.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mlda_[a-z_]+)\s*\(", header))
    assert len(declared) >= 18 and declared == set(mlda.EXPORTED)
    for name in declared:
        assert getattr(lib, name) is not None


def test_error_strings(lib):
    assert lib.mlda_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4):
        assert len(lib.mlda_strerror(code)) > 3
    assert lib.mlda_strerror(-99) == b"unknown error"


def test_workspace_bytes_validates_and_bounds(lib):
    n = ctypes.c_size_t()
    ok = lib.mlda_workspace_bytes(1000, 100_000, 5000, 32, ctypes.addressof(n))
    assert ok == 0
    # at least the arrays that certainly exist: 3 int32 + 2 uint16 per token, phi
    assert n.value >= 100_000 * 16 + 5000 * 32 * 4
    assert n.value < 64 * 1024 * 1024
    for D, T, V, K in [(-1, 10, 5, 4), (1, -1, 5, 4), (1, 10, 0, 4), (1, 10, 5, 0),
                       (1, 10, 5, 65536), (1, 2**31, 5, 4)]:
        assert lib.mlda_workspace_bytes(D, T, V, K, ctypes.addressof(n)) == -1
    assert lib.mlda_workspace_bytes(1, 10, 5, 4, None) == -1
    assert b"null" in lib.mlda_last_error()
    # a K whose column of p* does not fit the LDS of a workgroup: the workspace also holds the
    # 512 columns of p* that the sampler's workgroups then keep in device memory
    sizes = {}
    for K in (30_000, 31_000, 65_535):
        assert lib.mlda_workspace_bytes(10, 1000, 5, K, ctypes.addressof(n)) == 0
        sizes[K] = n.value
    assert sizes[30_000] < 8 * 1024 * 1024
    assert sizes[31_000] - sizes[30_000] >= 512 * 31_000 * 4
    assert sizes[65_535] >= 512 * 65_536 * 4


def test_create_rejects_bad_arguments_on_the_host(lib):
    ctx = ctypes.c_void_p()
    out = ctypes.addressof(ctx)
    doc_ptr = np.array([0, 2, 5], dtype=np.int64)
    words = np.array([0, 1, 2, 1, 0], dtype=np.int32)
    fake_ws = ctypes.c_void_p(256 * 1000)

    def create(dp=doc_ptr, w=words, D=2, V=3, K=4, alpha=0.5, beta=0.01, ws=fake_ws, nbytes=1 << 30):
        return lib.mlda_create(out, dp.ctypes.data if dp is not None else None,
                               w.ctypes.data if w is not None else None, D, V, K, alpha, beta, 1,
                               ws, nbytes, None)

    assert create(dp=None) == -1
    assert create(w=None) == -1
    assert create(K=0) == -1 and create(K=65536) == -1
    assert create(alpha=0.0) == -1 and create(beta=-1.0) == -1 and create(alpha=float("nan")) == -1
    assert create(dp=np.array([1, 2, 5], dtype=np.int64)) == -1
    assert create(dp=np.array([0, 3, 2], dtype=np.int64)) == -1
    assert create(ws=None) == -1
    assert create(ws=ctypes.c_void_p(100)) == -1          # misaligned
    assert create(nbytes=1000) == -2                       # workspace too small
    assert b"need" in lib.mlda_last_error()
    assert lib.mlda_create(None, doc_ptr.ctypes.data, words.ctypes.data, 2, 3, 4, 0.5, 0.01, 1,
                           fake_ws, 1 << 30, None) == -1
    assert ctx.value is None


def test_null_context_calls_fail_cleanly(lib):
    x = ctypes.c_int64()
    assert lib.mlda_init_random(None) == -1
    assert lib.mlda_step(None, 1, 0) == -1
    assert lib.mlda_get_doc_topic_nnz(None, ctypes.addressof(x)) == -1
    assert lib.mlda_philox_uniform(1, 1, 0, -5, None, None) == -1
    assert lib.mlda_philox_uniform(1, 1, 0, 0, None, None) == 0
    lib.mlda_destroy(None)


def test_binding_checks_array_lengths_before_the_library_reads_them(lib):
    words = np.array([0, 1, 2, 1, 0], dtype=np.int32)
    for bad_ptr in ([0, 2, 6], [0, 2, 4], [1, 2, 5], []):
        with pytest.raises(ValueError):
            mlda.Mlda(np.array(bad_ptr, dtype=np.int64), words, 3, 4, 0.5, 0.01, 1)
