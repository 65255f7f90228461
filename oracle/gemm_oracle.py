"""ctypes front-end of the C GEMM oracle (oracle/gemm_oracle.c) -- TEST INFRASTRUCTURE.

Operates on host numpy buffers only.  The matrices are passed as flat fp32
buffers plus leading dimensions, exactly as at the library boundary, so that
padded leading dimensions and both layouts go through the oracle's own index
arithmetic (Eq. 1, Section 2.2 of the paper; BLAS conventions where the paper
is silent).  Also holds `tolerance`, the elementwise acceptance bound the GPU
results are held to.

Nothing under paper_1806_07060_amd/ imports this module.
"""
import ctypes
import os

import numpy as np

from . import build as _build

ROW_MAJOR, COL_MAJOR = 101, 102
NO_TRANS, TRANS, CONJ_TRANS = 111, 112, 113

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i64, f32, ci = ctypes.c_int64, ctypes.c_float, ctypes.c_int
        fp = ctypes.POINTER(ctypes.c_float)
        ip = ctypes.POINTER(ctypes.c_int64)
        gemm_args = [ci, ci, ci, i64, i64, i64, f32, fp, i64, fp, i64, f32, fp, i64]
        for name in ("oracle_sgemm", "oracle_sgemm_ijk"):
            fn = getattr(L, name)
            fn.argtypes = gemm_args
            fn.restype = ci
        L.oracle_sgemm_elements.argtypes = gemm_args + [i64, ip, ip, fp]
        L.oracle_sgemm_elements.restype = ci
        L.oracle_max_threads.argtypes = []
        L.oracle_max_threads.restype = ci
        _lib = L
    return _lib


def _fptr(a):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def max_threads():
    return int(lib().oracle_max_threads())


def sgemm(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, scalar=False):
    """C (flat fp32 buffer) is updated in place; returns the status (0 = ok, -n = n-th argument bad)."""
    fn = lib().oracle_sgemm_ijk if scalar else lib().oracle_sgemm
    return int(fn(layout, transA, transB, M, N, K, alpha, _fptr(A), lda, _fptr(B), ldb, beta, _fptr(C), ldc))


def sgemm_elements(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, ii, jj):
    """The definition at positions (ii[t], jj[t]); C is read only. Returns an fp32 vector."""
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    out = np.empty(ii.shape[0], dtype=np.float32)
    ip = ctypes.POINTER(ctypes.c_int64)
    st = lib().oracle_sgemm_elements(layout, transA, transB, M, N, K, alpha, _fptr(A), lda, _fptr(B), ldb, beta,
                                     _fptr(C), ldc, ii.shape[0], ii.ctypes.data_as(ip), jj.ctypes.data_as(ip),
                                     _fptr(out))
    if st != 0:
        raise ValueError(f"oracle_sgemm_elements status {st}")
    return out


def tolerance(K, max_abs_a, max_abs_b, beta, C0):
    """Elementwise bound a GPU result must meet: 1e-6*K*max|a|*max|b| + 1e-6*|beta*C0|.

    max|a|, max|b| are taken over the logical M x K and K x N regions, C0 is the
    matching array (or scalar) of initial C values.
    """
    return 1e-6 * K * float(max_abs_a) * float(max_abs_b) + 1e-6 * np.abs(np.float64(beta) * np.asarray(C0, np.float64))
