"""Thin ctypes binding of the C ABI declared in include/mdg_sgemm.h.

Argument marshalling only: same names, same argument order, device pointers as
plain integers (`tensor.data_ptr()`), streams as integers
(`torch.cuda.current_stream().cuda_stream`).  No arithmetic of the method
happens here, and there is no fallback: if the HIP library has not been built,
`lib()` raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmdg_sgemm.so")

ROW_MAJOR, COL_MAJOR = 101, 102
NO_TRANS, TRANS, CONJ_TRANS = 111, 112, 113

OK = 0
ERR_WORKSPACE, ERR_ILLEGAL_VARIANT, ERR_LAUNCH, ERR_BAD_VARIANT, ERR_NULL, ERR_ALIGNMENT = -101, -102, -103, -104, -105, -106
ERR_SCRATCH_LIMIT = -107
STATIC_SCRATCH_BYTES = 32 << 20  # MDG_STATIC_SCRATCH_BYTES

FAMILY_DIRECT, FAMILY_TILED, FAMILY_SKINNY, FAMILY_INDIRECT = 0, 1, 2, 3
FAMILY_NAMES = {0: "direct", 1: "tiled", 2: "skinny", 3: "indirect"}

MAX_DIM = 2 ** 31 - 1 - 65536  # MDG_MAX_DIM

# every symbol include/mdg_sgemm.h declares
EXPORTS = ("mdg_sgemm", "mdg_sgemm_variant", "mdg_select", "mdg_select_default", "mdg_selector_name",
           "mdg_variant_count", "mdg_variant_info", "mdg_variant_legal", "mdg_workspace_bytes", "mdg_set_workspace",
           "mdg_status_string", "mdg_time_calls", "mdg_time_select_ns", "mdg_select_memo", "mdg_time_select_memo_ns",
           "mdg_sgemm_static_scratch")


class VariantDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("id", "family", "tile_m", "tile_n", "tile_k", "threads", "sub_m", "sub_n",
                                              "vec", "lds", "split_k", "fallback")] + [("name", ctypes.c_char * 48)]

    def as_dict(self):
        d = {n: int(getattr(self, n)) for n, _ in self._fields_[:-1]}
        d["name"] = self.name.decode()
        return d


_lib = None


def lib():
    """Load libmdg_sgemm.so (built by `python -m paper_1806_07060_amd.build`); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not built: run `python -m paper_1806_07060_amd.build` (needs hipcc). "
                           "There is no CPU fallback.")
    L = ctypes.CDLL(LIB_PATH)
    ci, i64, f32, vp, sz = ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
    gemm = [ci, ci, ci, i64, i64, i64, f32, vp, i64, vp, i64, f32, vp, i64, vp]
    L.mdg_sgemm.argtypes, L.mdg_sgemm.restype = gemm, ci
    L.mdg_sgemm_variant.argtypes, L.mdg_sgemm_variant.restype = [ci] + gemm, ci
    L.mdg_sgemm_static_scratch.argtypes, L.mdg_sgemm_static_scratch.restype = gemm, ci
    L.mdg_select.argtypes, L.mdg_select.restype = [ci, ci, i64, i64, i64], ci
    L.mdg_select_default.argtypes, L.mdg_select_default.restype = [ci, ci, i64, i64, i64], ci
    L.mdg_select_memo.argtypes, L.mdg_select_memo.restype = [ci, ci, i64, i64, i64], ci
    L.mdg_selector_name.argtypes, L.mdg_selector_name.restype = [], ctypes.c_char_p
    L.mdg_variant_count.argtypes, L.mdg_variant_count.restype = [], ci
    L.mdg_variant_info.argtypes, L.mdg_variant_info.restype = [ci, ctypes.POINTER(VariantDesc)], ci
    L.mdg_variant_legal.argtypes = [ci, ci, ci, i64, i64, i64, i64, i64, i64, vp, vp, vp]
    L.mdg_variant_legal.restype = ci
    L.mdg_workspace_bytes.argtypes, L.mdg_workspace_bytes.restype = [ci, i64, i64, i64], sz
    L.mdg_set_workspace.argtypes, L.mdg_set_workspace.restype = [vp, sz], ci
    L.mdg_status_string.argtypes, L.mdg_status_string.restype = [ci], ctypes.c_char_p
    L.mdg_time_calls.argtypes = [ci, ci, ci, i64, i64, i64, f32, vp, i64, vp, i64, f32, vp, i64, ci, i64, i64, i64, ci,
                                 ci, ci, ctypes.POINTER(ctypes.c_float), vp]
    L.mdg_time_calls.restype = ci
    p32, p64 = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    L.mdg_time_select_ns.argtypes, L.mdg_time_select_ns.restype = [p32, p32, p64, p64, p64, i64, ci], ctypes.c_double
    L.mdg_time_select_memo_ns.argtypes = [p32, p32, p64, p64, p64, i64, ci]
    L.mdg_time_select_memo_ns.restype = ctypes.c_double
    _lib = L
    return L


def mdg_sgemm(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=0):
    return int(lib().mdg_sgemm(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream))


def mdg_sgemm_static_scratch(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=0):
    return int(lib().mdg_sgemm_static_scratch(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                              stream))


def mdg_sgemm_variant(variant, layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=0):
    return int(lib().mdg_sgemm_variant(variant, layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                       stream))


def mdg_select(transA, transB, M, N, K):
    return int(lib().mdg_select(transA, transB, M, N, K))


def mdg_select_memo(transA, transB, M, N, K):
    return int(lib().mdg_select_memo(transA, transB, M, N, K))


def mdg_select_default(transA, transB, M, N, K):
    return int(lib().mdg_select_default(transA, transB, M, N, K))


def mdg_selector_name():
    return lib().mdg_selector_name().decode()


def mdg_variant_count():
    return int(lib().mdg_variant_count())


def mdg_variant_info(variant):
    d = VariantDesc()
    st = lib().mdg_variant_info(variant, ctypes.byref(d))
    if st != OK:
        raise ValueError(mdg_status_string(st))
    return d.as_dict()


def mdg_variant_legal(variant, transA, transB, M, N, K, lda, ldb, ldc, A=0, B=0, C=0):
    return int(lib().mdg_variant_legal(variant, transA, transB, M, N, K, lda, ldb, ldc, A, B, C))


def mdg_workspace_bytes(variant, M, N, K):
    return int(lib().mdg_workspace_bytes(variant, M, N, K))


def mdg_set_workspace(dev_ptr, nbytes):
    return int(lib().mdg_set_workspace(dev_ptr, nbytes))


def mdg_status_string(status):
    return lib().mdg_status_string(status).decode()


def mdg_time_calls(variant, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, n_sets=1, a_set_stride=0,
                   b_set_stride=0, c_set_stride=0, warmup=3, reps=5, spans=5, stream=0):
    """Returns (status, [ms per call of each span])."""
    out = (ctypes.c_float * spans)()
    st = lib().mdg_time_calls(variant, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, n_sets,
                              a_set_stride, b_set_stride, c_set_stride, warmup, reps, spans, out, stream)
    return int(st), [float(x) for x in out]


def mdg_time_select_ns(transA, transB, M, N, K, iters=100, memo=False):
    n = len(M)
    a32 = lambda v: (ctypes.c_int32 * n)(*[int(x) for x in v])
    a64 = lambda v: (ctypes.c_int64 * n)(*[int(x) for x in v])
    fn = lib().mdg_time_select_memo_ns if memo else lib().mdg_time_select_ns
    return float(fn(a32(transA), a32(transB), a64(M), a64(N), a64(K), n, iters))


def variants():
    """All variant descriptors, by id."""
    return [mdg_variant_info(v) for v in range(mdg_variant_count())]
