"""Helpers for the GPU parity tests: run one seeded case through the C ABI and hold it to the oracle."""
import numpy as np

from oracle import gemm_oracle as go
from paper_1806_07060_amd import binding as mdg
from paper_1806_07060_amd import workloads as wl

_WS = {}


def torch_mod():
    import torch
    return torch


def ensure_workspace(nbytes=256 << 20):
    """Register one workspace tensor (kept alive for the process)."""
    torch = torch_mod()
    if _WS.get("bytes", 0) < nbytes:
        t = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
        assert mdg.mdg_set_workspace(t.data_ptr(), t.numel() * 4) == 0
        _WS["t"], _WS["bytes"] = t, nbytes
    return _WS["t"]


def run_case(case, variant=None, poison=True):
    """Upload the case's operands, call the library, return (status, C_host_flat, A, B, C0) as host buffers."""
    torch = torch_mod()
    c = case.resolved()
    A, B, C0 = wl.make_operands(c, poison=poison)
    dA, dB, dC = (torch.from_numpy(x).cuda() for x in (A, B, C0))
    stream = torch.cuda.current_stream().cuda_stream
    args = (c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, dA.data_ptr(), c.lda, dB.data_ptr(), c.ldb, c.beta,
            dC.data_ptr(), c.ldc, stream)
    st = mdg.mdg_sgemm(*args) if variant is None else mdg.mdg_sgemm_variant(variant, *args)
    torch.cuda.synchronize()
    return st, dC.cpu().numpy(), A, B, C0


def oracle_result(case, A, B, C0):
    c = case.resolved()
    ref = C0.copy()
    assert go.sgemm(c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, A, c.lda, B, c.ldb, c.beta, ref, c.ldc) == 0
    return ref


def check_against_oracle(case, got, A, B, C0, exact=False, ref=None):
    """Elementwise |C - C_ref| <= 1e-6*K*max|a|*max|b| + 1e-6*|beta*C0| on the logical region; padding untouched."""
    c = case.resolved()
    if ref is None:
        ref = oracle_result(c, A, B, C0)
    shape = c.c_shape()
    g = wl.matrix_view(got, c.layout, shape, c.ldc)
    r = wl.matrix_view(ref, c.layout, shape, c.ldc)
    c0 = wl.matrix_view(C0, c.layout, shape, c.ldc)
    assert not np.any(np.isnan(g)), f"{c.name}: NaN in result (padding read?)"
    if exact:
        assert np.array_equal(g, r), f"{c.name}: not bit-exact, max diff {np.max(np.abs(g - r))}"
    else:
        amax = wl.logical_max_abs(A, c.layout, c.a_shape(), c.lda)
        bmax = wl.logical_max_abs(B, c.layout, c.b_shape(), c.ldb)
        tol = go.tolerance(c.K, amax, bmax, c.beta, np.where(np.isfinite(c0), c0, 0.0) if c.beta != 0 else 0.0)
        err = np.abs(g.astype(np.float64) - r.astype(np.float64))
        worst = np.max(err - tol) if err.size else -1.0
        assert worst <= 0.0, f"{c.name}: max error {err.max():.3e} exceeds tolerance by {worst:.3e}"
    # everything outside the logical region must be bit-identical to what was uploaded
    mask = np.ones(got.shape, bool)
    if shape[0] and shape[1]:
        idx = wl.matrix_view(np.arange(got.size), c.layout, shape, c.ldc)
        mask[idx.ravel()] = False
    assert np.array_equal(got[mask], C0[mask], equal_nan=True), f"{c.name}: padding of C was written"


def legal_variants(case):
    c = case.resolved()
    if c.layout == wl.COL_MAJOR:
        tA, tB, M, N, lda, ldb = c.tA(), c.tB(), c.M, c.N, c.lda, c.ldb
    else:
        tA, tB, M, N, lda, ldb = c.tB(), c.tA(), c.N, c.M, c.ldb, c.lda
    return [v for v in range(mdg.mdg_variant_count())
            if mdg.mdg_variant_legal(v, tA, tB, M, N, c.K, lda, ldb, c.ldc) == 1]


def run_case_many(case, variants, poison=False):
    """One upload of the case's operands, then one call per entry of `variants` (None = mdg_sgemm, i.e. the
    selector; an id = that variant forced), each on a fresh copy of C0.  Returns (A, B, C0, [(status, C_host)])."""
    torch = torch_mod()
    c = case.resolved()
    A, B, C0 = wl.make_operands(c, poison=poison)
    dA, dB, dC0 = (torch.from_numpy(x).cuda() for x in (A, B, C0))
    stream = torch.cuda.current_stream().cuda_stream
    outs = []
    for v in variants:
        dC = dC0.clone()
        args = (c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, dA.data_ptr(), c.lda, dB.data_ptr(), c.ldb,
                c.beta, dC.data_ptr(), c.ldc, stream)
        st = mdg.mdg_sgemm(*args) if v is None else mdg.mdg_sgemm_variant(v, *args)
        torch.cuda.synchronize()
        outs.append((st, dC.cpu().numpy()))
    return A, B, C0, outs
