"""The allocation-free entry point mdg_sgemm_static_scratch against mdg_sgemm, through the C ABI.

Both run the same variant on the same kernels (the selector's choice with a workspace that is large enough), and
the split-K reduce adds the slices in slice order, so the two results must be bit-identical; mdg_sgemm's result
is itself held to the oracle's tolerance.  Two calls in a row share the static array, the second with a smaller
input: stale partial sums of the first call must not leak into it.
"""
import numpy as np
import pytest

from paper_1806_07060_amd import binding as mdg
from paper_1806_07060_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _split_k_shapes():
    """Shapes for which the compiled selector picks a split-K variant that fits / does not fit the static array."""
    V = mdg.variants()
    fits, too_big = [], []
    for M in (3072, 1024, 512, 256, 128, 64):
        for N in (2048, 512, 128, 64, 16):
            for K in (16384, 8192, 4096, 1024):
                for tA in (0, 1):
                    d = V[mdg.mdg_select(tA, 0, M, N, K)]
                    if d["split_k"] > 1:
                        need = d["split_k"] * M * N * 4
                        (fits if need <= mdg.STATIC_SCRATCH_BYTES else too_big).append((M, N, K, tA, d["name"]))
    return fits, too_big


def _call(fn, c, dA, dB, dC, stream):
    return fn(c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, dA.data_ptr(), c.lda, dB.data_ptr(), c.ldb, c.beta,
              dC.data_ptr(), c.ldc, stream)


def test_static_scratch_entry_point_matches_mdg_sgemm_on_two_calls_in_a_row():
    import torch
    from tests import gpu_util as gu
    fits, _ = _split_k_shapes()
    assert len(fits) >= 2, "the selector picks no split-K variant on the probe shapes"
    big = max(fits, key=lambda s: s[0] * s[1])
    small = min(fits, key=lambda s: s[0] * s[1])
    assert small[0] * small[1] < big[0] * big[1]
    stream = torch.cuda.current_stream().cuda_stream
    results = []
    cases = []
    for i, (M, N, K, tA, name) in enumerate((big, small)):
        case = wl.GemmCase(M, N, K, wl.TRANS if tA else wl.NO_TRANS, wl.NO_TRANS, 1.25, -0.5,
                           seed=wl.case_seed(30, i), name=f"static-scratch/{name}/{M}x{N}x{K}").resolved()
        A, B, C0 = wl.make_operands(case, poison=False)
        cases.append((case, A, B, C0))
    # no workspace registered: the new entry point must not need one
    assert mdg.mdg_set_workspace(0, 0) == 0
    dev = [tuple(torch.from_numpy(x).cuda() for x in (A, B, C0)) for _, A, B, C0 in cases]
    torch.cuda.synchronize()
    for (case, *_), (dA, dB, dC) in zip(cases, dev):  # back to back, no synchronisation in between
        assert _call(mdg.mdg_sgemm_static_scratch, case, dA, dB, dC, stream) == 0
    torch.cuda.synchronize()
    results = [dC.cpu().numpy() for _, _, dC in dev]
    # the existing entry point, with a registered workspace that is large enough
    gu.ensure_workspace()
    ws = gu._WS["t"]
    assert mdg.mdg_set_workspace(ws.data_ptr(), ws.numel() * 4) == 0
    for (case, A, B, C0), (dA, dB, _), got in zip(cases, dev, results):
        dC = torch.from_numpy(C0).cuda()
        assert _call(mdg.mdg_sgemm, case, dA, dB, dC, stream) == 0
        torch.cuda.synchronize()
        want = dC.cpu().numpy()
        assert np.array_equal(got, want), f"{case.name}: max diff {np.abs(got - want).max()}"
        gu.check_against_oracle(case, got, A, B, C0)


def test_static_scratch_entry_point_refuses_what_does_not_fit_and_handles_plain_variants():
    import torch
    from tests import gpu_util as gu
    _, too_big = _split_k_shapes()
    stream = torch.cuda.current_stream().cuda_stream
    if too_big:
        M, N, K, tA, name = too_big[0]
        case = wl.GemmCase(M, N, K, wl.TRANS if tA else wl.NO_TRANS, wl.NO_TRANS, 1.0, 0.0, seed=wl.case_seed(30, 9)).resolved()
        dA = torch.zeros(M * K, device="cuda")
        dB = torch.zeros(K * N, device="cuda")
        dC = torch.full((M * N,), 3.0, device="cuda")
        assert _call(mdg.mdg_sgemm_static_scratch, case, dA, dB, dC, stream) == mdg.ERR_SCRATCH_LIMIT
        torch.cuda.synchronize()
        assert bool((dC == 3.0).all())  # nothing was enqueued
    # a shape served by a variant without split-K, a degenerate one, and an argument error
    case = wl.GemmCase(300, 200, 260, wl.TRANS, wl.TRANS, 1.0, 0.5, seed=wl.case_seed(30, 10), name="static-scratch/plain").resolved()
    A, B, C0 = wl.make_operands(case)
    dA, dB, dC = (torch.from_numpy(x).cuda() for x in (A, B, C0))
    assert _call(mdg.mdg_sgemm_static_scratch, case, dA, dB, dC, stream) == 0
    torch.cuda.synchronize()
    gu.check_against_oracle(case, dC.cpu().numpy(), A, B, C0)
    assert mdg.mdg_sgemm_static_scratch(case.layout, case.transA, case.transB, case.M, case.N, 0, 1.0, 0, case.lda, 0,
                                        case.ldb, 0.0, dC.data_ptr(), case.ldc, stream) == 0
    torch.cuda.synchronize()
    assert bool((dC.cpu() == 0).all()) or case.ldc > case.M
    assert mdg.mdg_sgemm_static_scratch(case.layout, case.transA, case.transB, case.M, case.N, case.K, 1.0, dA.data_ptr(),
                                        1, dB.data_ptr(), case.ldb, 0.0, dC.data_ptr(), case.ldc, stream) == -9
