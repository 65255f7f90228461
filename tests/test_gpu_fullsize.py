"""GPU parity at the sizes and in the launch configuration bench.py times: calls go through mdg_sgemm (selector,
legality, kernel) on the full-size square cases and are checked on sampled outputs the oracle computes one by one
(tile-boundary rows / columns plus random positions); skinny and convolution-lowered cases are checked in full.
"""
import numpy as np
import pytest

from paper_1806_07060_amd import binding as mdg
from paper_1806_07060_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _sample_positions(M, N, rng, n_random=2048):
    edges_m = sorted({0, 1, 31, 32, 63, 64, 127, 128, 255, 256, 257, M // 2, M - 257, M - 256, M - 129, M - 2, M - 1} & set(range(M)))
    edges_n = sorted({0, 1, 31, 32, 63, 64, 127, 128, 255, 256, 257, N // 2, N - 257, N - 256, N - 129, N - 2, N - 1} & set(range(N)))
    ii = [i for i in edges_m for _ in edges_n]
    jj = [j for _ in edges_m for j in edges_n]
    ii += rng.integers(0, M, n_random).tolist()
    jj += rng.integers(0, N, n_random).tolist()
    return np.array(ii, np.int64), np.array(jj, np.int64)


@pytest.mark.parametrize("n,combos", [(4096, ("NN", "NT", "TN", "TT")), (8192, ("NN", "TT"))])
def test_square_sweep_full_size_sampled(n, combos):
    from oracle import gemm_oracle as go
    from tests import gpu_util as gu
    torch = gu.torch_mod()
    gu.ensure_workspace()
    rng = np.random.default_rng(n)
    for case in wl.config1(sizes=(n,)):
        if case.name[-2:] not in combos:
            continue
        c = case.resolved()
        A, B, C0 = wl.make_operands(c, poison=False)
        dA, dB, dC = (torch.from_numpy(x).cuda() for x in (A, B, C0))
        st = mdg.mdg_sgemm(c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, dA.data_ptr(), c.lda, dB.data_ptr(),
                           c.ldb, c.beta, dC.data_ptr(), c.ldc, torch.cuda.current_stream().cuda_stream)
        assert st == 0, mdg.mdg_status_string(st)
        torch.cuda.synchronize()
        got = dC.cpu().numpy()
        del dA, dB, dC
        ii, jj = _sample_positions(c.M, c.N, rng)
        ref = go.sgemm_elements(c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, A, c.lda, B, c.ldb, c.beta, C0,
                                c.ldc, ii, jj)
        g = wl.matrix_view(got, c.layout, c.c_shape(), c.ldc)[ii, jj]
        c0 = wl.matrix_view(C0, c.layout, c.c_shape(), c.ldc)[ii, jj]
        tol = go.tolerance(c.K, np.abs(A).max(), np.abs(B).max(), c.beta, c0)
        err = np.abs(g.astype(np.float64) - ref.astype(np.float64))
        assert np.all(err <= tol), f"{c.name}: max err {err.max():.3e} vs tol {tol.min():.3e}"
        # a wrong tile anywhere shows up in the column / row sums of the whole result: compare a cheap
        # global invariant too -- sum over all of C against alpha * (1^T A)(B 1) + beta * sum(C0) in fp64
        Av = wl.matrix_view(A, c.layout, c.a_shape(), c.lda).astype(np.float64)
        Bv = wl.matrix_view(B, c.layout, c.b_shape(), c.ldb).astype(np.float64)
        sa = Av.sum(axis=1) if c.tA() else Av.sum(axis=0)  # sum over m of op(A)(m, k)
        sb = Bv.sum(axis=0) if c.tB() else Bv.sum(axis=1)  # sum over n of op(B)(k, n)
        want = c.alpha * float(sa @ sb) + c.beta * float(C0.astype(np.float64).sum())
        have = float(wl.matrix_view(got, c.layout, c.c_shape(), c.ldc).astype(np.float64).sum())
        assert abs(have - want) <= 1e-6 * c.K * c.M * c.N ** 0.5 + 1e-3 * abs(want), (c.name, have, want)


def test_skinny_and_conv_cases_full_check_through_the_selector():
    from tests import gpu_util as gu
    gu.ensure_workspace()
    picks = []
    c2 = wl.config2()
    picks += [c for c in c2 if (c.M, c.K) in ((1024, 1024), (7680, 2048)) and c.N in (1, 4, 16, 128)]
    c3 = wl.config3()
    picks += [c for c in c3 if (c.M, c.N, c.K) in ((32, 50176, 27), (128, 12544, 288), (512, 3136, 1152), (64, 3136, 2304))]
    assert len(picks) == 20
    for case in picks:
        st, got, A, B, C0 = gu.run_case(case, poison=False)
        assert st == 0
        gu.check_against_oracle(case, got, A, B, C0)


def test_unaligned_large_ragged_shapes_every_tiled_tile_shape():
    # sizes that are not multiples of any tile, odd leading dimensions (nothing 16-byte aligned): guarded path
    from tests import gpu_util as gu
    gu.ensure_workspace()
    base = wl.GemmCase(1031, 517, 777, wl.TRANS, wl.NO_TRANS, 1.0, 0.5, seed=wl.case_seed(13, 1), name="ragged-large").resolved()
    case = wl.GemmCase(**{**base.__dict__, "lda": base.lda + 1, "ldb": base.ldb + 3, "ldc": base.ldc + 1})
    A, B, C0 = wl.make_operands(case)
    ref = gu.oracle_result(case, A, B, C0)
    for v in gu.legal_variants(case):
        d = mdg.mdg_variant_info(v)
        if d["family"] != mdg.FAMILY_TILED:
            continue
        st, got, *_ = gu.run_case(case, variant=v)
        assert st == 0
        try:
            gu.check_against_oracle(case, got, A, B, C0, ref=ref)
        except AssertionError as e:
            raise AssertionError(f"{d['name']}: {e}") from None


@pytest.mark.parametrize("tA", [0, 1])
def test_leading_dimensions_that_put_elements_past_four_gigabytes(tA):
    # element offsets of A and C exceed 2^32 bytes: every index computation must be 64-bit.  The matrices are
    # small (40 x 36 x 40); only their leading dimensions are huge.  Device buffers are allocated uninitialised and
    # only the logical entries are written; the oracle sees the same matrices with tight leading dimensions.
    import torch
    from oracle import gemm_oracle as go
    from tests import gpu_util as gu
    gu.ensure_workspace()
    M, N, K = 40, 36, 40
    lda, ldb, ldc = (1 << 25) + 1, K + 4, (1 << 25) + 4
    rng = np.random.default_rng(77 + tA)
    a_rows, a_cols = (K, M) if tA else (M, K)  # stored shape of A
    A = rng.integers(-8, 9, (a_rows, a_cols)).astype(np.float32)
    B = rng.integers(-8, 9, (K, N)).astype(np.float32)
    C0 = rng.integers(-8, 9, (M, N)).astype(np.float32)
    assert 4 * lda * (a_cols - 1) > 2 ** 32 and 4 * ldc * (N - 1) > 2 ** 32
    dA = torch.empty(lda * (a_cols - 1) + a_rows, dtype=torch.float32, device="cuda")
    dB = torch.empty(ldb * (N - 1) + K, dtype=torch.float32, device="cuda")
    dC = torch.empty(ldc * (N - 1) + M, dtype=torch.float32, device="cuda")
    dA.as_strided((a_rows, a_cols), (1, lda)).copy_(torch.from_numpy(A))
    dB.as_strided((K, N), (1, ldb)).copy_(torch.from_numpy(B))
    ref = np.asfortranarray(C0).ravel(order="F").copy()
    alpha, beta = 2.0, -1.0
    tr = wl.TRANS if tA else wl.NO_TRANS
    assert go.sgemm(wl.COL_MAJOR, tr, wl.NO_TRANS, M, N, K, alpha, np.asfortranarray(A).ravel(order="F"), a_rows,
                    np.asfortranarray(B).ravel(order="F"), K, beta, ref, M) == 0
    ref = ref.reshape((M, N), order="F")
    stream = torch.cuda.current_stream().cuda_stream
    legal = [v for v in range(mdg.mdg_variant_count())
             if mdg.mdg_variant_legal(v, tA, 0, M, N, K, lda, ldb, ldc, dA.data_ptr(), dB.data_ptr(), dC.data_ptr()) == 1]
    assert 0 in legal and len(legal) > 20
    view = dC.as_strided((M, N), (1, ldc))
    for v in [None] + legal:
        view.copy_(torch.from_numpy(C0))
        args = (wl.COL_MAJOR, tr, wl.NO_TRANS, M, N, K, alpha, dA.data_ptr(), lda, dB.data_ptr(), ldb, beta, dC.data_ptr(), ldc, stream)
        st = mdg.mdg_sgemm(*args) if v is None else mdg.mdg_sgemm_variant(v, *args)
        assert st == 0, (v, mdg.mdg_status_string(st))
        torch.cuda.synchronize()
        got = view.cpu().numpy()
        name = "selector" if v is None else mdg.mdg_variant_info(v)["name"]
        assert np.array_equal(got, ref), f"{name}: max diff {np.abs(got - ref).max()}"  # integer data: exact
