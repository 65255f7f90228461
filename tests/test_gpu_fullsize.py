"""GPU parity on large awkward inputs: ragged, unaligned shapes through every tiled tile shape, and leading
dimensions that put elements more than 4 GB past the base pointer.  (The named workloads at their full sizes are
in test_gpu_named_configs.py.)
"""
import numpy as np
import pytest

from paper_1806_07060_amd import binding as mdg
from paper_1806_07060_amd import workloads as wl

pytestmark = pytest.mark.gpu


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
