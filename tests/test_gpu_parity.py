"""GPU parity: every kernel variant, through the C ABI, element by element against the CPU oracle.

Bar: |C - C_ref| <= 1e-6*K*max|a|*max|b| + 1e-6*|beta*C0| for floating-point data, bit-exact for
small-integer data (every partial sum is then exactly representable in fp32 whatever the summation order).
"""
import itertools

import numpy as np
import pytest

from paper_1806_07060_amd import binding as mdg
from paper_1806_07060_amd import workloads as wl
from paper_1806_07060_amd.workloads import GemmCase, NO_TRANS as NT, TRANS as TR, COL_MAJOR as CM, ROW_MAJOR as RM

pytestmark = pytest.mark.gpu

TT = list(itertools.product((NT, TR), (NT, TR)))


@pytest.fixture(scope="module", autouse=True)
def _workspace():
    from tests import gpu_util as gu
    gu.ensure_workspace()
    yield


def _gu():
    from tests import gpu_util as gu
    return gu


def test_config0_every_legal_variant_and_the_selector():
    gu = _gu()
    case = wl.config0()[0]
    st, got, A, B, C0 = gu.run_case(case)
    assert st == 0
    ref = gu.oracle_result(case, A, B, C0)
    gu.check_against_oracle(case, got, A, B, C0, ref=ref)
    legal = gu.legal_variants(case)
    assert 0 in legal and len(legal) >= 20
    for v in legal:
        st, got, *_ = gu.run_case(case, variant=v)
        assert st == 0, (v, mdg.mdg_status_string(st))
        gu.check_against_oracle(case, got, A, B, C0, ref=ref)


# shapes that span several tiles of every configuration and leave ragged tails in M, N and K
RAGGED = [(150, 77, 260), (257, 129, 65), (5, 300, 17), (300, 3, 1000), (33, 4, 2049), (515, 260, 40), (1, 1, 1),
          (64, 64, 64), (256, 256, 48), (130, 2, 515)]


@pytest.mark.parametrize("M,N,K", RAGGED)
def test_all_variants_all_transposes_ragged_shapes(M, N, K):
    gu = _gu()
    for i, (tA, tB) in enumerate(TT):
        # alternate tight / padded (odd, so nothing is 16-byte aligned) leading dimensions and alpha/beta mixes
        pad = (0, 0, 0) if i % 2 == 0 else (3, 1, 5)
        alpha, beta = [(1.0, 0.0), (0.75, 0.5), (-1.5, 1.0), (2.0, -0.25)][i]
        base = GemmCase(M, N, K, tA, tB, alpha, beta, seed=wl.case_seed(10, 1000 * i + M + N + K),
                        name=f"ragged/{M}x{N}x{K}/{tA}{tB}").resolved()
        case = GemmCase(**{**base.__dict__, "lda": base.lda + pad[0], "ldb": base.ldb + pad[1], "ldc": base.ldc + pad[2]})
        A, B, C0 = wl.make_operands(case)
        ref = gu.oracle_result(case, A, B, C0)
        for v in gu.legal_variants(case):
            st, got, *_ = gu.run_case(case, variant=v)
            assert st == 0, (v, mdg.mdg_status_string(st))
            try:
                gu.check_against_oracle(case, got, A, B, C0, ref=ref)
            except AssertionError as e:
                raise AssertionError(f"variant {v} {mdg.mdg_variant_info(v)['name']}: {e}") from None


@pytest.mark.parametrize("tA,tB", TT)
def test_small_integer_data_is_bit_exact_for_every_variant(tA, tB):
    gu = _gu()
    case = GemmCase(200, 100, 300, tA, tB, 2.0, -1.0, dist="smallint", c0="smallint", ldc=203,
                    seed=wl.case_seed(11, tA * 10 + tB), name=f"smallint/{tA}{tB}")
    A, B, C0 = wl.make_operands(case)
    ref = gu.oracle_result(case, A, B, C0)
    for v in gu.legal_variants(case):
        st, got, *_ = gu.run_case(case, variant=v)
        assert st == 0
        try:
            gu.check_against_oracle(case, got, A, B, C0, exact=True, ref=ref)
        except AssertionError as e:
            raise AssertionError(f"variant {v} {mdg.mdg_variant_info(v)['name']}: {e}") from None


def _variant_named(prefix):
    for d in mdg.variants():
        if d["name"].startswith(prefix):
            return d["id"]
    raise KeyError(prefix)


@pytest.mark.parametrize("prefix", ["direct_64x64", "direct_16x16", "tiled_128x128x16_w2x2_sk1", "tiled_32x32x32_w1x1_sk1",
                                    "tiled_32x32x32_w1x1_sk4", "tiled_32x32x64_w1x1x4_sk1", "tiled_64x64x32_w2x2x2_sk1",
                                    "skinny_nb4_sk1"])
def test_brute_force_tiny_shapes(prefix):
    # every combination of tiny sizes, all transposes, tight and padded leading dimensions
    gu = _gu()
    v = _variant_named(prefix)
    dims = (1, 2, 3, 5, 8, 16, 17)
    rng = np.random.default_rng(12)
    n = 0
    for M, N, K in itertools.product(dims, dims, dims):
        tA, tB = TT[n % 4]
        pad = int(rng.integers(0, 4))
        base = GemmCase(M, N, K, tA, tB, 1.25, 0.5 if n % 3 else 0.0, dist="smallint", c0="smallint",
                        seed=wl.case_seed(12, n), name=f"tiny/{M}x{N}x{K}").resolved()
        case = GemmCase(**{**base.__dict__, "lda": base.lda + pad, "ldb": base.ldb + pad, "ldc": base.ldc + pad})
        n += 1
        if v not in gu.legal_variants(case):
            continue
        st, got, A, B, C0 = gu.run_case(case, variant=v)
        assert st == 0
        gu.check_against_oracle(case, got, A, B, C0, exact=True)


@pytest.mark.parametrize("M,N,K", [(260, 16, 4096), (1027, 21, 2304), (64, 64, 4100), (512, 5, 8192), (4, 128, 300)])
def test_thin_matrix_core_variants_long_k(M, N, K):
    # K long enough for every wave to run its unguarded main loop (eight 16-byte loads in flight), rows and
    # columns that are / are not multiples of the 16-wide blocks, aligned (16-byte loads) and padded operands;
    # integer data, so every summation order must give the oracle's bits
    gu = _gu()
    thin = [d["id"] for d in mdg.variants() if d["name"].startswith("skinny_mfma")]
    assert len(thin) >= 2
    for i, (tA, tB) in enumerate(TT):
        for pad in ((0, 0, 0), (4, 8, 4), (1, 3, 2)):
            base = GemmCase(M, N, K, tA, tB, 1.5, (0.0, -0.5)[i % 2], dist="smallint", c0="smallint",
                            seed=wl.case_seed(15, 100 * i + M + N), name=f"thin/{M}x{N}x{K}/{tA}{tB}/{pad}").resolved()
            case = GemmCase(**{**base.__dict__, "lda": base.lda + pad[0], "ldb": base.ldb + pad[1], "ldc": base.ldc + pad[2]})
            A, B, C0 = wl.make_operands(case)
            ref = gu.oracle_result(case, A, B, C0)
            legal = gu.legal_variants(case)
            for v in thin:
                if v not in legal:
                    continue
                st, got, *_ = gu.run_case(case, variant=v)
                assert st == 0, (v, mdg.mdg_status_string(st))
                try:
                    gu.check_against_oracle(case, got, A, B, C0, exact=True, ref=ref)
                except AssertionError as e:
                    raise AssertionError(f"variant {mdg.mdg_variant_info(v)['name']}: {e}") from None


@pytest.mark.parametrize("layout", [CM, RM])
def test_special_scalars_degenerate_sizes_and_layouts(layout):
    gu = _gu()
    # beta = 0 with NaN in C: not read.  Through the selector and through a tiled and a direct variant.
    for variant in (None, 0, _variant_named("tiled_64x64x16_w2x2_sk1"), _variant_named("tiled_64x64x16_w2x2_sk4")):
        case = GemmCase(70, 90, 50, TR, NT, 1.0, 0.0, layout=layout, c0="nan", seed=5, name="beta0-nanC")
        st, got, A, B, C0 = gu.run_case(case, variant=variant)
        assert st == 0
        gu.check_against_oracle(case, got, A, B, C0)
    # alpha = 0 with NaN in A and B: not read; C = beta*C0
    case = GemmCase(70, 90, 50, NT, TR, 0.0, 0.5, layout=layout, dist="nan", seed=6, name="alpha0-nanAB")
    st, got, A, B, C0 = gu.run_case(case)
    assert st == 0
    gu.check_against_oracle(case, got, A, B, C0, exact=True)
    case = GemmCase(70, 90, 50, NT, TR, 0.0, 0.0, layout=layout, dist="nan", c0="nan", seed=6, name="alpha0-beta0")
    st, got, A, B, C0 = gu.run_case(case)
    gu.check_against_oracle(case, got, A, B, C0, exact=True)
    # K = 0, and beta = 1 (no scaling pass at all)
    for beta in (0.5, 1.0, 0.0):
        case = GemmCase(33, 21, 0, NT, NT, 1.0, beta, layout=layout, ldc=40, seed=7, name=f"K0-beta{beta}")
        st, got, A, B, C0 = gu.run_case(case)
        assert st == 0
        gu.check_against_oracle(case, got, A, B, C0, exact=True)
    # M = 0 / N = 0: success, nothing written
    for M, N in ((0, 5), (5, 0)):
        case = GemmCase(M, N, 4, layout=layout, beta=0.5, seed=8, name="empty")
        st, got, A, B, C0 = gu.run_case(case)
        assert st == 0 and np.array_equal(got, C0, equal_nan=True)
    # a row-major problem with both transposes and padded leading dimensions
    base = GemmCase(130, 75, 310, TR, TR, 1.5, -0.5, layout=layout, seed=9, name="TT-padded").resolved()
    case = GemmCase(**{**base.__dict__, "lda": base.lda + 3, "ldb": base.ldb + 2, "ldc": base.ldc + 4})
    for variant in [None] + gu.legal_variants(case)[::5]:
        st, got, A, B, C0 = gu.run_case(case, variant=variant)
        assert st == 0
        gu.check_against_oracle(case, got, A, B, C0)


def test_forced_variant_errors():
    gu = _gu()
    torch = gu.torch_mod()
    case = GemmCase(64, 64, 64, seed=1)
    skinny = _variant_named("skinny_nb1_sk1")
    st, *_ = gu.run_case(case, variant=skinny)
    assert st == mdg.ERR_ILLEGAL_VARIANT
    assert gu.run_case(case, variant=10 ** 6)[0] == mdg.ERR_BAD_VARIANT
    # without a workspace split-K variants are refused when forced, and replaced by variant 0 in mdg_sgemm
    sk = _variant_named("tiled_64x64x16_w2x2_sk4")
    assert mdg.mdg_set_workspace(0, 0) == 0
    try:
        assert gu.run_case(case, variant=sk)[0] == mdg.ERR_WORKSPACE
        assert mdg.mdg_variant_legal(sk, 0, 0, 64, 64, 64, 64, 64, 64) == 0
        st, got, A, B, C0 = gu.run_case(case)
        assert st == 0
        gu.check_against_oracle(case, got, A, B, C0)
    finally:
        ws = gu._WS["t"]
        assert mdg.mdg_set_workspace(ws.data_ptr(), ws.numel() * 4) == 0
    t = torch.empty(1024, dtype=torch.float32, device="cuda")
    assert mdg.mdg_set_workspace(t.data_ptr() + 4, 1024) != 0  # misaligned workspace refused


def test_non_default_stream_and_repeatability():
    gu = _gu()
    torch = gu.torch_mod()
    case = GemmCase(300, 200, 700, NT, TR, 1.0, 0.5, seed=13).resolved()
    A, B, C0 = wl.make_operands(case)
    s = torch.cuda.Stream()
    outs = []
    for rep in range(2):
        dA, dB, dC = (torch.from_numpy(x).cuda() for x in (A, B, C0))
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            st = mdg.mdg_sgemm(case.layout, case.transA, case.transB, case.M, case.N, case.K, case.alpha, dA.data_ptr(),
                               case.lda, dB.data_ptr(), case.ldb, case.beta, dC.data_ptr(), case.ldc, s.cuda_stream)
        assert st == 0
        s.synchronize()
        outs.append(dC.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])  # deterministic: no atomics anywhere
    gu.check_against_oracle(case, outs[0], A, B, C0)


def test_split_k_is_repeatable_and_exact():
    # K slices are added in slice order by the reduce pass: many back-to-back calls on one stream
    # (the workspace is re-used every time) must give bit-identical, oracle-exact results on integer data
    gu = _gu()
    torch = gu.torch_mod()
    case = GemmCase(300, 200, 1100, NT, TR, 1.0, 0.0, dist="smallint", c0="zero", seed=wl.case_seed(14, 0),
                    name="splitk-repeat").resolved()
    A, B, C0 = wl.make_operands(case)
    ref = gu.oracle_result(case, A, B, C0)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    for v in gu.legal_variants(case):
        d = mdg.mdg_variant_info(v)
        if d["family"] != mdg.FAMILY_TILED or d["split_k"] == 1:
            continue
        outs = [torch.from_numpy(C0).cuda() for _ in range(12)]
        for dC in outs:  # no synchronisation in between
            st = mdg.mdg_sgemm_variant(v, case.layout, case.transA, case.transB, case.M, case.N, case.K, case.alpha,
                                       dA.data_ptr(), case.lda, dB.data_ptr(), case.ldb, case.beta, dC.data_ptr(),
                                       case.ldc, stream)
            assert st == 0
        torch.cuda.synchronize()
        for dC in outs:
            assert np.array_equal(dC.cpu().numpy(), ref), d["name"]


@pytest.mark.parametrize("tA,tB", TT)
def test_indirect_variants_pack_pad_and_match_the_oracle(tA, tB):
    # the helper passes must zero-fill the padding they add, must not read the (NaN-poisoned) padding of the
    # caller's leading dimensions, and an operand that already has the packed form is used where it lies
    gu = _gu()
    ind = [d for d in mdg.variants() if d["family"] == mdg.FAMILY_INDIRECT]
    assert len(ind) >= 3
    for d in ind:
        bm, bn, bk = d["tile_m"], d["tile_n"], d["tile_k"]
        shapes = [(2 * max(bm, 64), max(bn, 64), 3 * bk, 0),           # whole tiles: NT needs no copy at all
                  (2 * max(bm, 64) - 5, max(bn, 64) + 3, 3 * bk + 1, 3),  # ragged in M, N and K, padded leading dimensions
                  (7, 5, 3, 1), (1, 300, 70, 0)]
        for M, N, K, pad in shapes:
            base = GemmCase(M, N, K, tA, tB, 1.5, -0.5, dist="smallint", c0="smallint",
                            seed=wl.case_seed(16, M + N + K), name=f"indirect/{d['name']}/{M}x{N}x{K}/{tA}{tB}").resolved()
            case = GemmCase(**{**base.__dict__, "lda": base.lda + pad, "ldb": base.ldb + pad, "ldc": base.ldc + pad})
            assert d["id"] in gu.legal_variants(case)
            st, got, A, B, C0 = gu.run_case(case, variant=d["id"])
            assert st == 0, (d["name"], mdg.mdg_status_string(st))
            gu.check_against_oracle(case, got, A, B, C0, exact=True)
    # without a workspace a transposed operand cannot be packed: refused when forced, replaced by the plain tile in mdg_sgemm
    case = GemmCase(300, 200, 100, TR, NT, 1.0, 0.0, seed=3).resolved()
    assert mdg.mdg_set_workspace(0, 0) == 0
    try:
        assert gu.run_case(case, variant=ind[0]["id"])[0] == mdg.ERR_WORKSPACE
    finally:
        ws = gu._WS["t"]
        assert mdg.mdg_set_workspace(ws.data_ptr(), ws.numel() * 4) == 0


@pytest.mark.parametrize("tA,tB", TT)
def test_interior_loop_of_every_tiled_and_indirect_variant_is_exact(tA, tB):
    # aligned operands with whole tiles and a long K: the lean interior loop (vector loads, direct-to-LDS loads,
    # every lane arrangement) does all the work; integer data, so the oracle's bits are the only right answer.
    # A second case breaks the alignment (leading dimensions + 1), which direct-to-LDS variants must refuse.
    gu = _gu()
    base = GemmCase(512, 768, 416, tA, tB, 1.0, 0.5, dist="smallint", c0="smallint", seed=wl.case_seed(17, 2 * tA + tB),
                    name=f"interior/{tA}{tB}").resolved()
    odd = GemmCase(**{**base.__dict__, "lda": base.lda + 1, "ldb": base.ldb + 1, "name": base.name + "/odd-ld"})
    n_direct = 0
    for case in (base, odd):
        A, B, C0 = wl.make_operands(case)
        ref = gu.oracle_result(case, A, B, C0)
        legal = gu.legal_variants(case)
        for d in mdg.variants():
            if d["family"] not in (mdg.FAMILY_TILED, mdg.FAMILY_INDIRECT) or d["split_k"] > 4:
                continue
            if d["lds"] == 2 and case is odd and (tA == NT or tB == TR):
                assert d["id"] not in legal, d["name"]  # an unaligned row-contiguous operand: not for direct loads
                continue
            assert d["id"] in legal, d["name"]
            n_direct += d["lds"] == 2
            st, got, *_ = gu.run_case(case, variant=d["id"])
            assert st == 0, (d["name"], mdg.mdg_status_string(st))
            try:
                gu.check_against_oracle(case, got, A, B, C0, exact=True, ref=ref)
            except AssertionError as e:
                raise AssertionError(f"{d['name']}: {e}") from None
    assert n_direct >= 2


@pytest.mark.parametrize("tA,tB", TT)
def test_operands_shorter_than_the_tile_are_exact(tA, tB):
    # M and N below every large tile with a long K: tiles whose operand ends inside them stand in its last rows
    # for the missing ones in the interior loop (a multiple of four rows, or k-contiguous rows) and take guarded
    # loads otherwise (M = 30); what the stand-ins produce must never reach C.  Every legal variant, split-K
    # included, with beta != 0 and integer data: the oracle's bits are the only right answer.
    gu = _gu()
    for M, N, K in ((100, 20, 1312), (30, 52, 1312), (20, 7, 2560)):
        case = GemmCase(M, N, K, tA, tB, 1.0, 0.5, dist="smallint", c0="smallint",
                        seed=wl.case_seed(18, 2 * tA + tB), name=f"short/{M}x{N}x{K}/{tA}{tB}").resolved()
        A, B, C0 = wl.make_operands(case)
        ref = gu.oracle_result(case, A, B, C0)
        n_split = 0
        for v in gu.legal_variants(case):
            d = mdg.variants()[v]
            st, got, *_ = gu.run_case(case, variant=v)
            assert st == 0, (d["name"], mdg.mdg_status_string(st))
            n_split += d["split_k"] > 1
            try:
                gu.check_against_oracle(case, got, A, B, C0, exact=True, ref=ref)
            except AssertionError as e:
                raise AssertionError(f"{d['name']}: {e}") from None
        assert n_split >= 10
