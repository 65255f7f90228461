"""GPU parity on the named workloads, every case, element by element against the fp64 oracle (Eq. 1, Section 2.2).

Every call goes through mdg_sgemm -- validation, compiled selector, legality / fallback, kernel -- exactly as the
benchmark issues it:
  * the square sweep: all 24 cases (256 ... 8192, four transpose combinations), the whole of C compared;
  * the skinny sweep: all 144 cases;
  * the convolution-lowered sweep: all 75 cases;
  * the held-out fifth of the random sweep (Section 3, 'Datasets'): all 400 cases with their own alpha / beta /
    transposes, and every tenth of them also through every variant that is legal for it.
Bar: |C - C_ref| <= 1e-6*K*max|a|*max|b| + 1e-6*|beta*C0| for every element, and nothing outside the logical
region of C is written.
"""
import numpy as np
import pytest

from paper_1806_07060_amd import binding as mdg
from paper_1806_07060_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _workspace():
    from tests import gpu_util as gu
    gu.ensure_workspace(1 << 30)
    yield


def _check(case, variants=(None,)):
    from tests import gpu_util as gu
    A, B, C0, outs = gu.run_case_many(case, variants)
    ref = gu.oracle_result(case, A, B, C0)
    for v, (st, got) in zip(variants, outs):
        name = "selector" if v is None else mdg.mdg_variant_info(v)["name"]
        assert st == 0, (case.name, name, mdg.mdg_status_string(st))
        try:
            gu.check_against_oracle(case, got, A, B, C0, ref=ref)
        except AssertionError as e:
            raise AssertionError(f"{name}: {e}") from None


_SQUARE = wl.config1()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("idx", range(len(_SQUARE)), ids=[c.name for c in _SQUARE])
def test_square_sweep_every_case_whole_matrix(idx):
    from oracle import gemm_oracle as go
    from tests import gpu_util as gu
    case = _SQUARE[idx]
    c = case.resolved()
    if not (c.tA() and c.tB() and c.M >= 2048):
        _check(case)
        return
    # Both operands transposed: the oracle then runs a dot product per element and walks B with a stride of a
    # whole column, which takes twenty times as long as the other cases at these sizes.  It is handed a
    # transposed copy of B with transB = none instead: op(B)(k, j) is the same number either way, every element
    # is the same sum in the same order, so oracle_sgemm returns the same bits (the identity is one of the
    # oracle's own pins).  The GPU still gets the original operands and both transposes.
    assert c.layout == wl.COL_MAJOR and c.ldb == c.N
    A, B, C0, outs = gu.run_case_many(c, [None])
    st, got = outs[0]
    assert st == 0, mdg.mdg_status_string(st)
    Bt = np.ascontiguousarray(B.reshape(c.K, c.N).T).ravel()  # stored N x K (ld N)  ->  stored K x N (ld K)
    ref = C0.copy()
    assert go.sgemm(c.layout, c.transA, wl.NO_TRANS, c.M, c.N, c.K, c.alpha, A, c.lda, Bt, c.K, c.beta, ref, c.ldc) == 0
    gu.check_against_oracle(c, got, A, B, C0, ref=ref)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("part", range(4))
def test_skinny_sweep_every_case(part):
    cases = wl.config2()
    assert len(cases) == 144
    for case in cases[part::4]:
        _check(case)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("part", range(5))
def test_convolution_lowered_sweep_every_case(part):
    cases = wl.config3()
    assert len(cases) == 75
    for case in cases[part::5]:
        _check(case)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("part", range(4))
def test_held_out_random_sweep_every_case_and_every_legal_variant_of_each_tenth(part):
    from tests import gpu_util as gu
    _, held = wl.split_train_heldout(wl.config4())
    assert len(held) == 400
    for i in range(part, len(held), 4):
        case = held[i]
        variants = [None]
        if i % 10 == 0:
            variants += gu.legal_variants(case)
        _check(case, variants)
