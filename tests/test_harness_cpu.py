"""The tuning harness's bookkeeping (pruning, second probe, extend and recheck modes) with a fake timer. CPU only."""
import math

import numpy as np
import pytest

from paper_1806_07060_amd import workloads as wl
from paper_1806_07060_amd.tuning import harness


class FakePools:
    class _T:
        def data_ptr(self):
            return 4096
    A = B = C = _T()

    def layout(self, case):
        return 1, 64, 64, 64


@pytest.fixture
def fake(monkeypatch):
    """Variants 0..3 all legal; `times[v]` is the true time, `first_call_penalty[v]` is added to the first single-call probe."""
    state = {"times": [10e-6, 2e-6, 50e-6, 3e-6], "penalty": [0, 0, 0, 0], "calls": []}

    def time_variant(v, case, pools, n_sets, sa, sb, sc, stream, warmup, reps, spans):
        state["calls"].append((v, warmup, reps, spans))
        t = state["times"][v]
        if reps == 1 and state["penalty"][v]:
            t += state["penalty"][v]
            state["penalty"][v] = 0
        return t

    monkeypatch.setattr(harness, "time_variant", time_variant)
    monkeypatch.setattr(harness.mdg, "mdg_variant_legal", lambda *a, **k: 1)
    return state


VARIANTS = [{"id": i, "family": 1 if i else 0, "name": f"v{i}"} for i in range(4)]
CASE = wl.GemmCase(64, 64, 64)


def test_slow_variants_are_recorded_from_probes_fast_ones_measured_fully(fake):
    out = harness.measure_case(CASE, FakePools(), 0, VARIANTS, span_ms=1.0, spans=3, prune=6.0)
    assert out.tolist() == fake["times"]
    full = [c for c in fake["calls"] if c[2] > 1]
    assert {c[0] for c in full} == {0, 1, 3}  # 50 us > 6 x 2 us: variant 2 is only probed (twice: second opinion)
    assert [c for c in fake["calls"] if c[0] == 2] == [(2, 1, 1, 1), (2, 1, 1, 1)]
    reps = {c[0]: c[2] for c in full}
    assert reps[1] == min(200, math.ceil(1e-3 / 2e-6)) and reps[0] == 100


def test_a_cold_first_probe_does_not_get_a_good_variant_pruned(fake):
    fake["penalty"][3] = 40e-6  # first launch of this kernel symbol is slow once
    out = harness.measure_case(CASE, FakePools(), 0, VARIANTS)
    assert out[3] == 3e-6 and (3, 1, 1, 1) in fake["calls"] and any(c[0] == 3 and c[2] > 1 for c in fake["calls"])


def test_known_times_are_kept_and_not_measured_again(fake):
    out = harness.measure_case(CASE, FakePools(), 0, VARIANTS, known={1: 2.5e-6, 2: math.inf})
    assert out[1] == 2.5e-6 and math.isinf(out[2])
    assert {c[0] for c in fake["calls"]} == {0, 3}


def test_recheck_only_touches_short_probe_only_entries(fake):
    row = [10e-6, 2e-6, 50e-6, 30e-6]  # variant 3 was recorded from a cold probe; its true time is 3 us
    out, changed = harness.recheck_case(CASE, FakePools(), 0, VARIANTS, row, prune=6.0)
    assert changed == 1 and out.tolist() == [10e-6, 2e-6, 50e-6, 3e-6]
    assert {c[0] for c in fake["calls"]} == {2, 3}  # entries within 6 x best are left alone
    # long entries (>= 1 ms) are never rechecked
    fake["calls"].clear()
    out, changed = harness.recheck_case(CASE, FakePools(), 0, VARIANTS, [10e-6, 2e-6, 5e-3, 3e-6])
    assert changed == 0 and fake["calls"] == []


def test_every_configuration_index_yields_resolved_column_major_cases():
    for cfg in range(12):
        if cfg in (5,):
            continue  # 3375 cases: covered by the size check below
        cases = harness.cases_for(cfg)
        assert cases and all(c.layout == wl.COL_MAJOR and c.lda >= 1 and c.ldb >= 1 and c.ldc >= 1 for c in cases[:50])
    assert len(harness.cases_for(5)) == 3375
    with pytest.raises(ValueError):
        harness.cases_for(99)


def test_training_set_generators_are_seeded_capped_and_cover_their_corners():
    # sizes and caps of the synthetic training sets the tuning run measures (recipes, not measured data)
    thin, flat = wl.config_thin(), wl.config_flat()
    assert len(thin) == 1000 and len(flat) == 1200
    assert all(1 <= c.N <= 64 and 256 <= c.M <= 16384 and 256 <= c.K <= 8192 for c in thin)
    assert all(16 <= c.M <= 512 and 1024 <= c.N <= 65536 and 16 <= c.K <= 4096 for c in flat)
    tg, fg = wl.config_thin_grid(), wl.config_flat_grid()
    assert (len(tg), len(fg)) == (1144, 1302)
    grid = wl._geometric_grid(16, 128)
    assert grid == [16, 24, 32, 48, 64, 96, 128]
    assert {c.N for c in tg} == {1, 2, 4, 8, 16, 32, 64, 128} and {c.M for c in fg} == {16, 32, 64, 128, 256, 512}
    for cases in (thin, flat, tg, fg):
        assert all(2 * c.M * c.N * c.K <= 2 ** 38 and 4 * max(c.M * c.K, c.K * c.N, c.M * c.N) <= 6e8 for c in cases)
        assert len({c.name for c in cases}) == len({(c.M, c.N, c.K) for c in cases})
    # prefix-stable: a longer sweep starts with the shorter one (tables are extended, never re-measured)
    assert [(c.M, c.N, c.K, c.transA, c.alpha) for c in wl.config_thin(50)] == [(c.M, c.N, c.K, c.transA, c.alpha) for c in thin[:50]]
    # seeded: two calls give the same cases
    assert [(c.M, c.N, c.K, c.transA, c.transB, c.alpha, c.beta) for c in wl.config_flat_grid()] == \
        [(c.M, c.N, c.K, c.transA, c.transB, c.alpha, c.beta) for c in fg]
    assert harness.cases_for(12)[0].name == tg[0].name and harness.cases_for(13)[-1].name == fg[-1].name


def test_second_sweeps_repeat_the_recipes_of_the_first_from_streams_of_their_own():
    first, second = wl.config4(), wl.config_sweep2()
    assert (len(first), len(second)) == (2000, 4000)
    assert all(1 <= min(c.M, c.N, c.K) and max(c.M, c.N, c.K) <= 8192 and 2 * c.M * c.N * c.K <= 2 ** 32 for c in second)
    key = lambda c: (c.M, c.N, c.K, c.transA, c.transB)
    assert len({key(c) for c in second} & {key(c) for c in first}) < 40  # another stream: only tiny shapes coincide
    assert second[0].name.startswith("sweep2/") and first[0].name.startswith("cfg4/")
    assert [key(c) for c in wl.config_sweep2()] == [key(c) for c in second]
    thin2, flat2 = wl.config_thin2(), wl.config_flat2()
    assert len(thin2) == 2000 and len(flat2) == 2000
    assert all(1 <= c.N <= 64 and 256 <= c.M <= 16384 and 256 <= c.K <= 8192 for c in thin2)
    assert all(16 <= c.M <= 512 and 1024 <= c.N <= 65536 and 16 <= c.K <= 4096 for c in flat2)
    assert [key(c) for c in thin2[:100]] != [key(c) for c in wl.config_thin()[:100]]
    assert harness.cases_for(14)[0].name == second[0].name and harness.cases_for(16)[-1].name == flat2[-1].name
    third = wl.config_sweep3()
    assert len(third) == 8000 and third[0].name.startswith("sweep3/")
    assert len({key(c) for c in third} & {key(c) for c in second}) < 80
    assert len(wl.config_thin3()) == 2000 and len(wl.config_flat3()) == 2000
    assert [key(c) for c in wl.config_thin3()[:100]] != [key(c) for c in thin2[:100]]
    assert harness.cases_for(17)[-1].name == third[-1].name and harness.cases_for(19)[0].name == wl.config_flat3()[0].name
    # the denser thin grid adds midpoints of N and quarter octaves of M, and repeats nothing of the first grid
    tg, tg2 = wl.config_thin_grid(), wl.config_thin_grid2()
    assert len(tg2) == 1854 and not {(c.M, c.N, c.K) for c in tg2} & {(c.M, c.N, c.K) for c in tg}
    assert {3, 6, 12, 24, 48, 96} <= {c.N for c in tg2} and {640, 896, 7168, 14336} <= {c.M for c in tg2}
    assert max(c.M for c in tg2) == 16384 and harness.cases_for(20)[0].name == tg2[0].name
