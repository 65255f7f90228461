"""Host-side checks of the C-ABI library that need no GPU: exports, variant table, validation, legality, selection."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1806_07060_amd import binding as mdg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mdg_sgemm.h")).read()
    declared = set(re.findall(r"\b(mdg_[a-z_]+)\s*\(", header))
    assert declared == set(mdg.EXPORTS)
    L = ctypes.CDLL(mdg.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


def test_variant_table_is_consistent():
    vs = mdg.variants()
    assert len(vs) == mdg.mdg_variant_count() >= 20
    assert len({v["name"] for v in vs}) == len(vs)
    assert vs[0]["family"] == mdg.FAMILY_DIRECT and vs[0]["split_k"] == 1
    fams = {v["family"] for v in vs}
    assert fams == {mdg.FAMILY_DIRECT, mdg.FAMILY_TILED, mdg.FAMILY_SKINNY, mdg.FAMILY_INDIRECT}
    for v in vs:
        assert v["id"] == vs.index(v)
        assert v["threads"] in (64, 128, 256, 512, 1024) and v["split_k"] >= 1
        if v["family"] == mdg.FAMILY_TILED:
            assert v["tile_m"] % v["sub_m"] == 0 and v["sub_m"] in (32, 64, 128)
            # threads = 64 x waves over the tile x wave groups that split each K step
            waves = (v["tile_m"] // v["sub_m"]) * (v["tile_n"] // v["sub_n"])
            assert v["threads"] % (64 * waves) == 0
            wgk = v["threads"] // (64 * waves)
            assert v["tile_k"] % wgk == 0 and (v["tile_k"] // wgk) % 2 == 0
            if wgk > 1:
                assert f"x{wgk}_sk{v['split_k']}" in v["name"]
    with pytest.raises(ValueError):
        mdg.mdg_variant_info(len(vs))


def test_fallback_chains_end_at_variant_zero_and_only_relax_the_variant():
    vs = mdg.variants()
    for v in vs:
        seen, x = set(), v
        while x["id"] != 0:
            assert x["id"] not in seen and len(seen) < len(vs), "cycle in fallback links"
            seen.add(x["id"])
            nxt = vs[x["fallback"]]
            if x["family"] == mdg.FAMILY_TILED and x["split_k"] > 1:  # fewer K slices of the same tile
                assert nxt["family"] == x["family"] and nxt["split_k"] < x["split_k"]
                assert (nxt["tile_m"], nxt["tile_n"], nxt["tile_k"]) == (x["tile_m"], x["tile_n"], x["tile_k"])
            elif x["family"] == mdg.FAMILY_TILED and x["lds"] == 2:  # the same tile with loads through registers
                assert nxt["family"] == mdg.FAMILY_TILED and nxt["split_k"] == 1 and nxt["lds"] == 1
                assert (nxt["tile_m"], nxt["tile_n"], nxt["tile_k"], nxt["threads"]) == (x["tile_m"], x["tile_n"], x["tile_k"], x["threads"])
            elif x["family"] == mdg.FAMILY_INDIRECT:  # the same tile without the helper passes
                assert nxt["family"] == mdg.FAMILY_TILED and nxt["split_k"] == 1
                assert (nxt["tile_m"], nxt["tile_n"], nxt["tile_k"]) == (x["tile_m"], x["tile_n"], x["tile_k"])
            elif x["family"] == mdg.FAMILY_SKINNY:  # wider with the same split, else fewer slices, else a tile
                assert (nxt["family"] == mdg.FAMILY_SKINNY and nxt["sub_n"] > x["sub_n"] and nxt["split_k"] == x["split_k"]) or \
                       (nxt["family"] == mdg.FAMILY_SKINNY and nxt["sub_n"] >= x["sub_n"] and nxt["split_k"] < x["split_k"]) or \
                       (nxt["family"] == mdg.FAMILY_TILED and nxt["split_k"] == 1)
            else:
                assert nxt["id"] == 0
            x = nxt
    assert vs[0]["fallback"] == 0


def test_argument_validation_reports_first_bad_argument():
    ok = dict(layout=102, transA=111, transB=111, M=4, N=4, K=4, alpha=1.0, A=256, lda=4, B=256, ldb=4, beta=0.0,
              C=256, ldc=4)

    def call(**kw):
        d = dict(ok)
        d.update(kw)
        return mdg.mdg_sgemm(**d)

    assert call(layout=0) == -1
    assert call(transA=110) == -2
    assert call(transB=0) == -3
    assert call(M=-1) == -4
    assert call(N=-2) == -5
    assert call(K=-3) == -6
    assert call(M=2 ** 31) == -4
    # the documented limit: the kernels add a tile or a K slice to a dimension in 32-bit arithmetic
    assert call(M=mdg.MAX_DIM + 1, lda=mdg.MAX_DIM + 1, ldc=mdg.MAX_DIM + 1) == -4
    assert call(N=mdg.MAX_DIM + 1) == -5 and call(K=mdg.MAX_DIM + 1, ldb=mdg.MAX_DIM + 1) == -6
    assert mdg.MAX_DIM == 2 ** 31 - 1 - 65536
    assert call(A=0) == -8
    assert call(lda=3) == -9
    assert call(B=0) == -10
    assert call(ldb=3) == -11
    assert call(C=0) == -13
    assert call(ldc=3) == -14
    assert call(transA=112, M=8, K=2, lda=1, ldc=8) == -9
    assert call(layout=101, M=2, N=8, K=4, ldb=7, ldc=8) == -11
    assert call(layout=101, M=2, N=8, K=4, ldb=8, ldc=7) == -14
    # nothing to do: returns before touching the GPU
    assert call(M=0, lda=1, ldc=1) == 0
    assert call(N=0) == 0
    # alpha == 0 never reads A or B, so NULL is fine there -- but that would launch; only validate
    assert "ldc" in mdg.mdg_status_string(-14) and mdg.mdg_status_string(0) == "ok"
    assert mdg.mdg_sgemm_variant(-1, **ok) == mdg.ERR_BAD_VARIANT


def test_legality_rules():
    vs = mdg.variants()
    n = len(vs)
    # variant 0 is legal for anything (soundness): odd sizes, unaligned pointers, huge N
    for M, N, K in ((1, 1, 1), (7, 3, 1), (8191, 5, 13), (1, mdg.MAX_DIM, 1), (mdg.MAX_DIM, 1, 1)):
        assert mdg.mdg_variant_legal(0, 1, 0, M, N, K, K, K, M, 4, 4, 4) == 1
    assert mdg.mdg_variant_legal(0, 1, 0, mdg.MAX_DIM + 1, 1, 1, 1, 1, mdg.MAX_DIM + 1, 4, 4, 4) == 0
    assert mdg.mdg_variant_legal(n, 0, 0, 1, 1, 1, 1, 1, 1) == mdg.ERR_BAD_VARIANT
    mdg.mdg_set_workspace(0, 0)
    for v in vs:
        need = mdg.mdg_workspace_bytes(v["id"], 100, 50, 4096)
        if v["family"] == mdg.FAMILY_INDIRECT:  # padded copies of both operands (see the test of the indirect variants)
            assert need > 4 * (100 + 50) * 4096
            continue
        assert need == (v["split_k"] * 100 * 50 * 4 if v["split_k"] > 1 else 0)
        if v["split_k"] > 1:
            assert mdg.mdg_variant_legal(v["id"], 0, 0, 100, 4, 4096, 100, 4096, 100) == 0  # no workspace registered
        if v["family"] == mdg.FAMILY_SKINNY:
            assert mdg.mdg_variant_legal(v["id"], 0, 0, 100, 4 * v["sub_n"] + 1, 64, 100, 64, 100) == 0
    # a fake (never dereferenced) workspace makes split-K legal when every slice owns a K step
    assert mdg.mdg_set_workspace(1 << 20, 1 << 30) == 0
    try:
        for v in vs:
            if v["split_k"] > 1 and v["family"] == mdg.FAMILY_TILED:
                kmin = v["split_k"] * v["tile_k"]
                assert mdg.mdg_variant_legal(v["id"], 0, 0, 64, 64, kmin, 64, kmin, 64) == 1
                assert mdg.mdg_variant_legal(v["id"], 0, 0, 64, 64, kmin - v["tile_k"], 64, kmin, 64) == 0
    finally:
        mdg.mdg_set_workspace(0, 0)
    assert mdg.mdg_set_workspace(12, 1024) != 0  # unaligned


def test_selectors_return_valid_ids_everywhere():
    n = mdg.mdg_variant_count()
    assert isinstance(mdg.mdg_selector_name(), str)
    for M in (1, 2, 63, 64, 65, 1000, 4096, 8192):
        for N in (1, 17, 512, 8192):
            for K in (1, 27, 1024, 8192):
                for tA in (0, 1):
                    for tB in (0, 1):
                        assert 0 <= mdg.mdg_select(tA, tB, M, N, K) < n
                        assert 0 <= mdg.mdg_select_default(tA, tB, M, N, K) < n
    ns = mdg.mdg_time_select_ns([0, 1], [1, 0], [64, 4096], [64, 4096], [64, 4096], iters=1000)
    assert 0 < ns < 1e5


def test_the_memo_in_front_of_the_model_returns_what_the_model_returns():
    # mdg_sgemm asks mdg_select_memo; it must agree with the model for fresh shapes, repeated shapes and shapes
    # that push each other out of the 1024-entry table
    rng = np.random.default_rng(31)
    shapes = np.column_stack([np.rint(2.0 ** (13 * rng.uniform(size=(3000, 3)))).astype(np.int64),
                              rng.integers(0, 2, size=(3000, 2))])
    order = np.concatenate([np.arange(3000), rng.integers(0, 3000, 6000), np.repeat(np.arange(40), 5)])
    for i in order:
        M, N, K, tA, tB = (int(x) for x in shapes[i])
        assert mdg.mdg_select_memo(tA, tB, M, N, K) == mdg.mdg_select(tA, tB, M, N, K)
    # same sizes, different transposes are different keys
    for tA in (0, 1):
        for tB in (0, 1):
            assert mdg.mdg_select_memo(tA, tB, 777, 33, 2049) == mdg.mdg_select(tA, tB, 777, 33, 2049)
    X = shapes[:64]
    assert mdg.mdg_time_select_ns(X[:, 3], X[:, 4], X[:, 0], X[:, 1], X[:, 2], iters=3, memo=True) > 0


def test_first_calls_from_many_threads_agree():
    # the variant table is built on first use: concurrent first calls from several threads must all see the
    # finished table (a fresh process, so that no earlier test has built it already)
    import subprocess
    import sys
    code = r'''
import sys, threading
sys.path.insert(0, %r)
from paper_1806_07060_amd import binding as mdg
L = mdg.lib()
n = 16
out = [None] * n
go = threading.Barrier(n)
def work(i):
    go.wait()
    rows = []
    for v in range(mdg.mdg_variant_count()):
        d = mdg.mdg_variant_info(v)
        rows.append((d["name"], d["fallback"], d["split_k"], mdg.mdg_variant_legal(v, 0, 0, 300, 40, 5000, 300, 5000, 300)))
    rows.append(mdg.mdg_select(i & 1, 0, 100 + i, 200, 300))
    out[i] = rows
ts = [threading.Thread(target=work, args=(i,)) for i in range(n)]
[t.start() for t in ts]
[t.join() for t in ts]
assert all(o is not None and o[:-1] == out[0][:-1] for o in out)
assert all(0 <= f < len(out[0]) - 1 for _, f, _, _ in out[0][:-1])
print("ok")
''' % ROOT
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stderr


def test_workspace_registration_errors_have_their_own_code():
    assert mdg.mdg_set_workspace(4096 + 4, 1 << 20) == mdg.ERR_ALIGNMENT
    assert "aligned" in mdg.mdg_status_string(mdg.ERR_ALIGNMENT)
    assert mdg.mdg_set_workspace(4096, 1 << 20) == 0  # host code only stores the pair; nothing is dereferenced
    sk = next(d["id"] for d in mdg.variants() if d["split_k"] == 4 and d["family"] == mdg.FAMILY_TILED)
    assert mdg.mdg_variant_legal(sk, 0, 0, 128, 128, 4096, 128, 4096, 128) == 1
    assert mdg.mdg_set_workspace(0, 0) == 0
    assert mdg.mdg_variant_legal(sk, 0, 0, 128, 128, 4096, 128, 4096, 128) == 0


def test_direct_to_lds_variants_demand_aligned_row_contiguous_operands():
    vs = [v for v in mdg.variants() if v["family"] == mdg.FAMILY_TILED and v["lds"] == 2]
    assert len(vs) >= 2
    for v in vs:
        i = v["id"]
        # A not transposed: lda and the pointer must keep 16-byte alignment; a transposed A goes through registers
        assert mdg.mdg_variant_legal(i, 0, 0, 512, 512, 512, 512, 512, 512, 4096, 4096, 4096) == 1
        assert mdg.mdg_variant_legal(i, 0, 0, 512, 512, 512, 513, 512, 512, 4096, 4096, 4096) == 0
        assert mdg.mdg_variant_legal(i, 0, 0, 512, 512, 512, 512, 512, 512, 4100, 4096, 4096) == 0
        assert mdg.mdg_variant_legal(i, 1, 0, 512, 512, 512, 513, 513, 512, 4100, 4100, 4096) == 1
        # B transposed: the same for ldb and B
        assert mdg.mdg_variant_legal(i, 1, 1, 512, 512, 512, 513, 512, 512, 4100, 4096, 4096) == 1
        assert mdg.mdg_variant_legal(i, 1, 1, 512, 512, 512, 512, 514, 512, 4096, 4096, 4096) == 0
        assert mdg.mdg_variant_legal(i, 1, 1, 512, 512, 512, 512, 512, 512, 4096, 4104, 4096) == 0


def test_indirect_variants_need_workspace_for_the_packed_copies_only():
    vs = mdg.variants()
    ind = [v for v in vs if v["family"] == mdg.FAMILY_INDIRECT]
    assert len(ind) >= 3
    for v in ind:
        bm, bn, bk = v["tile_m"], v["tile_n"], v["tile_k"]
        qm, qn = max(bm, 64), max(bn, 64)
        M, N, K = 3 * qm, 2 * qn, 5 * bk
        assert mdg.mdg_set_workspace(0, 0) == 0
        # operands already in packed form (A not transposed, B transposed, whole tiles): no copy, no workspace
        assert mdg.mdg_variant_legal(v["id"], 0, 1, M, N, K, M, N, M) == 1
        # a transposed A must be copied: illegal without workspace, legal with enough of it
        assert mdg.mdg_variant_legal(v["id"], 1, 1, M, N, K, K, N, M) == 0
        assert mdg.mdg_set_workspace(4096, 4 * M * K) == 0
        assert mdg.mdg_variant_legal(v["id"], 1, 1, M, N, K, K, N, M) == 1
        assert mdg.mdg_variant_legal(v["id"], 1, 0, M, N, K, K, K, M) == 0  # now B needs a copy as well
        # ragged sizes are padded to whole tiles (and to multiples of 64 for the transposing helper)
        Mr, Nr, Kr = M - 1, N - 3, K - 1
        need = 4 * (M * K + N * K)
        assert mdg.mdg_workspace_bytes(v["id"], Mr, Nr, Kr) == need
        assert mdg.mdg_set_workspace(4096, need - 4) == 0
        assert mdg.mdg_variant_legal(v["id"], 0, 1, Mr, Nr, Kr, Mr, Nr, Mr) == 0
        assert mdg.mdg_set_workspace(4096, need) == 0
        assert mdg.mdg_variant_legal(v["id"], 0, 1, Mr, Nr, Kr, Mr, Nr, Mr) == 1
    assert mdg.mdg_set_workspace(0, 0) == 0
