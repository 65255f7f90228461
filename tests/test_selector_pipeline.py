"""Parity of the product's off-line pipeline (numpy CART, metrics, code generator) with the selector oracle. CPU only.

Integer work (labels, tree structure, predictions, generated code) must agree exactly; the ratio metrics to
rounding error.  Inputs are seeded synthetic timing tables (no measured data is involved here).
"""
import ctypes
import json
import os
import subprocess

import numpy as np
import pytest

from oracle import selector_oracle as so
from paper_1806_07060_amd import workloads as wl
from paper_1806_07060_amd.tuning import cart, codegen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _table(n, v, seed):
    feats, times = wl.synthetic_timing_table(n, v, seed)
    # product side: raw [n, 5] inputs (it expands them itself); oracle side: tuples expanded by the oracle's own rule
    return feats, times, [so.expand_features(tuple(int(a) for a in r)) for r in feats], [list(map(float, r)) for r in times]


def _probe(feature, value, base=(64, 64, 64, 0, 1)):
    """A raw input (M, N, K, tA, tB) whose tree feature `feature` equals `value` (products via N = K = 1)."""
    p = list(base)
    if feature < 5:
        p[feature] = value
    elif feature == 5:
        p[0], p[1] = value, 1
    elif feature == 6:
        p[0], p[1], p[2] = value, 1, 1
    else:  # tile-fit features: padM32/64/128 (7-9), padN32/64/128 (10-12) = (t - X mod t) mod t
        t = (32, 64, 128)[(feature - 7) % 3]
        p[0 if feature < 10 else 1] = 3 * t - (value % t)
    return tuple(p)


@pytest.mark.parametrize("seed,n,v", [(1, 200, 8), (2, 320, 14)])
def test_labels_and_trees_are_identical_to_the_oracle(seed, n, v):
    X, T, Xl, Tl = _table(n, v, seed)
    assert cart.labels_from_table(T).tolist() == so.labels_from_table(Tl)
    y = so.labels_from_table(Tl)
    for rule in ("majority", "logratio", "regret"):
        for H, L in ((1, 1), (2, 4), (4, 0.1), (8, 2), (None, 1), (None, 4), (None, 0.3), (3, 0.5)):
            ours = cart.fit_cart(X, T, H, L, rule).to_nested()
            ref = so.fit_cart(Xl, y, H, L, rule, Tl, 0)
            assert ours == ref, (rule, H, L)


def test_predictions_and_metrics_match_the_oracle():
    X, T, Xl, Tl = _table(300, 10, 3)
    tr, te = slice(0, 240), slice(240, 300)
    for rule in ("majority", "logratio", "regret"):
        ours = cart.sweep(X[tr], T[tr], X[te], T[te], leaf_rule=rule)
        ref = so.sweep(Xl[tr], Tl[tr], Xl[te], Tl[te], leaf_rule=rule)
        assert [r["name"] for r in ours] == [r["name"] for r in ref]
        for a, b in zip(ours, ref):
            assert a["tree"].to_nested() == b["tree"]
            assert a["tree"].predict(X[te]).tolist() == [so.predict(b["tree"], x) for x in Xl[te]]
            assert a["leaves"] == b["leaves"] and a["height"] == b["height"]
            assert a["accuracy"] == pytest.approx(b["accuracy"], abs=1e-15)
            assert a["dtpr"] == pytest.approx(b["dtpr"], rel=1e-12)
            assert a["geomean"] == pytest.approx(b["geomean"], rel=1e-12)


def test_min_samples_and_names_match_the_oracle():
    for L in cart.L_SET:
        for n in (10, 192, 1600, 1601):
            assert cart.min_samples_leaf(L, n) == so.min_samples_leaf(L, n)
    assert [cart.model_name(H, L) for H in cart.H_SET for L in cart.L_SET] == \
           [so.model_name(H, L) for H in so.H_SET for L in so.L_SET]


def test_illegal_predictions_are_priced_as_the_fallback():
    T = np.array([[2.0, np.inf, 1.0], [3.0, 1.0, np.inf]])
    assert cart.ratios(T, [1, 2]).tolist() == [0.5, 1.0 / 3.0]
    assert cart.ratios(T, [1, 2]).tolist() == [so.performance_ratio(list(T[0]), 1), so.performance_ratio(list(T[1]), 2)]


def test_fallback_links_price_illegal_predictions_like_the_oracle():
    X, T, Xl, Tl = _table(220, 9, 17)
    rng = np.random.default_rng(3)
    T = T.copy()
    T[rng.uniform(size=T.shape) < 0.25] = np.inf
    T[:, 0] = np.where(np.isfinite(T[:, 0]), T[:, 0], 1.0)  # variant 0 legal everywhere
    Tl = [list(map(float, r)) for r in T]
    links = [0, 0, 1, 2, 3, 0, 5, 6, 7]
    E = cart.effective_times(T, links)
    for i in range(0, 220, 7):
        for v in range(9):
            assert E[i, v] == so.effective_time(Tl[i], v, links)
    y = so.labels_from_table(Tl)
    for rule in ("logratio", "regret"):
        ours = cart.fit_cart(X, T, None, 3, rule, links)
        ref = so.fit_cart(Xl, y, None, 3, rule, Tl, links)
        assert ours.to_nested() == ref
        pred = ours.predict(X)
        assert cart.geomean_ratio(T, pred, links) == pytest.approx(so.geomean_ratio(Tl, pred.tolist(), links), rel=1e-12)


def test_cross_validation_selects_a_model_without_the_heldout_set():
    X, T, _, _ = _table(250, 9, 4)
    best, table = cart.select_model(X[:200], T[:200], folds=4, H_set=(2, None), L_set=(1, 4, 0.2))
    assert len(table) == 18 and best in table  # 2 heights x 3 leaf sizes x 3 rules
    assert all(0 < r["cv_geomean"] <= 1 for r in table)
    assert best["cv_geomean"] == max(r["cv_geomean"] for r in table)


def _compile_selector(header_text, tmp_path):
    (tmp_path / "mdg_select_generated.h").write_text(header_text)
    (tmp_path / "sel.cpp").write_text('#include "mdg_select_generated.h"\nextern "C" int sel(int a,int b,long long M,long long N,long long K)'
                                      '{return mdg_generated_select(a,b,M,N,K);}\n'
                                      'extern "C" const char* name(){return MDG_GENERATED_SELECTOR_NAME;}\n'
                                      'extern "C" int dflt(int w){return w==0?MDG_GENERATED_DEFAULT_TILED:MDG_GENERATED_DEFAULT_DIRECT;}\n')
    lib = tmp_path / "libsel.so"
    subprocess.run(["g++", "-O1", "-shared", "-fPIC", "-o", str(lib), str(tmp_path / "sel.cpp")], check=True)
    L = ctypes.CDLL(str(lib))
    L.sel.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_longlong, ctypes.c_longlong, ctypes.c_longlong]
    L.name.restype = ctypes.c_char_p
    return L


@pytest.mark.parametrize("style", ["branches", "table"])
@pytest.mark.parametrize("H,L,rule", [(None, 1, "majority"), (4, 2, "logratio"), (0, 1, "majority")])
def test_generated_cpp_equals_the_tree_everywhere(H, L, rule, style, tmp_path):
    X, T, _, _ = _table(260, 11, 5)
    tree = cart.fit_cart(X, T, H, L, rule)
    nested = tree.to_nested()
    text = codegen.tree_to_cpp(nested, "test-model", variant_names=[f"v{i}" for i in range(11)], default_tiled=3,
                               default_direct=1, style=style)
    lib = _compile_selector(text, tmp_path)
    assert lib.name() == b"test-model" and lib.dflt(0) == 3 and lib.dflt(1) == 1
    # all training shapes plus threshold-1 / threshold / threshold+1 probes of every internal node
    probes = [tuple(r) for r in X.tolist()]
    for f, thr in codegen.internal_thresholds(nested):
        for d in (-1, 0, 1):
            probes.append(_probe(f, max(thr + d, 0), base=tuple(X[0].tolist())))
            probes.append(_probe(f, max(thr + d, 0), base=(1, 1, 1, 0, 0)))
    assert {f for f, _ in codegen.internal_thresholds(nested)} & {5, 6} or H == 0  # the products are used
    P = np.array(probes, dtype=np.int64)
    want = tree.predict(P)
    got = [lib.sel(int(p[3]), int(p[4]), int(p[0]), int(p[1]), int(p[2])) for p in P]
    assert got == want.tolist()
    assert got == [so.predict(nested, so.expand_features(tuple(int(x) for x in p))) for p in P]
    # saturation of the products: huge dimensions must not wrap around
    big = (2 ** 31 - 1, 2 ** 31 - 1, 2 ** 31 - 1, 0, 0)
    assert lib.sel(0, 0, big[0], big[1], big[2]) == so.predict(nested, so.expand_features(big)) == int(tree.predict([big])[0])


@pytest.mark.parametrize("seed,n,v,trees", [(7, 220, 9, 3), (8, 300, 12, 5)])
def test_forest_is_identical_to_the_oracle_and_to_its_generated_code(seed, n, v, trees, tmp_path):
    X, T, Xl, Tl = _table(n, v, seed)
    ntr = n - 60
    boot = wl.bootstrap_indices(ntr, trees)
    assert len(boot) == trees and all(b.shape == (ntr,) and b.min() >= 0 and b.max() < ntr for b in boot)
    assert all(np.array_equal(a, b) for a, b in zip(boot, wl.bootstrap_indices(ntr, trees)))  # seeded
    y = so.labels_from_table(Tl[:ntr])
    for rule, H, L in (("logratio", None, 4), ("majority", 3, 2)):
        ours = cart.fit_forest(X[:ntr], T[:ntr], boot, H, L, rule, 0)
        ref = so.fit_forest(Xl[:ntr], y, Tl[:ntr], [b.tolist() for b in boot], H, L, rule, 0)
        nested = ours.to_nested()
        assert nested == ref, rule
        want = ours.predict(X)
        assert want.tolist() == [so.predict_forest(ref, x, v) for x in Xl]
        assert ours.scores(X[:20]).tolist() == [so.forest_scores(ref, x, v) for x in Xl[:20]]
        text = codegen.tree_to_cpp(nested, "test-forest", variant_names=[f"v{i}" for i in range(v)])
        sub = tmp_path / rule  # a fresh path per library: the loader would hand back the first one otherwise
        sub.mkdir()
        lib = _compile_selector(text, sub)
        probes = [tuple(r) for r in X.tolist()]
        for f, thr in codegen.internal_thresholds(nested):
            for d in (-1, 0, 1):
                probes.append(_probe(f, max(thr + d, 0), base=tuple(X[0].tolist())))
        P = np.array(probes, dtype=np.int64)
        got = [lib.sel(int(p[3]), int(p[4]), int(p[0]), int(p[1]), int(p[2])) for p in P]
        assert got == ours.predict(P).tolist()
        assert got == [so.predict_forest(ref, so.expand_features(tuple(int(x) for x in p)), v) for p in P]


def test_gated_model_and_its_gate_are_identical_to_the_oracle_and_to_the_generated_code(tmp_path):
    X, T, Xl, Tl = _table(320, 10, 31)
    ntr = 260
    boot = wl.bootstrap_indices(ntr, 4)
    tree = cart.fit_cart(X[:ntr], T[:ntr], None, 4, "logratio", 0)
    forest = cart.fit_forest(X[:ntr], T[:ntr], boot, None, 4, "logratio", 0)
    nested_tree, nested_forest = tree.to_nested(), forest.to_nested()
    pt, pf = tree.predict(X), forest.predict(X)
    assert (pt != pf).sum() > 10  # the two models disagree often enough for the gate to matter
    # gate choice: same candidate set, same costs -> same gate and score as the plain-Python oracle
    gates = (0, 1 << 12, 1 << 18, 1 << 22, 1 << 26, 1 << 30, cart.INT64_MAX)
    for tree_ns, forest_ns in ((30.0, 500.0), (30.0, 30.0), (0.0, 5e4)):
        g, table = cart.choose_gate(X, T, pt, pf, tree_ns, forest_ns, 0, gate_set=gates)
        g_ref, score_ref = so.choose_gate(Xl, Tl, pt.tolist(), pf.tolist(), tree_ns, forest_ns, gates, 0)
        assert g == g_ref
        assert max(r["geomean_with_cost"] for r in table) == pytest.approx(score_ref, rel=1e-12)
    # with a free selector the cost-inclusive score of a forest-only gate is the plain geomean ratio
    _, table = cart.choose_gate(X, T, pt, pf, 0.0, 0.0, 0, gate_set=(0, cart.INT64_MAX))
    assert table[0]["geomean_with_cost"] == pytest.approx(cart.geomean_ratio(T, pf, 0), rel=1e-12)
    assert table[1]["geomean_with_cost"] == pytest.approx(cart.geomean_ratio(T, pt, 0), rel=1e-12)
    # generated code of the gated pair == product == oracle, also right at the gate
    gate = 1 << 18
    text = codegen.tree_to_cpp({"gate": gate, "tree": nested_tree, "forest": nested_forest}, "test-gated",
                               variant_names=[f"v{i}" for i in range(10)])
    lib = _compile_selector(text, tmp_path)
    probes = [tuple(r) for r in X.tolist()] + [(gate - 1, 1, 1, 0, 0), (gate, 1, 1, 0, 0), (gate + 1, 1, 1, 1, 1),
                                                 (1 << 9, 1 << 9, 1, 0, 1), (1 << 9, 1 << 9, 2, 1, 0), (511, 512, 1, 0, 0)]
    for f, thr in codegen.internal_thresholds({"gate": gate, "tree": nested_tree, "forest": nested_forest})[::7]:
        probes += [_probe(f, max(thr + d, 0), base=tuple(X[0].tolist())) for d in (-1, 0, 1)]
    P = np.array(probes, dtype=np.int64)
    got = [lib.sel(int(p[3]), int(p[4]), int(p[0]), int(p[1]), int(p[2])) for p in P]
    assert got == cart.gated_predict(P, gate, tree.predict(P), forest.predict(P)).tolist()
    assert got == [so.predict_gated(nested_tree, nested_forest, gate, so.expand_features(tuple(int(a) for a in p)), 10) for p in P]
    sides = {int(p[0]) * int(p[1]) * int(p[2]) < gate for p in P}
    assert sides == {True, False}


def test_forest_cross_validation_is_seeded_and_bounded():
    X, T, _, _ = _table(260, 9, 11)
    boot_for = lambda n: wl.bootstrap_indices(n, 4)  # noqa: E731
    a = cart.cross_validate_forest(X[:200], T[:200], boot_for, None, 2, "logratio", 0, folds=4)
    b = cart.cross_validate_forest(X[:200], T[:200], boot_for, None, 2, "logratio", 0, folds=4)
    assert a == b and 0 < a <= 1
    forest = cart.fit_forest(X[:200], T[:200], boot_for(200), None, 2, "logratio", 0)
    st = forest.stats()
    assert st["trees"] == 4 and st["leaves"] == sum(t.stats()["leaves"] for t in forest.trees)
    # every leaf lists at most FOREST_KEEP variants, cheapest first, and `rest` is no smaller than the last listed cost
    for tree in forest.to_nested():
        stack = [tree]
        while stack:
            n = stack.pop()
            if "leaf" in n:
                assert 1 <= len(n["ids"]) <= cart.FOREST_KEEP and n["costs"] == sorted(n["costs"]) and n["rest"] >= n["costs"][-1]
                assert len(set(n["ids"])) == len(n["ids"]) and n["costs"][0] >= 0
            else:
                stack += [n["left"], n["right"]]
    # a forest's training-set prediction is never worse than guessing the globally best single variant
    base = int(np.argmin(np.sum(np.log(T[:200]), axis=0)))
    assert cart.geomean_ratio(T[:200], forest.predict(X[:200]), 0) >= cart.geomean_ratio(T[:200], np.full(200, base), 0)


def test_shipped_selector_matches_the_stored_model():
    # the header compiled into the library must be the one generated from results/model.json
    from paper_1806_07060_amd import binding as mdg
    path = os.path.join(ROOT, "paper_1806_07060_amd", "tuning", "results", "model.json")
    if not os.path.exists(path):
        pytest.skip("no trained model stored yet")
    model = json.load(open(path))
    assert mdg.mdg_selector_name() == model["name"]
    # the model was trained on the variant table as it stood; variants added since sit behind those it knows
    assert model["variants"] == [v["name"] for v in mdg.variants()][:len(model["variants"])]
    rng = np.random.default_rng(6)
    P = np.column_stack([np.rint(2.0 ** (13 * rng.uniform(size=(3000, 3)))).astype(np.int64),
                         rng.integers(0, 2, size=(3000, 2))])
    extra = []
    # what ships: the tree alone, the forest alone (gate 0), or the gated pair
    n_var = len(model["variants"])
    gate = model.get("gate")
    if not model.get("forest"):
        shipped = model["tree"]
        want_of = lambda x: so.predict(shipped, x)  # noqa: E731
    elif gate in (None, 0):
        shipped = model["forest"]
        want_of = lambda x: so.predict_forest(shipped, x, n_var)  # noqa: E731
    else:
        shipped = {"gate": gate, "tree": model["tree"], "forest": model["forest"]}
        want_of = lambda x: so.predict_gated(model["tree"], model["forest"], gate, x, n_var)  # noqa: E731
    thresholds = codegen.internal_thresholds(shipped)
    if len(thresholds) > 4000:  # a forest has tens of thousands of nodes: probe a seeded sample of them
        thresholds = [thresholds[i] for i in rng.choice(len(thresholds), 4000, replace=False)]
    for f, thr in thresholds:
        for d in (-1, 0, 1):
            extra.append(_probe(f, max(0, thr + d)))
    P = np.vstack([P, np.array(extra, dtype=np.int64).reshape(-1, 5)])
    if gate not in (None, 0):  # both sides of the gate, and the gate itself
        extra += [(gate - 1, 1, 1, 0, 0), (gate, 1, 1, 0, 0), (2048, 2048, 2048, 0, 1), (4096, 4096, 4096, 1, 0), (8192, 8192, 8192, 0, 0)]
        P = np.vstack([P, np.array(extra[-5:], dtype=np.int64)])
    for p in P:
        x = so.expand_features(tuple(int(a) for a in p))
        assert mdg.mdg_select(int(p[3]), int(p[4]), int(p[0]), int(p[1]), int(p[2])) == want_of(x)
    d = model["default_dispatch"]
    assert mdg.mdg_select_default(0, 0, 4096, 4096, 4096) == d["tiled"]
    assert mdg.mdg_select_default(0, 0, 8, 8, 8) == d["direct"]


def test_training_union_keeps_evaluation_shapes_out_and_is_seeded():
    from paper_1806_07060_amd.tuning import train
    X4, T4, _, _ = _table(100, 5, 21)
    Xe, Te, _, _ = _table(40, 5, 22)
    tab4 = {"X": X4, "T": T4}
    extra = {"X": np.vstack([Xe, X4[90:95]]), "T": np.vstack([Te, T4[90:95]])}
    banned = {"X": Xe[:7], "T": Te[:7]}
    X, T, src = train.training_union(tab4, [("grid", extra)], [banned])
    # 80 rows of the sweep + 45 extra rows minus the 7 banned shapes and the 5 that repeat held-out shapes
    assert X.shape[0] == 80 + 45 - 7 - 5 and src.count("cfg4") == 80 and src.count("grid") == 33
    assert not ({tuple(r[:3]) for r in X4[80:].tolist()} & {tuple(r[:3]) for r in X.tolist()})  # no held-out shape leaks in
    have = {tuple(r[:3]) for r in X.tolist()}
    assert not ({tuple(r[:3]) for r in Xe[:7].tolist()} & have)
    # the held-out 20 % of the sweep never enters through the sweep itself
    assert {tuple(r) for r in X[[i for i, s in enumerate(src) if s == "cfg4"]].tolist()} == {tuple(r) for r in X4[:80].tolist()}
    X2, T2, src2 = train.training_union(tab4, [("grid", extra)], [banned])
    assert np.array_equal(X, X2) and np.array_equal(T, T2) and src == src2


def test_default_dispatch_picks_per_family_bests_on_the_two_cubes():
    from paper_1806_07060_amd.tuning import train
    meta = [{"family": 0, "split_k": 1}, {"family": 0, "split_k": 1}, {"family": 1, "split_k": 1},
            {"family": 1, "split_k": 1}, {"family": 1, "split_k": 4}]
    X = np.array([[256, 256, 256, a, b] for a in (0, 1) for b in (0, 1)] + [[1024, 1024, 1024, a, b] for a in (0, 1) for b in (0, 1)])
    T = np.ones((8, 5))
    T[:4] = [2.0, 1.5, 1.0, 3.0, 0.5]  # 256-cube: best direct is variant 1 (tiled ones do not count)
    T[4:] = [9.0, 9.0, 4.0, 3.0, 1.0]  # 1024-cube: best tiled without split-K is variant 3
    tiled, direct, thr = train.default_dispatch({"X": X, "T": T}, meta)
    assert (tiled, direct, thr) == (3, 1, 512.0 ** 3)


def test_product_and_oracle_agree_on_measured_tables():
    # the same trees on a slice of the real timing table (illegal entries, fallback links, dozens of classes)
    from paper_1806_07060_amd import binding as mdg
    from paper_1806_07060_amd.tuning import train
    path = os.path.join(train.RESULTS, "timings_cfg4.csv")
    if not os.path.exists(path):
        pytest.skip("no timing table stored")
    tab = train.load_table(path)
    if tab["variants"] != [v["name"] for v in mdg.variants()]:
        pytest.skip("stored table belongs to another variant table")
    links = train.fallback_links(mdg.variants())
    X, T = tab["X"][:300], tab["T"][:300]
    Xl = [so.expand_features(tuple(int(a) for a in r)) for r in X]
    Tl = [list(map(float, r)) for r in T]
    y = so.labels_from_table(Tl)
    for rule, H, L in (("majority", None, 1), ("logratio", 6, 4), ("regret", 5, 3)):
        ours = cart.fit_cart(X, T, H, L, rule, links)
        ref = so.fit_cart(Xl, y, H, L, rule, Tl, links)
        assert ours.to_nested() == ref, rule
        pred = ours.predict(tab["X"][300:500])
        assert pred.tolist() == [so.predict(ref, so.expand_features(tuple(int(a) for a in r))) for r in tab["X"][300:500]]
        Th = [list(map(float, r)) for r in tab["T"][300:500]]
        assert cart.dtpr(tab["T"][300:500], pred, links) == pytest.approx(so.dtpr(Th, pred.tolist(), links), rel=1e-12)
