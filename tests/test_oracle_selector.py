"""Pins for the selector oracle (CPU only).

The oracle follows Section 3 ('Datasets', 'Model and code generation'),
Section 4.2 (H and L) and Section 5.2 (accuracy, DTPR).  Pins: hand-computed
toy trees, invariants that hold for any data and that the paper's own go2
table exhibits (tests/golden/go2_p100_trees.txt), and scikit-learn's CART
(the learner the paper used) as an independent judge of every split.
"""
import math
import os

import numpy as np
import pytest

from oracle import selector_oracle as so
from paper_1806_07060_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_best_variant_is_argmin_time_lowest_id_on_ties():
    assert so.best_variant([3.0, 1.0, 2.0]) == 1
    assert so.best_variant([2.0, 1.0, 1.0]) == 1
    assert so.best_variant([math.inf, 5.0]) == 1
    assert so.labels_from_table([[1, 2], [2, 1]]) == [0, 1]


def test_min_samples_leaf_readings():
    assert so.min_samples_leaf(1, 1600) == 1
    assert so.min_samples_leaf(4, 1600) == 4
    assert so.min_samples_leaf(0.1, 1600) == 160
    assert so.min_samples_leaf(0.3, 1601) == 481  # ceil(480.3)
    assert so.min_samples_leaf(0.5, 7) == 4


def test_one_dimensional_separable_threshold_is_midpoint():
    X = [(1,), (2,), (10,), (11,)]
    y = [0, 0, 1, 1]
    t = so.fit_cart(X, y)
    assert (t["feature"], t["threshold"]) == (0, 6)
    assert t["left"] == {"leaf": 0, "n": 2} and t["right"] == {"leaf": 1, "n": 2}
    assert [so.predict(t, (v,)) for v in (-5, 6, 7, 100)] == [0, 0, 1, 1]


def test_hand_computed_gini_tree():
    # values 1..6 with labels A A B B B A.  Weighted Gini by hand: split after 2 -> 1/4 (best),
    # after 1 or 5 -> 2/5, after 3 -> 4/9, after 4 -> 1/2.  The right child {B,B,B,A} then splits after 5.
    X = [(v,) for v in range(1, 7)]
    y = [0, 0, 1, 1, 1, 0]
    t = so.fit_cart(X, y)
    assert (t["feature"], t["threshold"]) == (0, 2)
    assert t["left"] == {"leaf": 0, "n": 2}
    r = t["right"]
    assert (r["feature"], r["threshold"]) == (0, 5)
    assert r["left"] == {"leaf": 1, "n": 3} and r["right"] == {"leaf": 0, "n": 1}
    # with L = 2 the split after 5 is forbidden (one sample on the right); {3,4 | 5,6} is the only legal one
    t2 = so.fit_cart(X, y, L=2)
    assert t2["right"]["threshold"] == 4
    assert t2["right"]["right"] == {"leaf": 0, "n": 2}  # tie B/A -> lowest id
    # H = 1 stops below the root
    t3 = so.fit_cart(X, y, H=1)
    assert t3["right"] == {"leaf": 1, "n": 4}


def test_xor_needs_height_two():
    X = [(a, b) for a in (0, 1) for b in (0, 1)] * 3
    y = [a ^ b for a, b in X]
    t1 = so.fit_cart(X, y, H=1)
    assert so.accuracy([so.predict(t1, x) for x in X], y) == 0.5
    t2 = so.fit_cart(X, y, H=2)
    assert so.accuracy([so.predict(t2, x) for x in X], y) == 1.0
    assert so.tree_stats(t2)["height"] == 2 and so.tree_stats(t2)["leaves"] == 4
    # first split is a zero-gain tie between both features -> lowest feature index
    assert t2["feature"] == 0


def test_height_zero_tree_is_most_frequent_label():
    X = [(i,) for i in range(7)]
    y = [2, 1, 2, 1, 1, 2, 0]
    assert so.fit_cart(X, y, H=0) == {"leaf": 1, "n": 7}  # 3 x label 1, 3 x label 2 -> lowest id
    assert so.fit_cart(X, y, L=0.5) == {"leaf": 1, "n": 7}  # 7 < 2 * ceil(3.5): the root cannot be split


def _table(n=300, v=10, seed=3):
    feats, times = wl.synthetic_timing_table(n, v, seed)
    X = [tuple(int(a) for a in r) for r in feats]
    T = [list(map(float, r)) for r in times]
    return X, T


def test_ratio_metrics_by_hand_and_bounded_by_one():
    T = [[1.0, 2.0, 4.0], [math.inf, 3.0, 1.5], [2.0, math.inf, 1.0]]
    # row 0: best 0; predicting 2 gives 1/4.  row 1: best 2 (1.5); predicting 0 is illegal -> fallback 0 is
    # itself illegal here, so use fallback = 1: 1.5/3.  row 2: predicting 1 illegal -> fallback 0: 1/2
    assert so.performance_ratio(T[0], 2) == 0.25
    assert so.performance_ratio(T[1], 0, fallback=1) == 0.5
    assert so.performance_ratio(T[2], 1, fallback=0) == 0.5
    assert so.dtpr(T, [0, 2, 2]) == 1.0
    assert math.isclose(so.dtpr(T, [2, 1, 1], fallback=0), (0.25 + 0.5 + 0.5) / 3)
    assert math.isclose(so.geomean_ratio(T, [2, 1, 1], fallback=0), (0.25 * 0.5 * 0.5) ** (1 / 3))
    X, T = _table()
    y = so.labels_from_table(T)
    for H, L in ((2, 1), (None, 4), (8, 0.1)):
        tree = so.fit_cart(X, y, H, L)
        pred = [so.predict(tree, x) for x in X]
        assert all(0 < so.performance_ratio(r, p) <= 1.0 for r, p in zip(T, pred))
        assert so.dtpr(T, pred) <= 1.0 and so.geomean_ratio(T, pred) <= so.dtpr(T, pred) + 1e-15


def test_fully_grown_tree_reproduces_training_labels():
    X, T = _table()
    assert len(set(X)) == len(X)
    y = so.labels_from_table(T)
    tree = so.fit_cart(X, y, None, 1)
    pred = [so.predict(tree, x) for x in X]
    assert pred == y
    assert so.dtpr(T, pred) == 1.0 and so.geomean_ratio(T, pred) == 1.0


@pytest.mark.parametrize("rule", ["majority", "logratio"])
def test_structural_invariants_for_every_model_of_the_sweep(rule):
    X, T = _table(240, 8, 11)
    n_train = 192
    rows = so.sweep(X[:n_train], T[:n_train], X[n_train:], T[n_train:], leaf_rule=rule)
    assert len(rows) == 40
    assert rows[0]["name"] == "h1-L1" and rows[-1]["name"] == "hMax-L0.5"
    for r in rows:
        st = so.tree_stats(r["tree"])
        L_abs = so.min_samples_leaf(r["L"], n_train)
        assert st["min_leaf_samples"] >= L_abs
        assert st["leaves"] <= n_train // L_abs
        if r["H"] is not None:
            assert st["height"] <= r["H"] and st["leaves"] <= 2 ** r["H"]
        if isinstance(r["L"], float):
            assert st["leaves"] <= math.floor(1 / r["L"] + 1e-9)
        assert 0 < r["geomean"] <= r["dtpr"] <= 1.0
        assert 0 <= r["accuracy"] <= 1.0


def test_papers_go2_table_shows_the_same_invariants():
    # our reading of H and L (height cap; L as a fraction of the samples) must be consistent with
    # every row the paper prints for go2 on the P100
    rows = [l.split() for l in open(os.path.join(GOLD, "go2_p100_trees.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 40
    for name, acc, dtpr_, dttr, leaves, height, L in rows:
        leaves, height = int(leaves), int(height)
        H = name.split("-")[0][1:]
        if H != "Max":
            assert height <= int(H) and leaves <= 2 ** int(H)
        assert leaves >= 1 and height <= max(leaves - 1, 0)
        L_name = name.split("-L")[1]  # the row name, not the min-samples column (one row misprints it)
        if "." in L_name:
            assert leaves <= math.floor(1 / float(L_name) + 1e-9)
        assert float(dtpr_) <= 1.0
    sizes = dict(l.split() for l in open(os.path.join(GOLD, "dataset_sizes.txt")) if not l.startswith("#"))
    assert len(wl.go2()) == int(sizes["go2"]) and len(wl.po2()) == int(sizes["po2"])
    assert min(min(t) for t in wl.go2()) == 256 and max(max(t) for t in wl.go2()) == 3840
    assert min(min(t) for t in wl.po2()) == 64 and max(max(t) for t in wl.po2()) == 2048


def _weighted_gini(y_left, y_right):
    def g(y):
        _, c = np.unique(y, return_counts=True)
        p = c / c.sum()
        return 1.0 - float(np.sum(p * p))
    n = len(y_left) + len(y_right)
    return len(y_left) / n * g(y_left) + len(y_right) / n * g(y_right)


@pytest.mark.parametrize("L", [1, 3, 0.1])
def test_every_split_is_optimal_according_to_scikit_learn(L):
    # scikit-learn's CART (what the paper used) judges each internal node: a depth-1 sklearn tree fitted on the
    # node's samples with the same minimum leaf size must not find a split with lower weighted Gini impurity.
    from sklearn.tree import DecisionTreeClassifier
    X, T = _table(200, 9, 5)
    y = so.labels_from_table(T)
    L_abs = so.min_samples_leaf(L, len(X))
    tree = so.fit_cart(X, y, 6, L)
    Xa, ya = np.array(X), np.array(y)
    checked = 0
    stack = [(tree, np.arange(len(X)))]
    while stack:
        node, idx = stack.pop()
        if "leaf" in node:
            continue
        f, thr = node["feature"], node["threshold"]
        li, ri = idx[Xa[idx, f] <= thr], idx[Xa[idx, f] > thr]
        assert len(li) >= L_abs and len(ri) >= L_abs and len(li) + len(ri) == node["n"]
        ours = _weighted_gini(ya[li], ya[ri])
        sk = DecisionTreeClassifier(criterion="gini", max_depth=1, min_samples_leaf=L_abs, random_state=0)
        sk.fit(Xa[idx], ya[idx])
        if sk.tree_.node_count == 3:
            t_ = sk.tree_
            theirs = (t_.weighted_n_node_samples[1] * t_.impurity[1] + t_.weighted_n_node_samples[2] * t_.impurity[2]) \
                / t_.weighted_n_node_samples[0]
            assert abs(ours - theirs) < 1e-12
            checked += 1
        stack.append((node["left"], li))
        stack.append((node["right"], ri))
    assert checked >= 5


def test_matches_scikit_learn_training_accuracy_when_fully_grown():
    from sklearn.tree import DecisionTreeClassifier
    X, T = _table(150, 6, 9)
    y = so.labels_from_table(T)
    for L in (1, 2, 5):
        tree = so.fit_cart(X, y, None, L)
        sk = DecisionTreeClassifier(criterion="gini", min_samples_leaf=L, random_state=0).fit(np.array(X), np.array(y))
        ours = so.accuracy([so.predict(tree, x) for x in X], y)
        if L == 1:
            assert ours == 1.0 and sk.score(np.array(X), np.array(y)) == 1.0
        else:
            # greedy ties may be broken differently; the trees must still be of similar quality
            assert abs(ours - sk.score(np.array(X), np.array(y))) < 0.1


def test_logratio_leaf_label_by_hand():
    rows = [[1.0, 1.1, 5.0], [1.0, 1.1, 5.0], [9.0, 1.0, 5.0]]
    # majority label is 0, but variant 1 is nearly as good on rows 0, 1 and far better on row 2
    assert so._majority(so.labels_from_table(rows)) == 0
    assert so.logratio_label(rows) == 1
    # variant 0 is illegal on the first row: it is priced as the fallback (variant 1) there -> log-sums tie at
    # log(1) + log(1) for variant 0 and log(1) + log(1/3) for variant 1 -> variant 0
    assert so.logratio_label([[math.inf, 2.0], [1.0, 3.0]], fallback=1) == 0
    t = so.fit_cart([(1,), (2,), (3,)], [0, 0, 1], H=0, leaf_rule="logratio", table=rows)
    assert t == {"leaf": 1, "n": 3}


def test_regret_tree_by_hand():
    # two variants; costs in units of log-ratio.  Inputs 1..4 on one feature:
    #   x=1,2: variant 0 is best (variant 1 twice as slow);  x=3: variant 1 best (variant 0 4x slower);
    #   x=4: variant 1 best (variant 0 only 1 % slower).
    X = [(1,), (2,), (3,), (4,)]
    T = [[1.0, 2.0], [1.0, 2.0], [4.0, 1.0], [1.01, 1.0]]
    y = so.labels_from_table(T)
    cost = so.regret_cost_rows(T)
    assert cost[0] == [0, round(math.log(2) * 2 ** 20)] and cost[2] == [round(math.log(4) * 2 ** 20), 0]
    # depth-0 tree: variant 0 costs log4 + log1.01, variant 1 costs 2 log2 = log4 -> variant 1
    assert so.fit_cart(X, y, H=0, leaf_rule="regret", table=T) == {"leaf": 1, "n": 4}
    # the cut after x=2 leaves both sides with a zero-cost variant: it must be chosen
    t = so.fit_cart(X, y, H=1, leaf_rule="regret", table=T)
    assert (t["feature"], t["threshold"]) == (0, 2) and t["left"]["leaf"] == 0 and t["right"]["leaf"] == 1
    # Gini sees the same labels here; make x=4 prefer variant 0 by a hair: Gini now wants {1,2},{3},{4} (3 leaves),
    # the regret tree with L=2 must keep {3,4} together and label it 1 (the hair costs less than the factor 4)
    T2 = [[1.0, 2.0], [1.0, 2.0], [4.0, 1.0], [1.0, 1.01]]
    t2 = so.fit_cart(X, so.labels_from_table(T2), L=2, leaf_rule="regret", table=T2)
    assert t2["threshold"] == 2 and t2["right"] == {"leaf": 1, "n": 2}
    # a node whose best single variant already costs nothing is not split, whatever the labels say
    T3 = [[1.0, 1.0], [1.0, 2.0], [1.0, 1.0], [1.0, 3.0]]
    assert so.fit_cart(X, [1, 0, 1, 0], leaf_rule="regret", table=T3) == {"leaf": 0, "n": 4}


def test_regret_trees_never_score_below_their_own_root_and_respect_limits():
    X, T = _table(200, 8, 13)
    y = so.labels_from_table(T)
    root = so.fit_cart(X, y, H=0, leaf_rule="regret", table=T)
    base = so.geomean_ratio(T, [root["leaf"]] * len(X))
    for H, L in ((2, 1), (4, 5), (None, 10), (None, 0.2)):
        tree = so.fit_cart(X, y, H, L, "regret", T)
        st = so.tree_stats(tree)
        assert st["min_leaf_samples"] >= so.min_samples_leaf(L, len(X))
        if H is not None:
            assert st["height"] <= H
        pred = [so.predict(tree, x) for x in X]
        # every split lowers (or keeps) the summed training cost, so the training geomean cannot get worse
        assert so.geomean_ratio(T, pred) >= base - 1e-12
    full = so.fit_cart(X, y, None, 1, "regret", T)
    assert so.geomean_ratio(T, [so.predict(full, x) for x in X]) == 1.0  # distinct inputs -> zero training cost


def test_expand_features_by_hand_and_saturation():
    # padding by hand: 3 rows -> 29 / 61 / 125 more to the next multiple of 32 / 64 / 128; 5 columns -> 27 / 59 / 123
    assert so.expand_features((3, 5, 7, 1, 0)) == (3, 5, 7, 1, 0, 15, 105, 29, 61, 125, 27, 59, 123)
    # exact multiples add nothing
    assert so.expand_features((8192, 8192, 8192, 0, 1)) == (8192, 8192, 8192, 0, 1, 2 ** 26, 2 ** 39) + (0,) * 6
    # 96 = 3 x 32 fits the 32-grid, needs 32 more for the 64- and the 128-grid; 100 -> 28, 28, 28
    assert so.expand_features((96, 100, 1, 0, 0))[7:] == (0, 32, 32, 28, 28, 28)
    assert so.expand_features((129, 127, 1, 0, 0))[7:] == (31, 63, 127, 1, 1, 1)
    big = 2 ** 31 - 1
    f = so.expand_features((big, big, big, 0, 0))
    assert f[5] == big * big and f[6] == 2 ** 63 - 1  # M*N fits in 63 bits, M*N*K saturates
    assert f[7:] == (1, 1, 1, 1, 1, 1)  # 2^31 - 1 is one short of a multiple of every power of two
    assert so.expand_features((0, 9, 9, 0, 0))[5:7] == (0, 0)
    assert so.expand_features((0, 9, 9, 0, 0))[7:10] == (0, 0, 0)


def test_fallback_links_are_followed_to_the_first_legal_variant():
    inf = math.inf
    links = [0, 0, 1, 2]  # 3 -> 2 -> 1 -> 0
    row = [8.0, inf, inf, inf]
    assert so.effective_time(row, 3, links) == 8.0  # three hops
    row = [8.0, 4.0, inf, inf]
    assert so.effective_time(row, 3, links) == 4.0 and so.effective_time(row, 2, links) == 4.0
    assert so.effective_time(row, 1, links) == 4.0 and so.effective_time(row, 0, links) == 8.0
    assert so.performance_ratio([8.0, 4.0, inf, 2.0], 2, links) == 0.5
    # a universal fallback id still works and differs where the chain stops earlier
    assert so.effective_time(row, 3, 0) == 8.0
    with pytest.raises(ValueError):
        so.effective_time([inf, inf], 1, [0, 0])


def test_forest_leaf_cost_lists_and_vote_by_hand(monkeypatch):
    # one feature, two variants plus a third that is never good; times chosen so that the costs are round numbers:
    # ratio 1 -> cost 0, ratio 1/e -> cost 2^20, ratio 1/e^2 -> cost 2^21
    e = math.e
    X = [so.expand_features((m, 1, 1, 0, 0)) for m in (10, 20, 30, 40)]
    T = [[1.0, e, e * e], [1.0, e, e * e], [e, 1.0, e * e], [e * e, 1.0, e]]
    y = so.labels_from_table(T)
    assert y == [0, 0, 1, 1]
    cost = so.regret_cost_rows(T)
    S = so.REGRET_SCALE
    assert cost == [[0, S, 2 * S], [0, S, 2 * S], [S, 0, 2 * S], [2 * S, 0, S]]
    monkeypatch.setattr(so, "FOREST_KEEP", 2)
    # tree 0 sees rows (0, 1, 2, 3): one split at M <= 25, pure leaves.  left leaf: means (0, S, 2S) -> keeps variants
    # 0 and 1, rest = 2S; right leaf: sums (3S, 0, 3S) over 2 rows -> means (3S//2, 0, 3S//2) -> keeps 1 then 0
    # (equal means: lower id first), rest = 3S//2
    # tree 1 sees rows (0, 0, 2, 2): split at M <= 20; left leaf (row 0 twice): (0, S, 2S); right leaf (row 2 twice): (S, 0, 2S)
    forest = so.fit_forest(X, y, T, [[0, 1, 2, 3], [0, 0, 2, 2]], None, 1, "majority", 0)
    t0, t1 = forest
    assert (t0["feature"], t0["threshold"]) == (0, 25) and (t1["feature"], t1["threshold"]) == (0, 20)
    assert (t0["left"]["ids"], t0["left"]["costs"], t0["left"]["rest"]) == ([0, 1], [0, S], 2 * S)
    assert (t0["right"]["ids"], t0["right"]["costs"], t0["right"]["rest"]) == ([1, 0], [0, 3 * S // 2], 3 * S // 2)
    assert (t1["left"]["ids"], t1["left"]["costs"], t1["left"]["rest"]) == ([0, 1], [0, S], 2 * S)
    assert (t1["right"]["ids"], t1["right"]["costs"], t1["right"]["rest"]) == ([1, 0], [0, S], 2 * S)
    # M = 22: tree 0 goes left (22 <= 25), tree 1 goes right (22 > 20):
    # variant 0: 0 + S, variant 1: S + 0, variant 2: rest 2S + rest 2S -> tie between 0 and 1 -> lowest id
    x = so.expand_features((22, 1, 1, 0, 0))
    assert so.forest_scores(forest, x, 3) == [S, S, 4 * S]
    assert so.predict_forest(forest, x, 3) == 0
    # M = 35: both right: variant 0: 3S//2 + S, variant 1: 0, variant 2: 3S//2 + 2S
    x = so.expand_features((35, 1, 1, 0, 0))
    assert so.forest_scores(forest, x, 3) == [3 * S // 2 + S, 0, 3 * S // 2 + 2 * S]
    assert so.predict_forest(forest, x, 3) == 1


def test_forest_of_identical_full_samples_predicts_like_its_tree_when_leaves_are_pure():
    # bootstrap = the whole training set, fully grown tree, distinct inputs: every leaf holds one input, whose
    # best variant has cost 0 -> the forest (any number of copies) reproduces the labels
    rows = [(m, n, 3, 0, 0) for m in (1, 5, 9, 13) for n in (2, 4, 8)]
    X = [so.expand_features(r) for r in rows]
    T = [[1.0 + ((3 * i + 2 * v) % 7) for v in range(5)] for i in range(len(rows))]
    y = so.labels_from_table(T)
    whole = list(range(len(rows)))
    forest = so.fit_forest(X, y, T, [whole, whole, whole], None, 1, "majority", 0)
    assert [so.predict_forest(forest, x, 5) for x in X] == y
    assert so.geomean_ratio(T, [so.predict_forest(forest, x, 5) for x in X]) == 1.0


def test_gated_model_and_gate_choice_worked_out_by_hand():
    # two inputs, two variants.  Input A is small (work 8), input B is large (work 10^9).
    #   times (seconds)      v0        v1
    #   A                    4e-6      2e-6      best v1
    #   B                    2e-3      1e-3      best v1
    # the 'tree' always answers v0 except it is right on A; the 'forest' is right on both.
    tree = {"feature": 6, "threshold": 100, "n": 2, "left": {"leaf": 1, "n": 1}, "right": {"leaf": 0, "n": 1}}
    forest = [{"leaf": 1, "n": 2, "ids": [1, 0], "costs": [0, 700000], "rest": 700000}]
    xa, xb = so.expand_features((2, 2, 2, 0, 0)), so.expand_features((1000, 1000, 1000, 0, 0))
    assert xa[6] == 8 and xb[6] == 10 ** 9
    assert so.predict_gated(tree, forest, 9, xa, 2) == so.predict(tree, xa) == 1          # below the gate: the tree
    assert so.predict_gated(tree, forest, 8, xa, 2) == so.predict_forest(forest, xa, 2) == 1  # at the gate: the forest
    assert so.predict_gated(tree, forest, 10 ** 9 + 1, xb, 2) == 0 and so.predict_gated(tree, forest, 10 ** 9, xb, 2) == 1
    times = [[4e-6, 2e-6], [2e-3, 1e-3]]
    # selector costs: tree 0 ns, forest 2000 ns.  Ratios t_best / (t_pred + c):
    #   gate 0   (forest, forest): A 2e-6 / 4e-6 = 0.5       B 1e-3 / 1.002e-3
    #   gate 100 (tree, forest)  : A 2e-6 / 2e-6 = 1         B 1e-3 / 1.002e-3       <- best
    #   gate inf (tree, tree)    : A 1                        B 1e-3 / 2e-3 = 0.5
    assert so.ratio_with_selector_cost(times[0], 1, 2000e-9) == pytest.approx(0.5)
    assert so.ratio_with_selector_cost(times[1], 0, 0.0) == pytest.approx(0.5)
    g, score = so.choose_gate([xa, xb], times, [1, 0], [1, 1], 0.0, 2000.0, (0, 100, 2 ** 63 - 1))
    assert g == 100 and score == pytest.approx(math.sqrt(1.0 * (1e-3 / 1.002e-3)))
    # a forest as cheap as the tree wins everywhere: first maximum in candidate order is gate 0
    g, score = so.choose_gate([xa, xb], times, [1, 0], [1, 1], 0.0, 0.0, (0, 100, 2 ** 63 - 1))
    assert g == 0 and score == pytest.approx(1.0)
    # a forest that costs ten milliseconds per evaluation never pays (B: 1e-3 / 11e-3 < 0.5): the tree alone
    g, _ = so.choose_gate([xa, xb], times, [1, 0], [1, 1], 0.0, 1e7, (0, 100, 2 ** 63 - 1))
    assert g == 2 ** 63 - 1
