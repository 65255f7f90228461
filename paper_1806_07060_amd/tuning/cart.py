"""Off-line phase, step 2: labels, CART decision trees and the ratio metrics (numpy, vectorised).

Follows Section 3 ('Datasets', 'Model and code generation'), Section 4.2 (the
hyper-parameters H = maximum height and L = minimum samples per leaf) and
Section 5.2 (accuracy and DTPR) of the paper:

  label(s)   = argmax_a f_a(s) = the variant with the smallest measured time
  tree       = CART on integer features of the input description (M, N, K, tA, tB):
               the five raw values, the two products M*N (size of C, i.e. how many
               tiles there are to share among the CUs) and M*N*K (the work), and six
               tile-fit values: the rows (columns) a 32-, 64- or 128-wide tile grid adds
               beyond M (N), 0 when the size is an exact multiple; Gini impurity
  DTPR       = mean over inputs of f_predicted / f_best

Rules fixed where the paper leaves them open: fractional L = ceil(L * n)
samples; an impure node below height H is split whenever some split leaves L
samples on both sides (also at zero gain); thresholds are floor(midpoint) of
consecutive distinct values, tested as feature <= threshold; ties go to the
lowest feature index, then the lowest threshold; majority ties to the lowest
variant id; an illegal prediction is priced as the fallback variant.  Split
scores are compared exactly (integer arithmetic), so the tree is a pure
function of the table.

Leaf labels: 'majority' (plain CART) or 'logratio' (the variant maximising the
summed log performance ratio over the leaf's training inputs, which prices a
misclassification by what it costs -- the weakness Section 5.2 points out for
accuracy-driven trees).

A third rule, 'regret', also makes the *splits* cost-sensitive (one of the
"more effective models" the paper's conclusion asks for): every (input,
variant) pair gets an integer cost round(-2^20 * log(f_variant / f_best)), a
node's cost is the smallest column sum over its inputs (the loss of the best
single variant for that node), and a split is chosen to minimise the summed
cost of its two children.  Integer costs keep every comparison exact.  A node
whose cost is zero is not split; its label is the minimising variant.

Forest (another of those "more effective models"): several trees, each grown on
a bootstrap sample of the training inputs (the sample indices are an input of
fit_forest, drawn by the seeded generator in workloads.py).  A leaf does not
vote for one variant; it carries, for the FOREST_KEEP variants that are cheapest
on the bootstrap inputs it holds, their mean integer cost floor(sum / count)
(costs as in 'regret', capped at COST_CAP), and `rest`, the mean cost of the
next cheapest variant, which stands in for every variant not listed.  The
forest predicts the variant with the smallest cost summed over its trees (ties
to the lowest id).  Everything is integer arithmetic, so the numpy code here,
the plain-Python oracle and the generated C++ agree bit for bit.
"""
from fractions import Fraction
import math

import sys

import numpy as np

RAW_FEATURES = ("M", "N", "K", "tA", "tB")
TILE_WIDTHS = (32, 64, 128)
FEATURES = (RAW_FEATURES + ("MN", "MNK") + tuple(f"padM{t}" for t in TILE_WIDTHS)
            + tuple(f"padN{t}" for t in TILE_WIDTHS))
INT64_MAX = (1 << 63) - 1


def expand_features(X):
    """[n, 5] raw (M, N, K, tA, tB) -> [n, 13]: M*N and M*N*K appended (saturating at INT64_MAX, exactly as
    the generated C++ computes them), then padM32, padM64, padM128, padN32, padN64, padN128 with
    pad<X><t> = (t - X mod t) mod t.  Arrays that already have 13 columns pass through."""
    X = np.asarray(X, dtype=np.int64).reshape(-1, np.asarray(X).shape[-1])
    if X.shape[1] == len(FEATURES):
        return X
    assert X.shape[1] == len(RAW_FEATURES)
    mn = [int(m) * int(n) for m, n in zip(X[:, 0].tolist(), X[:, 1].tolist())]  # Python ints: no overflow
    mnk = [min(a * int(k), INT64_MAX) for a, k in zip(mn, X[:, 2].tolist())]
    mn = [min(a, INT64_MAX) for a in mn]
    pads = [(t - X[:, c] % t) % t for c in (0, 1) for t in TILE_WIDTHS]
    return np.column_stack([X, np.array(mn, dtype=np.int64), np.array(mnk, dtype=np.int64)] + pads)
H_SET = (1, 2, 4, 8, None)
L_SET = (1, 2, 4, 0.1, 0.2, 0.3, 0.4, 0.5)


def model_name(H, L):
    return f"h{'Max' if H is None else H}-L{L}"


def labels_from_table(times):
    """argmin over variants per row (first minimum = lowest id on ties)."""
    return np.argmin(np.asarray(times, dtype=np.float64), axis=1).astype(np.int64)


def min_samples_leaf(L, n_train):
    if isinstance(L, float) and 0.0 < L < 1.0:
        return max(1, math.ceil(Fraction(L).limit_denominator(1000) * n_train))
    return max(1, int(L))


def effective_times(times, fallback=0):
    """Times the library really spends per predicted variant: illegal entries (inf) are replaced by the time of
    the variant the dispatch falls back to.  `fallback` is either one universal variant id, or the library's
    per-variant links (fallback[v] = variant tried next when v is illegal; chains end at a legal variant)."""
    T = np.asarray(times, dtype=np.float64)
    if np.ndim(fallback) == 0:
        return np.where(np.isfinite(T), T, T[:, [int(fallback)]])
    link = np.asarray(fallback, dtype=np.int64)
    E = T.copy()
    for _ in range(T.shape[1]):  # every pass resolves at least one more hop of each chain
        bad = ~np.isfinite(E)
        if not bad.any():
            break
        E = np.where(bad, E[:, link], E)
    return E


def ratios(times, pred, fallback=0):
    """f_pred / f_best per row = t_best / t_pred (with the fallback rule)."""
    T = np.asarray(times, dtype=np.float64)
    E = effective_times(T, fallback)
    rows = np.arange(T.shape[0])
    return T.min(axis=1) / E[rows, np.asarray(pred)]


def dtpr(times, pred, fallback=0):
    return float(np.mean(ratios(times, pred, fallback)))


def geomean_ratio(times, pred, fallback=0):
    return float(np.exp(np.mean(np.log(ratios(times, pred, fallback)))))


def accuracy(pred, labels):
    return float(np.mean(np.asarray(pred) == np.asarray(labels)))


REGRET_SCALE = 1 << 20


def regret_costs(times, fallback=0):
    """Integer cost of running variant v on input s: round(-2^20 * log(t_best / t_v)), fallback-priced."""
    T = np.asarray(times, dtype=np.float64)
    return np.rint(-np.log(T.min(axis=1, keepdims=True) / effective_times(T, fallback)) * REGRET_SCALE).astype(np.int64)


class Tree:
    """Flat arrays: node i is a leaf iff feature[i] < 0."""

    def __init__(self):
        self.feature, self.threshold, self.left, self.right, self.label, self.n = [], [], [], [], [], []

    def _new(self, n):
        for a in (self.feature, self.threshold, self.left, self.right, self.label):
            a.append(-1)
        self.n.append(n)
        return len(self.n) - 1

    def apply(self, X):
        """Index of the leaf node every input ends in."""
        X = expand_features(X)
        feature, threshold = np.array(self.feature), np.array(self.threshold)
        left, right = np.array(self.left), np.array(self.right)
        node = np.zeros(X.shape[0], dtype=np.int64)
        active = feature[node] >= 0
        while active.any():
            f = feature[node[active]]
            go_left = X[active, f] <= threshold[node[active]]
            node[active] = np.where(go_left, left[node[active]], right[node[active]])
            active = feature[node] >= 0
        return node

    def predict(self, X):
        return np.array(self.label)[self.apply(X)]

    def stats(self):
        leaves = [i for i, f in enumerate(self.feature) if f < 0]

        def depth(i):
            return 0 if self.feature[i] < 0 else 1 + max(depth(self.left[i]), depth(self.right[i]))

        return {"leaves": len(leaves), "height": depth(0), "classes": sorted({self.label[i] for i in leaves}),
                "min_leaf_samples": min(self.n[i] for i in leaves)}

    def to_nested(self, payload=None):
        """Nested-dict form (same shape as the oracle's trees; used by tests and the code generator).
        `payload` maps leaf node index -> extra keys of that leaf (the cost lists of a forest member)."""
        def rec(i):
            if self.feature[i] < 0:
                leaf = {"leaf": int(self.label[i]), "n": int(self.n[i])}
                if payload is not None:
                    leaf.update(payload[i])
                return leaf
            return {"feature": int(self.feature[i]), "threshold": int(self.threshold[i]), "n": int(self.n[i]),
                    "left": rec(self.left[i]), "right": rec(self.right[i])}
        return rec(0)


def _best_split(X, y_idx, idx, n_classes, L_abs):
    """(feature, threshold) maximising SL/nL + SR/nR exactly, or None."""
    n = idx.size
    best = None  # (Fraction score, feature, threshold)
    for f in range(X.shape[1]):
        xs = X[idx, f]
        order = np.argsort(xs, kind="stable")
        xs = xs[order]
        ys = y_idx[idx][order]
        onehot = np.zeros((n, n_classes), dtype=np.int64)
        onehot[np.arange(n), ys] = 1
        cum = np.cumsum(onehot, axis=0)[:-1]  # counts left of a cut after position pos
        tot = cum[-1] + onehot[-1] if n > 1 else onehot[0]
        nL = np.arange(1, n, dtype=np.int64)
        nR = n - nL
        valid = (xs[:-1] != xs[1:]) & (nL >= L_abs) & (nR >= L_abs)
        if not valid.any():
            continue
        SL = np.sum(cum * cum, axis=1)
        SR = np.sum((tot - cum) ** 2, axis=1)
        score = SL / nL + SR / nR
        score[~valid] = -1.0
        top = score.max()
        cand = np.flatnonzero(valid & (score >= top * (1.0 - 1e-9)))
        for pos in cand:  # exact comparison among the float near-ties, in threshold order
            s = Fraction(int(SL[pos]), int(nL[pos])) + Fraction(int(SR[pos]), int(nR[pos]))
            if best is None or s > best[0]:
                best = (s, f, (int(xs[pos]) + int(xs[pos + 1])) // 2)
    return None if best is None else (best[1], best[2])


def _best_split_regret(X, cost, idx, L_abs):
    """(feature, threshold) minimising  min_v sum_left cost + min_v sum_right cost  (exact integers), or None."""
    n = idx.size
    best = None  # (score, feature, threshold)
    for f in range(X.shape[1]):
        xs = X[idx, f]
        order = np.argsort(xs, kind="stable")
        xs = xs[order]
        C = cost[idx][order]
        P = np.cumsum(C, axis=0)
        tot = P[-1]
        P = P[:-1]
        nL = np.arange(1, n, dtype=np.int64)
        valid = (xs[:-1] != xs[1:]) & (nL >= L_abs) & (n - nL >= L_abs)
        if not valid.any():
            continue
        score = P.min(axis=1) + (tot - P).min(axis=1)
        score[~valid] = np.iinfo(np.int64).max
        pos = int(np.argmin(score))  # first minimum = lowest threshold
        if best is None or score[pos] < best[0]:
            best = (int(score[pos]), f, (int(xs[pos]) + int(xs[pos + 1])) // 2)
    return None if best is None else (best[1], best[2])


def fit_cart(X, times, H=None, L=1, leaf_rule="majority", fallback=0, labels=None):
    """Grow a tree on the inputs X [n, 5] (expanded to the 13 features) and the timing table `times` [n, V]."""
    X = expand_features(X)
    T = np.asarray(times, dtype=np.float64)
    y = labels_from_table(T) if labels is None else np.asarray(labels, dtype=np.int64)
    classes, y_idx = np.unique(y, return_inverse=True)
    L_abs = min_samples_leaf(L, X.shape[0])
    logr = None
    if leaf_rule == "logratio":
        logr = np.log(T.min(axis=1, keepdims=True) / effective_times(T, fallback))
    cost = regret_costs(T, fallback) if leaf_rule == "regret" else None
    tree = Tree()

    def leaf_label(idx):
        if leaf_rule == "majority":
            cnt = np.bincount(y_idx[idx], minlength=classes.size)
            return int(classes[np.argmax(cnt)])  # first maximum = lowest id
        if leaf_rule == "regret":
            return int(np.argmin(np.sum(cost[idx], axis=0)))  # first minimum = lowest id
        return int(np.argmax(np.sum(logr[idx], axis=0)))

    def grow(idx, depth):
        node = tree._new(int(idx.size))
        if leaf_rule == "regret":
            pure = int(np.sum(cost[idx], axis=0).min()) == 0
        else:
            pure = np.all(y_idx[idx] == y_idx[idx[0]])
        sp = None
        if not pure and (H is None or depth < H) and idx.size >= 2 * L_abs:
            sp = (_best_split_regret(X, cost, idx, L_abs) if leaf_rule == "regret"
                  else _best_split(X, y_idx, idx, classes.size, L_abs))
        if sp is None:
            tree.label[node] = leaf_label(idx)
            return node
        f, thr = sp
        tree.feature[node], tree.threshold[node] = f, thr
        go_left = X[idx, f] <= thr
        tree.left[node] = grow(idx[go_left], depth + 1)
        tree.right[node] = grow(idx[~go_left], depth + 1)
        return node

    limit = sys.getrecursionlimit()
    sys.setrecursionlimit(max(limit, 20000))  # one Python frame per tree level; unbalanced trees run hundreds deep
    try:
        grow(np.arange(X.shape[0]), 0)
    finally:
        sys.setrecursionlimit(limit)
    return tree


def sweep(X_train, T_train, X_test, T_test, leaf_rule="majority", fallback=0, H_set=H_SET, L_set=L_SET):
    """One tree per (H, L) (Section 5): the per-model statistics the paper tabulates."""
    y_test = labels_from_table(T_test)
    rows = []
    for H in H_set:
        for L in L_set:
            tree = fit_cart(X_train, T_train, H, L, leaf_rule, fallback)
            pred = tree.predict(X_test)
            st = tree.stats()
            rows.append({"name": model_name(H, L), "H": H, "L": L, "leaf_rule": leaf_rule,
                         "accuracy": accuracy(pred, y_test), "dtpr": dtpr(T_test, pred, fallback),
                         "geomean": geomean_ratio(T_test, pred, fallback), "leaves": st["leaves"],
                         "height": st["height"], "classes": st["classes"], "tree": tree})
    return rows


def cross_predict(X, T, fit, folds=5):
    """Out-of-fold predictions: `folds` contiguous folds of the (already shuffled) training set; every row is
    predicted by the model `fit(X_train, T_train)` grown without its fold.  Returns one variant id per row."""
    X = np.asarray(X, dtype=np.int64)
    T = np.asarray(T, dtype=np.float64)
    n = X.shape[0]
    edges = np.linspace(0, n, folds + 1).astype(int)
    pred = np.empty(n, dtype=np.int64)
    for k in range(folds):
        test = np.arange(edges[k], edges[k + 1])
        train = np.concatenate([np.arange(0, edges[k]), np.arange(edges[k + 1], n)])
        pred[test] = fit(X[train], T[train]).predict(X[test])
    return pred


def cross_validate(X, T, H, L, leaf_rule, fallback=0, folds=5):
    """Geometric mean of the out-of-fold performance ratio (`folds` contiguous folds of the training set)."""
    pred = cross_predict(X, T, lambda Xa, Ta: fit_cart(Xa, Ta, H, L, leaf_rule, fallback), folds)
    return geomean_ratio(T, pred, fallback)


def select_model(X_train, T_train, fallback=0, folds=5, H_set=H_SET, L_set=L_SET,
                 leaf_rules=("majority", "logratio", "regret")):
    """Choose (H, L, leaf rule) by cross-validation inside the training set; the held-out set is not touched."""
    table = []
    for rule in leaf_rules:
        for H in H_set:
            for L in L_set:
                table.append({"name": model_name(H, L), "H": H, "L": L, "leaf_rule": rule,
                              "cv_geomean": cross_validate(X_train, T_train, H, L, rule, fallback, folds)})
    best = max(table, key=lambda r: r["cv_geomean"])  # first maximum in sweep order
    return best, table


FOREST_KEEP = 8
COST_CAP = 1 << 26


class Forest:
    """Trees plus, per tree, the leaf cost lists: ids[node, FOREST_KEEP] (-1 = unused), costs[node, FOREST_KEEP],
    rest[node]."""

    def __init__(self, trees, ids, costs, rest, n_variants):
        self.trees, self.ids, self.costs, self.rest, self.n_variants = trees, ids, costs, rest, n_variants

    def scores(self, X):
        X = expand_features(X)
        total = np.zeros((X.shape[0], self.n_variants), dtype=np.int64)
        rows = np.arange(X.shape[0])
        for tree, ids, costs, rest in zip(self.trees, self.ids, self.costs, self.rest):
            leaf = tree.apply(X)
            total += rest[leaf][:, None]
            for e in range(ids.shape[1]):
                v = ids[leaf, e]
                ok = v >= 0
                np.add.at(total, (rows[ok], v[ok]), costs[leaf, e][ok] - rest[leaf][ok])
        return total

    def predict(self, X):
        return np.argmin(self.scores(X), axis=1).astype(np.int64)  # first minimum = lowest id

    def stats(self):
        st = [t.stats() for t in self.trees]
        return {"trees": len(self.trees), "leaves": int(sum(s["leaves"] for s in st)),
                "height": int(max(s["height"] for s in st))}

    def to_nested(self):
        out = []
        for tree, ids, costs, rest in zip(self.trees, self.ids, self.costs, self.rest):
            payload = {}
            for i, f in enumerate(tree.feature):
                if f < 0:
                    keep = ids[i] >= 0
                    payload[i] = {"ids": [int(v) for v in ids[i][keep]], "costs": [int(c) for c in costs[i][keep]],
                                  "rest": int(rest[i])}
            out.append(tree.to_nested(payload))
        return out


def leaf_cost_lists(tree, X, cost):
    """Per leaf of `tree`: the FOREST_KEEP variants with the lowest mean cost over the rows of X (with their
    multiplicity) that end in the leaf, ordered by (mean cost, id), and the mean cost of the next one."""
    n_nodes, V = len(tree.n), cost.shape[1]
    keep = min(FOREST_KEEP, V)
    leaf = tree.apply(X)
    sums = np.zeros((n_nodes, V), dtype=np.int64)
    cnt = np.zeros(n_nodes, dtype=np.int64)
    np.add.at(sums, leaf, np.minimum(cost, COST_CAP))
    np.add.at(cnt, leaf, 1)
    mean = sums // np.maximum(cnt, 1)[:, None]
    order = np.argsort(mean, axis=1, kind="stable")  # stable: equal means stay in id order
    ids = np.full((n_nodes, FOREST_KEEP), -1, dtype=np.int64)
    costs = np.zeros((n_nodes, FOREST_KEEP), dtype=np.int64)
    ids[:, :keep] = order[:, :keep]
    costs[:, :keep] = np.take_along_axis(mean, order[:, :keep], axis=1)
    rest = np.take_along_axis(mean, order[:, [keep if keep < V else V - 1]], axis=1)[:, 0]
    return ids, costs, rest


def fit_forest(X, times, bootstrap, H=None, L=4, leaf_rule="logratio", fallback=0):
    """One tree per entry of `bootstrap` (arrays of row indices into X, drawn with replacement by the caller)."""
    X = expand_features(X)
    T = np.asarray(times, dtype=np.float64)
    cost = regret_costs(T, fallback)
    trees, ids, costs, rest = [], [], [], []
    for idx in bootstrap:
        idx = np.asarray(idx, dtype=np.int64)
        tree = fit_cart(X[idx], T[idx], H, L, leaf_rule, fallback)
        i, c, r = leaf_cost_lists(tree, X[idx], cost[idx])
        trees.append(tree), ids.append(i), costs.append(c), rest.append(r)
    return Forest(trees, ids, costs, rest, T.shape[1])


def cross_predict_forest(X, T, bootstrap_for, H, L, leaf_rule, fallback=0, folds=5):
    """Out-of-fold predictions of a forest; `bootstrap_for(n)` returns the bootstrap index arrays for n training rows."""
    return cross_predict(X, T, lambda Xa, Ta: fit_forest(Xa, Ta, bootstrap_for(Xa.shape[0]), H, L, leaf_rule, fallback), folds)


def cross_validate_forest(X, T, bootstrap_for, H, L, leaf_rule, fallback=0, folds=5):
    """As cross_validate, for a forest."""
    return geomean_ratio(T, cross_predict_forest(X, T, bootstrap_for, H, L, leaf_rule, fallback, folds), fallback)


# ---- cost of the selector itself (Section 3, requirement 2: the cost of selecting must be lower than the
# improvement, f_a-bar(i) + c_a-bar < f_a(i)) --------------------------------------------------------------------
# A forest predicts a little better than one tree and costs an order of magnitude more to evaluate; for a call
# of a few microseconds that cost exceeds what the better prediction saves.  The gated model lets the single tree
# answer inputs whose work M*N*K is below a gate G and the forest the others.  G is chosen on out-of-fold
# predictions with every predicted time charged the evaluation cost of the model that made it.

GATE_SET = (0,) + tuple(1 << e for e in range(20, 43)) + (INT64_MAX,)  # 0 = forest only, INT64_MAX = tree only


def selector_cost_ratios(times, pred, cost_seconds, fallback=0):
    """t_best / (t_pred + c) per row: the performance ratio with the selector's own cost charged to the model."""
    T = np.asarray(times, dtype=np.float64)
    E = effective_times(T, fallback)
    rows = np.arange(T.shape[0])
    return T.min(axis=1) / (E[rows, np.asarray(pred)] + np.asarray(cost_seconds, dtype=np.float64))


def gated_predict(X, gate, pred_tree, pred_forest):
    """Row-wise: the tree's prediction where M*N*K < gate, the forest's elsewhere."""
    work = expand_features(X)[:, FEATURES.index("MNK")]
    return np.where(work < int(gate), np.asarray(pred_tree), np.asarray(pred_forest)).astype(np.int64)


def choose_gate(X, T, pred_tree, pred_forest, tree_ns, forest_ns, fallback=0, gate_set=GATE_SET):
    """The gate with the highest cost-inclusive geomean ratio (first maximum in gate_set order), and the table
    of all candidates.  pred_tree / pred_forest are out-of-fold predictions for the rows of X."""
    work = expand_features(X)[:, FEATURES.index("MNK")]
    table = []
    for G in gate_set:
        by_tree = work < int(G)
        pred = np.where(by_tree, pred_tree, pred_forest)
        cost = np.where(by_tree, tree_ns, forest_ns) * 1e-9
        r = selector_cost_ratios(T, pred, cost, fallback)
        table.append({"gate": int(G), "geomean_with_cost": float(np.exp(np.mean(np.log(r)))),
                      "rows_by_tree": int(by_tree.sum())})
    best = max(table, key=lambda r: r["geomean_with_cost"])
    return best["gate"], table
