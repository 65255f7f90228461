"""Selector oracle -- TEST INFRASTRUCTURE, never imported by the product.

Plain-Python statement of the off-line phase of the paper (Section 3,
'Framework design and workflow', 'Datasets', 'Model and code generation';
Section 4.2; metrics of Section 5.2), step by step and in the paper's notation:

  dataset D        a table T[s][v] of measured seconds of variant v on input s
                   (+inf where v cannot run on s); FLOPS f = 2 M N K / T
  a-bar(s)         argmax_a f_a(s): the best variant of each input (the label)
  X, Y             first 80 % / last 20 % of the (already shuffled) inputs
  CART             binary decision tree on integer features of I = (M, N, K, tA, tB):
                   the raw values plus M*N, M*N*K and the padding a grid of 32-, 64- or
                   128-wide tiles adds to M and to N (expand_features; the paper uses
                   the raw triple only -- the derived values are this build's addition)
                   grown with the Gini impurity, limited by H (maximum height,
                   None = unlimited) and L (minimum samples per leaf: an integer,
                   or a fraction in (0, 1) of the training samples)
  forest           several such trees, each grown on a bootstrap sample whose row indices are an
                   input; leaves list the mean integer cost of their cheapest variants and the
                   forest predicts the variant with the smallest summed cost (see 'forest' below)
  gated model      the single tree for inputs whose work M*N*K is below a gate, the forest for the
                   others; the gate maximises the ratio metric with each model's evaluation time
                   charged to its predictions (cost-effectiveness, Section 3 requirement 2)
  accuracy         right predictions / test instances
  DTPR             mean over the test inputs of f_pred(s) / f_best(s)

Readings where the paper is silent or ambiguous:
  - fractional L means ceil(L * n_train) samples (scikit-learn's meaning);
  - a node is split whenever it is impure, below height H, and some split leaves
    at least L samples on both sides -- also when the split does not lower the
    impurity (as scikit-learn does), which XOR-like labels need;
  - candidate thresholds: midpoints of consecutive distinct values, stored as
    floor(midpoint) and tested as  feature <= threshold  (features are integers);
  - ties between equally good splits: lowest feature index, then lowest threshold
    (scikit-learn randomises; only behaviour, not structure, is comparable);
  - majority ties at a leaf: lowest variant id;
  - a predicted variant that is illegal for an input is replaced by a fallback
    variant -- one universal variant, or per-variant links followed until a
    legal variant is reached -- and the fallback's time is what the ratio sees;
  - besides the arithmetic mean (the paper's DTPR) the geometric mean is reported;
  - leaf labels: 'majority' (plain CART) or 'logratio' (the variant maximising
    the summed log performance ratio of the leaf's training inputs -- uses the
    whole table; answers the misclassification-cost issue raised in Section 5.2);
  - 'regret' (an extension in the direction of the paper's future work, not in
    the paper): integer costs c[s][v] = round(-2^20 * log(performance ratio)),
    cost of a node = min over v of the column sum over its inputs, a split
    minimises the summed cost of its children (ties: lowest feature, lowest
    threshold), a node of cost 0 is a leaf, the label is the minimising variant.

All split comparisons are done in exact rational arithmetic, so the tree is a
pure function of the data and the rules above.

Pins (tests, CPU only): hand-computed toy trees, structural invariants that
hold for any data (leaves <= 2^H, leaves <= floor(1/L), samples per leaf >= L,
DTPR <= 1, a fully grown tree reproduces its training labels), depth-0 tree =
most frequent label, and scikit-learn's CART where no ties occur.
"""
from fractions import Fraction
import math

FEATURE_NAMES = ("M", "N", "K", "tA", "tB", "MN", "MNK", "padM32", "padM64", "padM128", "padN32", "padN64", "padN128")
INT64_MAX = 2 ** 63 - 1


def expand_features(x):
    """Input description (M, N, K, tA, tB) -> the thirteen tree features: the five raw values, the size of C
    (M*N) and the work (M*N*K), the products saturating at 2^63 - 1 like the 64-bit code that evaluates the tree,
    and how many rows (columns) a grid of 32-, 64-, 128-wide tiles adds beyond M (N): 0 for an exact multiple."""
    M, N, K, tA, tB = x
    pad = []
    for size in (M, N):
        for width in (32, 64, 128):
            tiles = -(-size // width)  # ceiling
            pad.append(tiles * width - size)
    return (M, N, K, tA, tB, min(M * N, INT64_MAX), min(M * N * K, INT64_MAX)) + tuple(pad)


# ----- labelling ---------------------------------------------------------------------------

def best_variant(times_row):
    """a-bar = argmax_a f_a(i) = the variant with the smallest time; ties -> lowest id."""
    best, best_t = -1, math.inf
    for v, t in enumerate(times_row):
        if t < best_t:
            best, best_t = v, t
    return best


def labels_from_table(times):
    return [best_variant(row) for row in times]


def min_samples_leaf(L, n_train):
    """L as an absolute sample count: integers as they are, fractions as ceil(L * n)."""
    if isinstance(L, float) and 0.0 < L < 1.0:
        return max(1, math.ceil(Fraction(L).limit_denominator(1000) * n_train))
    return max(1, int(L))


# ----- CART --------------------------------------------------------------------------------

def _counts(y):
    c = {}
    for lab in y:
        c[lab] = c.get(lab, 0) + 1
    return c


def _majority(y):
    c = _counts(y)
    top = max(c.values())
    return min(lab for lab, n in c.items() if n == top)


def _best_split(X, y, idx, L_abs):
    """Lowest weighted Gini over all (feature, threshold); None if no split leaves L_abs on each side.

    Weighted Gini of a split = (nL/n) (1 - sum_c pL_c^2) + (nR/n) (1 - sum_c pR_c^2)
                             = 1 - (SL/nL + SR/nR) / n   with S = sum of squared class counts,
    so the best split maximises SL/nL + SR/nR (exact rationals).
    """
    n = len(idx)
    best = None  # (score, feature, threshold)
    n_features = len(X[0])
    for f in range(n_features):
        order = sorted(idx, key=lambda s: X[s][f])
        left, right = {}, _counts([y[s] for s in order])
        SL, SR = 0, sum(v * v for v in right.values())
        for pos in range(n - 1):
            s = order[pos]
            c = y[s]
            cl, cr = left.get(c, 0), right[c]
            SL += 2 * cl + 1
            SR -= 2 * cr - 1
            left[c], right[c] = cl + 1, cr - 1
            a, b = X[s][f], X[order[pos + 1]][f]
            if a == b:
                continue
            nL, nR = pos + 1, n - pos - 1
            if nL < L_abs or nR < L_abs:
                continue
            score = Fraction(SL, nL) + Fraction(SR, nR)
            thr = (a + b) // 2
            if best is None or score > best[0]:
                best = (score, f, thr)
            # equal score: keep the earlier (lower feature, lower threshold) candidate
    return best


REGRET_SCALE = 2 ** 20


def regret_cost_rows(rows, fallback=0):
    """Integer cost of every (input, variant): round(-2^20 * log(f_v / f_best)), fallback-priced."""
    return [[round(-math.log(performance_ratio(r, v, fallback)) * REGRET_SCALE) for v in range(len(r))] for r in rows]


def _node_cost(cost, idx):
    n_var = len(cost[0])
    return min(sum(cost[s][v] for s in idx) for v in range(n_var))


def _node_label_regret(cost, idx):
    n_var = len(cost[0])
    sums = [sum(cost[s][v] for s in idx) for v in range(n_var)]
    return sums.index(min(sums))


def _best_split_regret(X, cost, idx, L_abs):
    """Lowest  cost(left) + cost(right)  over all (feature, threshold); None if no split is allowed."""
    n, n_var = len(idx), len(cost[0])
    best = None  # (score, feature, threshold)
    for f in range(len(X[0])):
        order = sorted(idx, key=lambda s: X[s][f])
        left = [0] * n_var
        right = [sum(cost[s][v] for s in order) for v in range(n_var)]
        for pos in range(n - 1):
            s = order[pos]
            for v in range(n_var):
                left[v] += cost[s][v]
                right[v] -= cost[s][v]
            a, b = X[s][f], X[order[pos + 1]][f]
            if a == b or pos + 1 < L_abs or n - pos - 1 < L_abs:
                continue
            score = min(left) + min(right)
            if best is None or score < best[0]:
                best = (score, f, (a + b) // 2)
    return best


def fit_cart(X, y, H=None, L=1, leaf_rule="majority", table=None, fallback=0):
    """Grow the tree. X: list of integer feature tuples, y: list of labels.

    leaf_rule 'logratio' needs `table` (times of every variant for the same
    rows as X) and `fallback`.
    Returns nested dicts: {'feature', 'threshold', 'left', 'right', 'n'} or {'leaf': label, 'n': samples}.
    """
    L_abs = min_samples_leaf(L, len(X))
    cost = regret_cost_rows(table, fallback) if leaf_rule == "regret" else None

    def leaf(idx):
        if leaf_rule == "majority":
            lab = _majority([y[s] for s in idx])
        elif leaf_rule == "regret":
            lab = _node_label_regret(cost, idx)
        else:
            lab = logratio_label([table[s] for s in idx], fallback)
        return {"leaf": lab, "n": len(idx)}

    def grow(idx, depth):
        if leaf_rule == "regret":
            pure = _node_cost(cost, idx) == 0
        else:
            pure = len(set(y[s] for s in idx)) == 1
        if pure or (H is not None and depth >= H) or len(idx) < 2 * L_abs:
            return leaf(idx)
        sp = _best_split_regret(X, cost, idx, L_abs) if leaf_rule == "regret" else _best_split(X, y, idx, L_abs)
        if sp is None:
            return leaf(idx)
        _, f, thr = sp
        li = [s for s in idx if X[s][f] <= thr]
        ri = [s for s in idx if X[s][f] > thr]
        return {"feature": f, "threshold": thr, "n": len(idx), "left": grow(li, depth + 1),
                "right": grow(ri, depth + 1)}

    return grow(list(range(len(X))), 0)


def predict(tree, x):
    node = tree
    while "leaf" not in node:
        node = node["left"] if x[node["feature"]] <= node["threshold"] else node["right"]
    return node["leaf"]


# ----- forest ------------------------------------------------------------------------------
# Bagging (one of the "more effective models" the paper's conclusion leaves to future work): tree t is grown on
# the rows bootstrap[t] of the training set (indices drawn with replacement by the caller -- this module draws
# no random numbers).  Leaves do not vote for a class; each carries the mean cost of its cheapest variants.

FOREST_KEEP = 8
COST_CAP = 2 ** 26


def _leaf_of(tree, x):
    node = tree
    while "leaf" not in node:
        node = node["left"] if x[node["feature"]] <= node["threshold"] else node["right"]
    return node


def attach_leaf_costs(tree, X, cost_rows):
    """For every leaf: mean cost (floor of sum / count, each cost capped at COST_CAP) of every variant over the
    rows that end in the leaf; the FOREST_KEEP variants with the lowest (mean, id) are listed with their means
    ('ids', 'costs'), and 'rest' is the mean of the next one in that order (of the last one if none is left)."""
    sums = {}
    for x, c in zip(X, cost_rows):
        leaf = _leaf_of(tree, x)
        acc = sums.setdefault(id(leaf), (leaf, [0] * len(c), [0]))
        for v, cv in enumerate(c):
            acc[1][v] += min(cv, COST_CAP)
        acc[2][0] += 1
    for leaf, total, count in sums.values():
        mean = [t // count[0] for t in total]
        order = sorted(range(len(mean)), key=lambda v: (mean[v], v))
        kept = order[:FOREST_KEEP]
        leaf["ids"] = kept
        leaf["costs"] = [mean[v] for v in kept]
        leaf["rest"] = mean[order[FOREST_KEEP]] if len(order) > FOREST_KEEP else mean[order[-1]]
    return tree


def fit_forest(X, y, table, bootstrap, H=None, L=4, leaf_rule="logratio", fallback=0):
    cost = regret_cost_rows(table, fallback)
    trees = []
    for idx in bootstrap:
        Xb, yb, Tb = [X[i] for i in idx], [y[i] for i in idx], [table[i] for i in idx]
        tree = fit_cart(Xb, yb, H, L, leaf_rule, Tb, fallback)
        trees.append(attach_leaf_costs(tree, Xb, [cost[i] for i in idx]))
    return trees


def forest_scores(trees, x, n_variants):
    """Summed cost of every variant: a tree contributes the listed mean cost of its leaf, or the leaf's 'rest'."""
    total = [0] * n_variants
    for tree in trees:
        leaf = _leaf_of(tree, x)
        listed = dict(zip(leaf["ids"], leaf["costs"]))
        for v in range(n_variants):
            total[v] += listed.get(v, leaf["rest"])
    return total


def predict_forest(trees, x, n_variants):
    total = forest_scores(trees, x, n_variants)
    return total.index(min(total))  # first minimum = lowest id


# ----- the selector's own cost ---------------------------------------------------------------
# Section 3, requirement 2 (cost-effectiveness): the time to select a-bar counts against it,
# f_a-bar(i) + c_a-bar < f_a(i).  A forest costs an order of magnitude more to evaluate than one tree, so a
# gated model lets the tree answer the inputs whose work M*N*K is below a gate and the forest the others.

def predict_gated(tree, trees, gate, x, n_variants):
    """x = expanded feature tuple (x[6] = M*N*K): the single tree below the gate, the forest at or above it."""
    return predict(tree, x) if x[6] < gate else predict_forest(trees, x, n_variants)


def ratio_with_selector_cost(times_row, v, cost_seconds, fallback=0):
    """t_best / (t_v + c): the performance ratio when the model that predicted v took cost_seconds to evaluate."""
    return times_row[best_variant(times_row)] / (effective_time(times_row, v, fallback) + cost_seconds)


def choose_gate(X, times, pred_tree, pred_forest, tree_ns, forest_ns, gate_set, fallback=0):
    """The gate of gate_set (first maximum in its order) with the highest geometric mean of the cost-inclusive
    ratio, given each model's prediction for every row of X (expanded feature tuples)."""
    best, best_score = None, -math.inf
    for G in gate_set:
        logs = []
        for x, row, pt, pf in zip(X, times, pred_tree, pred_forest):
            if x[6] < G:
                logs.append(math.log(ratio_with_selector_cost(row, pt, tree_ns * 1e-9, fallback)))
            else:
                logs.append(math.log(ratio_with_selector_cost(row, pf, forest_ns * 1e-9, fallback)))
        score = math.exp(math.fsum(logs) / len(logs))
        if score > best_score:
            best, best_score = G, score
    return best, best_score


def tree_stats(tree):
    """Leaves, height and distinct predicted variants (the per-model columns of the paper's tables)."""
    leaves, height, classes, min_n = 0, 0, set(), None
    stack = [(tree, 0)]
    while stack:
        node, d = stack.pop()
        if "leaf" in node:
            leaves += 1
            height = max(height, d)
            classes.add(node["leaf"])
            min_n = node["n"] if min_n is None else min(min_n, node["n"])
        else:
            stack.append((node["left"], d + 1))
            stack.append((node["right"], d + 1))
    return {"leaves": leaves, "height": height, "classes": sorted(classes), "min_leaf_samples": min_n}


# ----- metrics -----------------------------------------------------------------------------

def effective_time(times_row, v, fallback=0):
    """Seconds the library would really spend when variant v is predicted.

    `fallback` is one universal variant id, or a list of links (fallback[v] = the variant tried next when v is
    illegal for the input): links are followed until a variant with a finite time is found.
    """
    if isinstance(fallback, int):
        t = times_row[v]
        return t if math.isfinite(t) else times_row[fallback]
    for _ in range(len(times_row) + 1):
        if math.isfinite(times_row[v]):
            return times_row[v]
        v = fallback[v]
    raise ValueError("fallback links never reach a legal variant")


def performance_ratio(times_row, v, fallback=0):
    """f_v(s) / f_best(s) = t_best / t_v  (same flop count cancels)."""
    return times_row[best_variant(times_row)] / effective_time(times_row, v, fallback)


def logratio_label(rows, fallback=0):
    """Variant maximising sum over rows of log(performance ratio); ties -> lowest id."""
    n_var = len(rows[0])
    best, best_s = -1, -math.inf
    for v in range(n_var):
        s = math.fsum(math.log(performance_ratio(r, v, fallback)) for r in rows)
        if s > best_s:
            best, best_s = v, s
    return best


def accuracy(pred, labels):
    return sum(1 for p, l in zip(pred, labels) if p == l) / len(labels)


def dtpr(times, pred, fallback=0):
    """Arithmetic mean of the performance ratio (the paper's DTPR)."""
    return math.fsum(performance_ratio(r, p, fallback) for r, p in zip(times, pred)) / len(pred)


def geomean_ratio(times, pred, fallback=0):
    return math.exp(math.fsum(math.log(performance_ratio(r, p, fallback)) for r, p in zip(times, pred)) / len(pred))


def model_name(H, L):
    return f"h{'Max' if H is None else H}-L{L}"


H_SET = (1, 2, 4, 8, None)
L_SET = (1, 2, 4, 0.1, 0.2, 0.3, 0.4, 0.5)


def sweep(X_train, T_train, X_test, T_test, leaf_rule="majority", fallback=0, H_set=H_SET, L_set=L_SET):
    """One tree per (H, L) pair (Section 5): name, accuracy, DTPR, geomean, leaves, height."""
    y_train = labels_from_table(T_train)
    y_test = labels_from_table(T_test)
    rows = []
    for H in H_set:
        for L in L_set:
            tree = fit_cart(X_train, y_train, H, L, leaf_rule, T_train, fallback)
            pred = [predict(tree, x) for x in X_test]
            st = tree_stats(tree)
            rows.append({"name": model_name(H, L), "H": H, "L": L, "accuracy": accuracy(pred, y_test),
                         "dtpr": dtpr(T_test, pred, fallback), "geomean": geomean_ratio(T_test, pred, fallback),
                         "leaves": st["leaves"], "height": st["height"], "tree": tree})
    return rows
