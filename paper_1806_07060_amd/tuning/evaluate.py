"""Off-line phase, last step: score the selector that is compiled into the library.

  python -m paper_1806_07060_amd.tuning.evaluate

Predictions come from the library itself (mdg_select / mdg_select_default
through the C ABI), so what is scored is the generated if-then-else, not the
Python tree.  Against the timing tables of the tuning run it reports, per
dataset (Section 5.2 of the paper):
  accuracy            right predictions / inputs
  DTPR                arithmetic mean of  f_model / f_peak   ("peak" = best variant of the exhaustive run)
  geomean             geometric mean of the same ratio (the figure this build is judged on)
  DTTR                mean of  f_model / f_default  (model against the traditional default dispatch)
  max speed-up        largest f_model / f_default
and the cost of evaluating the model next to the kernel times (end of Section 5.4; Section 3, requirement 2:
the cost of selecting counts against the selected routine), both for a fresh shape and for a shape the
per-thread memo in front of the model has seen.  The evaluation cost is measured on tens of thousands of
distinct seeded shapes (nothing for a branch predictor or a cache to remember from the previous pass), per side
of the gate when the model is a gated pair, and every ratio is also reported with that cost added to the
model's time: t_best / (t_model + c).
Writes results/selector_eval.json.
"""
import json
import os

import numpy as np

from . import cart
from .train import RESULTS, load_table, split
from .. import binding as mdg


def predict_with_library(X, default=False):
    fn = mdg.mdg_select_default if default else mdg.mdg_select
    return np.array([fn(int(r[3]), int(r[4]), int(r[0]), int(r[1]), int(r[2])) for r in X], dtype=np.int64)


def selector_cost_seconds(X, cost):
    """Seconds the compiled model takes on each input of X, from the measured per-evaluation costs in `cost`
    ({"gate": G or None, "ns_tree": ..., "ns_forest": ..., "ns": ...})."""
    if cost is None:
        return np.zeros(X.shape[0])
    if cost.get("gate") in (None, 0):
        return np.full(X.shape[0], cost["ns"] * 1e-9)
    work = cart.expand_features(X)[:, cart.FEATURES.index("MNK")]
    return np.where(work < cost["gate"], cost["ns_tree"], cost["ns_forest"]) * 1e-9


def measure_selector_cost(gate):
    """Host nanoseconds per evaluation of the compiled model on fresh shapes: over a sweep-like pool, and for a
    gated pair also per side of the gate."""
    from .. import workloads as wl
    timed = lambda P, it: mdg.mdg_time_select_ns(P[:, 3], P[:, 4], P[:, 0], P[:, 1], P[:, 2], iters=it)  # noqa: E731
    pool = wl.fresh_shapes(100000, 0)
    out = {"gate": gate, "ns": timed(pool, 3), "fresh_shapes": int(pool.shape[0])}
    if gate not in (None, 0):
        work = pool[:, 0] * pool[:, 1] * pool[:, 2]
        below = pool[work < gate]
        above = wl.fresh_shapes(50000, 1, log2_max_dim=14.0, max_flops=2 ** 44, min_work=gate)
        out["ns_tree"] = timed(below, 3) if below.shape[0] else out["ns"]
        out["ns_forest"] = timed(above, 3)
    return out


def score(X, T, fallback=None, cost=None):
    if fallback is None:
        fallback = [int(v["fallback"]) for v in mdg.variants()]
    pred = predict_with_library(X)
    dflt = predict_with_library(X, default=True)
    y = cart.labels_from_table(T)
    E = cart.effective_times(T, fallback)
    rows = np.arange(T.shape[0])
    t_model, t_default, t_best = E[rows, pred], E[rows, dflt], T.min(axis=1)
    r = t_best / t_model
    c = selector_cost_seconds(X, cost)
    rc = t_best / (t_model + c)
    return {
        "geomean_with_selector_cost": float(np.exp(np.mean(np.log(rc)))),
        "dtpr_with_selector_cost": float(np.mean(rc)),
        "selector_mean_pct_of_call": float(100 * np.mean(c / t_model)),
        "selector_max_pct_of_call": float(100 * np.max(c / t_model)),
        "inputs": int(T.shape[0]),
        "accuracy": cart.accuracy(pred, y),
        "dtpr": float(np.mean(r)),
        "geomean": float(np.exp(np.mean(np.log(r)))),
        "min_ratio": float(r.min()),
        "fallback_used": int(np.sum(~np.isfinite(T[rows, pred]))),
        "dttr": float(np.mean(t_default / t_model)),
        "dttr_geomean": float(np.exp(np.mean(np.log(t_default / t_model)))),
        "max_speedup_vs_default": float(np.max(t_default / t_model)),
        "default_geomean_vs_peak": float(np.exp(np.mean(np.log(t_best / t_default)))),
        "distinct_predicted": int(np.unique(pred).size),
        "distinct_best": int(np.unique(y).size),
    }


def main():
    mdg.lib()
    out = {"selector": mdg.mdg_selector_name(), "variants": mdg.mdg_variant_count(), "datasets": {}}
    gate = None
    mpath = os.path.join(RESULTS, "model.json")
    if os.path.exists(mpath):
        model = json.load(open(mpath))
        assert model["name"] == out["selector"], "results/model.json is not the model compiled into the library"
        gate = model.get("gate")
    cost = measure_selector_cost(gate)
    p4 = os.path.join(RESULTS, "timings_cfg4.csv")
    tab4 = load_table(p4)
    assert tab4["variants"] == [v["name"] for v in mdg.variants()], "timing table does not match the variant table"
    tr, te = split(tab4)
    out["datasets"]["random_sweep_train"] = score(tab4["X"][tr], tab4["T"][tr], cost=cost)
    out["datasets"]["random_sweep_heldout"] = score(tab4["X"][te], tab4["T"][te], cost=cost)
    for key, fn in (("square_sweep", "timings_cfg1.csv"), ("skinny_fc", "timings_cfg2.csv"),
                    ("conv_lowered", "timings_cfg3.csv")):
        p = os.path.join(RESULTS, fn)
        if os.path.exists(p):
            t = load_table(p)
            out["datasets"][key] = score(t["X"], t["T"], cost=cost)
    held = out["datasets"]["random_sweep_heldout"]
    out["heldout_geomean_pct"] = 100.0 * held["geomean"]
    out["heldout_geomean_with_selector_cost_pct"] = 100.0 * held["geomean_with_selector_cost"]
    out["heldout_dtpr"] = held["dtpr"]

    # the same 200 shapes over and over through the memo mdg_sgemm uses (every lookup after the first pass hits)
    Xte, Tte = tab4["X"][te], tab4["T"][te]
    pred = predict_with_library(Xte)
    t_model = cart.effective_times(Tte, [int(v["fallback"]) for v in mdg.variants()])[np.arange(Tte.shape[0]), pred]
    ns_memo = mdg.mdg_time_select_ns(Xte[:200, 3], Xte[:200, 4], Xte[:200, 0], Xte[:200, 1], Xte[:200, 2], iters=4000,
                                     memo=True)
    out["selector_overhead"] = {"fresh_shape": cost,
                                "mean_pct_of_call": held["selector_mean_pct_of_call"],
                                "max_pct_of_call": held["selector_max_pct_of_call"],
                                "ns_per_call_repeated_shape": ns_memo,
                                "mean_pct_of_call_repeated_shape": float(100 * (ns_memo * 1e-9 / t_model).mean()),
                                "max_pct_of_call_repeated_shape": float(100 * (ns_memo * 1e-9 / t_model).max())}
    for k, v in out["datasets"].items():
        print(f"{k:22s} n={v['inputs']:5d} acc={100 * v['accuracy']:5.1f}% DTPR={v['dtpr']:.3f} geomean={v['geomean']:.3f} "
              f"(with selector cost {v['geomean_with_selector_cost']:.3f}) min={v['min_ratio']:.2f} DTTR={v['dttr']:.3f} "
              f"max-speedup={v['max_speedup_vs_default']:.2f}x default/peak={v['default_geomean_vs_peak']:.3f}")
    so = out["selector_overhead"]
    print(f"selector: {out['selector']}  evaluation on fresh shapes {cost['ns']:.1f} ns"
          + (f" (tree side {cost['ns_tree']:.1f} ns, forest side {cost['ns_forest']:.1f} ns)" if "ns_tree" in cost else "")
          + f" = {so['mean_pct_of_call']:.3f}% of a held-out call on average (max {so['max_pct_of_call']:.3f}%); "
          f"repeated shape (memo hit) {ns_memo:.1f} ns = {so['mean_pct_of_call_repeated_shape']:.3f}% "
          f"(max {so['max_pct_of_call_repeated_shape']:.3f}%)")
    with open(os.path.join(RESULTS, "selector_eval.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
