"""How small can the training set be?  (The paper's conclusion names the cost of building the dataset as the
price of the approach and asks for more compact datasets; Section 5 shows a 216-point power-of-two grid doing
almost as well as a 3375-point one inside its own range.)

  python -m paper_1806_07060_amd.tuning.compaction

The training union is already in seeded random order, so a prefix of it is a uniform subsample of every
generation rule at once.  For each fraction one tree with the shipped hyper-parameters (H, L and leaf rule
read from results/model.json; a single tree also when the shipped selector is a forest of such trees) is
trained on that prefix and scored on the usual test sets:
the held-out 20 % of the random sweep and the square / skinny / convolution-lowered sets no training set
contains.  Also reports what the prefix cost to measure: the sum of the recorded times of every legal variant
on its inputs (one call each; the tuning run spends a small multiple of that).  Writes results/compaction.json.
"""
import json
import os

import numpy as np

from . import cart
from .train import RESULTS, load_table, split, training_union

FRACTIONS = (1.0, 0.5, 0.25, 0.125, 0.0625, 0.03125, 0.015625)
EXTRA = ("go2", "wide", "po2", "big", "large", "thin", "flat", "tgrid", "fgrid", "sweep2", "thin2", "flat2", "sweep3", "thin3", "flat3", "tgrid2")  # the order train.py joins them in


def _load(name):
    p = os.path.join(RESULTS, f"timings_{name}.csv")
    return load_table(p) if os.path.exists(p) else None


def main():
    with open(os.path.join(RESULTS, "model.json")) as f:
        model = json.load(f)
    H, L, rule = model["H"], model["L"], model["leaf_rule"]
    tab4 = _load("cfg4")
    tr, te = split(tab4)
    tests = {"random_sweep_heldout": (tab4["X"][te], tab4["T"][te])}
    excl = []
    for key, name in (("square_sweep", "cfg1"), ("skinny_fc", "cfg2"), ("conv_lowered", "cfg3")):
        t = _load(name)
        if t is not None:
            tests[key] = (t["X"], t["T"])
            excl.append(t)
    extras = [(n, _load(n)) for n in EXTRA]
    extras = [(n, t) for n, t in extras if t is not None]
    X, T, _ = training_union(tab4, extras, excl)

    from .. import binding as mdg
    links = [int(v["fallback"]) for v in mdg.variants()]
    name = f"{cart.model_name(H, L)}/{rule}"  # one tree with the shipped hyper-parameters, also when a forest ships
    out = {"model": name, "rows": []}
    print(f"model {name} (single tree); full training set {X.shape[0]} inputs")
    print(f"{'fraction':>9s} {'inputs':>6s} {'leaves':>6s} {'one pass s':>10s} " + " ".join(f"{k[:20]:>20s}" for k in tests))
    for frac in FRACTIONS:
        n = max(8, int(round(frac * X.shape[0])))
        Xs, Ts = X[:n], T[:n]
        tree = cart.fit_cart(Xs, Ts, H, L, rule, links)
        row = {"fraction": frac, "inputs": n, "leaves": tree.stats()["leaves"],
               "one_pass_seconds": float(np.sum(Ts[np.isfinite(Ts)])), "scores": {}}
        cells = []
        for k, (Xt, Tt) in tests.items():
            pred = tree.predict(Xt)
            row["scores"][k] = {"dtpr": cart.dtpr(Tt, pred, links), "geomean": cart.geomean_ratio(Tt, pred, links)}
            cells.append(f"{row['scores'][k]['geomean']:.3f}")
        out["rows"].append(row)
        print(f"{frac:9.4f} {n:6d} {row['leaves']:6d} {row['one_pass_seconds']:10.1f} " + " ".join(f"{c:>20s}" for c in cells))
    with open(os.path.join(RESULTS, "compaction.json"), "w") as f:
        json.dump(out, f, indent=1)
    return out


if __name__ == "__main__":
    main()
