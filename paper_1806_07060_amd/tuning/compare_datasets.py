"""Which training set makes the best selector?  (Section 5 of the paper compares models learned from a dense
grid, a sparse power-of-two grid and a real-world set.)

  python -m paper_1806_07060_amd.tuning.compare_datasets

Trains the same model family (every (H, L) pair, both leaf rules, the pair chosen by cross-validation inside
the training set) on each synthetic dataset alone and on their union, and scores every resulting tree on the
same test sets: the held-out 20 % of the random sweep, and the square / skinny / convolution-lowered sets that
no training set contains.  Reports accuracy, DTPR (arithmetic mean of f_model / f_peak) and the geometric mean
of the same ratio.  Writes results/dataset_comparison.json.
"""
import json
import os

import numpy as np

from . import cart
from .train import RESULTS, load_table, split, training_union


def _load(name):
    p = os.path.join(RESULTS, f"timings_{name}.csv")
    return load_table(p) if os.path.exists(p) else None


def main(folds=5):
    tab4 = _load("cfg4")
    tr, te = split(tab4)
    tests = {"random_sweep_heldout": (tab4["X"][te], tab4["T"][te])}
    excl = []
    for key, name in (("square_sweep", "cfg1"), ("skinny_fc", "cfg2"), ("conv_lowered", "cfg3")):
        t = _load(name)
        if t is not None:
            tests[key] = (t["X"], t["T"])
            excl.append(t)
    extras = {n: _load(n) for n in ("go2", "po2", "wide", "big", "large", "thin", "flat", "tgrid", "fgrid", "sweep2", "thin2", "flat2", "sweep3", "thin3", "flat3", "tgrid2")}
    extras = {n: t for n, t in extras.items() if t is not None}
    banned = set()
    for t in excl:
        banned |= {tuple(r[:3]) for r in t["X"].tolist()}

    def only(t):
        keep = np.array([tuple(r[:3]) not in banned for r in t["X"].tolist()], dtype=bool)
        return t["X"][keep], t["T"][keep]

    trainsets = {"random_sweep_train": (tab4["X"][tr], tab4["T"][tr])}
    for n, t in extras.items():
        trainsets[n] = only(t)
    Xu, Tu, _ = training_union(tab4, list(extras.items()), excl)
    trainsets["union"] = (Xu, Tu)

    from .. import binding as mdg
    links = [int(v["fallback"]) for v in mdg.variants()]
    out = {}
    print(f"{'training set':20s} {'n':>5s} {'model':22s} " + " ".join(f"{k[:18]:>18s}" for k in tests))
    for name, (X, T) in trainsets.items():
        best, _ = cart.select_model(X, T, fallback=links, folds=folds)
        tree = cart.fit_cart(X, T, best["H"], best["L"], best["leaf_rule"], links)
        st = tree.stats()
        row = {"inputs": int(X.shape[0]), "model": f"{best['name']}/{best['leaf_rule']}", "cv_geomean": best["cv_geomean"],
               "leaves": st["leaves"], "height": st["height"], "scores": {}}
        cells = []
        for k, (Xt, Tt) in tests.items():
            pred = tree.predict(Xt)
            sc = {"accuracy": cart.accuracy(pred, cart.labels_from_table(Tt)), "dtpr": cart.dtpr(Tt, pred, links),
                  "geomean": cart.geomean_ratio(Tt, pred, links)}
            row["scores"][k] = sc
            cells.append(f"{100 * sc['accuracy']:4.0f}% {sc['dtpr']:.3f} {sc['geomean']:.3f}")
        out[name] = row
        print(f"{name:20s} {X.shape[0]:5d} {row['model']:22s} " + " ".join(f"{c:>18s}" for c in cells))
    with open(os.path.join(RESULTS, "dataset_comparison.json"), "w") as f:
        json.dump(out, f, indent=1)
    return out


if __name__ == "__main__":
    main()
