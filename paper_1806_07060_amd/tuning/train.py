"""Off-line phase, steps 2-3 as a command: timing table -> trees -> chosen model -> generated C++.

  python -m paper_1806_07060_amd.tuning.train [--table results/timings_cfg4.csv]

Reads the dataset written by the tuning run, takes the first 80 % of its
(already shuffled) rows as the training set X and the rest as the held-out set
Y (Section 3, 'Datasets'), trains one tree per (H, L) pair of Section 5 for
every leaf rule and prints the table of model statistics the paper reports
(accuracy, DTPR, leaves, height) on Y.  Further synthetic tables (--extra: the
go2 and po2 grids of Section 4.1, wider sweeps, grids and sweeps over the thin
and flat corners) are added to X only -- a
hybrid of several generation rules, as Section 3 allows -- after dropping any
input whose (M, N, K) occurs in the square, skinny or convolution-lowered
evaluation sets, which stay unseen.  The model that is compiled into the
library is chosen by 5-fold cross-validation inside X -- the paper picks the
best DTPR on the test set itself, which leaks; Y is only used for reporting.
A forest of bagged trees with the chosen hyper-parameters (--forest-trees) is
cross-validated the same way.  What ships is the gated pair of both: the tree
answers inputs whose work M*N*K is below a gate, the forest the others, and the
gate is the one that maximises the out-of-fold ratio with the evaluation time of
the answering model (--tree-ns, --forest-ns: measured host nanoseconds per
evaluation) added to every predicted time -- Section 3, requirement 2: the cost
of selecting must stay below the improvement.  Gate 0 ships the forest alone,
an infinite gate the tree alone.
Then writes csrc/mdg_select_generated.h and results/model.json.  Rebuild the
library afterwards.
"""
import argparse
import csv
import json
import os

import numpy as np

from . import cart, codegen

HERE = os.path.dirname(os.path.abspath(__file__))
RESULTS = os.path.join(HERE, "results")


def load_table(path):
    """-> dict(index, names, X [n,5] int64, alpha, beta, T [n,V] seconds, variants [V] names)."""
    with open(path) as f:
        rows = list(csv.reader(f))
    hdr, rows = rows[0], [r for r in rows[1:] if r]
    rows.sort(key=lambda r: int(r[0]))
    return {
        "index": np.array([int(r[0]) for r in rows]),
        "names": [r[1] for r in rows],
        "X": np.array([[int(r[2]), int(r[3]), int(r[4]), int(r[5]), int(r[6])] for r in rows], dtype=np.int64),
        "alpha": np.array([float(r[7]) for r in rows]),
        "beta": np.array([float(r[8]) for r in rows]),
        "T": np.array([[float(x) for x in r[9:]] for r in rows], dtype=np.float64),
        "variants": hdr[9:],
    }


def split(table, train_fraction=0.8):
    n = table["X"].shape[0]
    n_train = int(round(train_fraction * n))
    return slice(0, n_train), slice(n_train, n)


def training_union(tab4, extra_tables, exclude_tables, seed=180607060):
    """X = first 80 % of the random sweep + the extra tables, minus shapes of the excluded tables and of the
    held-out 20 % of the sweep; shuffled."""
    tr, te = split(tab4)
    Xs, Ts, src = [tab4["X"][tr]], [tab4["T"][tr]], ["cfg4"] * tab4["X"][tr].shape[0]
    banned = {tuple(r[:3]) for r in tab4["X"][te].tolist()}  # a held-out (M, N, K) may not come back through an extra table
    for t in exclude_tables:
        banned |= {tuple(r[:3]) for r in t["X"].tolist()}
    for name, t in extra_tables:
        keep = np.array([tuple(r[:3]) not in banned for r in t["X"].tolist()], dtype=bool)
        Xs.append(t["X"][keep])
        Ts.append(t["T"][keep])
        src += [name] * int(keep.sum())
    X, T = np.vstack(Xs), np.vstack(Ts)
    held = {tuple(r[:3]) for r in tab4["X"][te].tolist()}
    assert not any(tuple(r[:3]) in held for x in Xs[1:] for r in x.tolist()), "held-out inputs leaked into the training set"
    perm = np.random.Generator(np.random.PCG64(seed)).permutation(X.shape[0])
    return X[perm], T[perm], [src[i] for i in perm]


def fallback_links(variants_meta):
    """fallback[v] for every variant, as the library reports them (mdg_variant_info)."""
    return [int(m["fallback"]) for m in variants_meta]


def default_dispatch(cfg1_table, variants_meta):
    """The traditional configuration (Section 5, 'default'): the tiled variant that is best on the 1024-cube
    and the direct variant that is best on the 256-cube (summed log time over the four transpose cases),
    switched at M*N*K = 512^3."""
    X, T = cfg1_table["X"], cfg1_table["T"]
    fam = np.array([m["family"] for m in variants_meta])
    split_k = np.array([m["split_k"] for m in variants_meta])

    def best(size, mask):
        rows = np.flatnonzero((X[:, 0] == size) & (X[:, 1] == size) & (X[:, 2] == size))
        score = np.sum(np.log(T[rows]), axis=0)
        score[~mask | ~np.all(np.isfinite(T[rows]), axis=0)] = np.inf
        return int(np.argmin(score))

    tiled = best(1024, (fam == 1) & (split_k == 1))
    direct = best(256, fam == 0)
    return tiled, direct, 512.0 ** 3


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--table", default=os.path.join(RESULTS, "timings_cfg4.csv"))
    ap.add_argument("--cfg1", default=os.path.join(RESULTS, "timings_cfg1.csv"))
    ap.add_argument("--extra", nargs="*", default=["timings_go2.csv", "timings_wide.csv", "timings_po2.csv", "timings_big.csv", "timings_large.csv",
                                                      "timings_thin.csv", "timings_flat.csv", "timings_tgrid.csv", "timings_fgrid.csv",
                                                      "timings_sweep2.csv", "timings_thin2.csv", "timings_flat2.csv",
                                                      "timings_sweep3.csv", "timings_thin3.csv", "timings_flat3.csv", "timings_tgrid2.csv"],
                    help="further tables (file names under results/) whose inputs join the training set")
    ap.add_argument("--exclude", nargs="*", default=["timings_cfg1.csv", "timings_cfg2.csv", "timings_cfg3.csv"],
                    help="tables whose shapes must stay out of the training set")
    ap.add_argument("--folds", type=int, default=5)
    ap.add_argument("--forest-trees", type=int, default=12,
                    help="also cross-validate a forest of this many bagged trees with the chosen (H, L, leaf rule) and "
                         "ship it instead of the single tree if it scores higher (0 = single tree only)")
    ap.add_argument("--tree-ns", type=float, default=32.0,
                    help="host nanoseconds per evaluation of the single tree (if-then-else), fresh shapes")
    ap.add_argument("--forest-ns", type=float, default=490.0,
                    help="host nanoseconds per evaluation of the forest (table walk), fresh shapes")
    ap.add_argument("--leaf-rules", nargs="*", default=["majority", "logratio", "regret"],
                    help="leaf rules to sweep (the cost-sensitive splits of `regret` grow chain-like trees for L = 1 on "
                         "tens of thousands of inputs and take hours; leave it out there)")
    ap.add_argument("--no-write", action="store_true")
    args = ap.parse_args(argv)

    tab = load_table(args.table)
    tr, te = split(tab)
    Xte, Tte = tab["X"][te], tab["T"][te]
    extras = [(os.path.splitext(f)[0].replace("timings_", ""), load_table(os.path.join(RESULTS, f)))
              for f in args.extra if os.path.exists(os.path.join(RESULTS, f))]
    excl = [load_table(os.path.join(RESULTS, f)) for f in args.exclude if os.path.exists(os.path.join(RESULTS, f))]
    for _, t in extras:
        assert t["variants"] == tab["variants"], "extra table was written for a different variant table"
    Xtr, Ttr, src = training_union(tab, extras, excl)
    print(f"dataset: {tab['X'].shape[0]} inputs x {tab['T'].shape[1]} variants; held-out {Xte.shape[0]}; "
          f"train {Xtr.shape[0]} = " + " + ".join(f"{src.count(n)} {n}" for n in dict.fromkeys(sorted(src))))
    y = cart.labels_from_table(tab["T"])
    print(f"classes in use: {np.unique(y).size}; most frequent best variant: {tab['variants'][np.bincount(y).argmax()]}")

    from .. import binding as mdg
    meta = mdg.variants()
    assert [m["name"] for m in meta] == tab["variants"], "timing table was written for a different variant table"
    links = fallback_links(meta)  # what the dispatch does with an illegal prediction

    report = []
    for rule in args.leaf_rules:
        rows = cart.sweep(Xtr, Ttr, Xte, Tte, leaf_rule=rule, fallback=links)
        print(f"\nleaf rule: {rule}\n{'model':12s} {'acc%':>6s} {'DTPR':>6s} {'geomean':>8s} {'leaves':>6s} {'height':>6s} {'classes':>7s}")
        for r in rows:
            print(f"{r['name']:12s} {100 * r['accuracy']:6.1f} {r['dtpr']:6.3f} {r['geomean']:8.3f} {r['leaves']:6d} "
                  f"{r['height']:6d} {len(r['classes']):7d}")
            report.append({k: v for k, v in r.items() if k != "tree"})

    best, cv_table = cart.select_model(Xtr, Ttr, fallback=links, folds=args.folds)
    print(f"\nchosen by {args.folds}-fold cross-validation on the training set: {best['name']}/{best['leaf_rule']} "
          f"(cv geomean {best['cv_geomean']:.4f})")
    tree = cart.fit_cart(Xtr, Ttr, best["H"], best["L"], best["leaf_rule"], links)
    pred = tree.predict(Xte)
    held = {"accuracy": cart.accuracy(pred, cart.labels_from_table(Tte)), "dtpr": cart.dtpr(Tte, pred, links),
            "geomean": cart.geomean_ratio(Tte, pred, links)}
    st = tree.stats()
    print(f"held-out: accuracy {100 * held['accuracy']:.1f}%  DTPR {held['dtpr']:.4f}  geomean {held['geomean']:.4f}  "
          f"leaves {st['leaves']} height {st['height']}")

    # forest of bagged trees with the same hyper-parameters: shipped only if cross-validation prefers it
    forest, forest_cv, forest_held = None, None, None
    gate, gate_table = cart.INT64_MAX, None
    if args.forest_trees > 0:
        from .. import workloads as wl
        boot_for = lambda n: wl.bootstrap_indices(n, args.forest_trees)  # noqa: E731
        oof_forest = cart.cross_predict_forest(Xtr, Ttr, boot_for, best["H"], best["L"], best["leaf_rule"], links, args.folds)
        forest_cv = cart.geomean_ratio(Ttr, oof_forest, links)
        oof_tree = cart.cross_predict(Xtr, Ttr, lambda Xa, Ta: cart.fit_cart(Xa, Ta, best["H"], best["L"], best["leaf_rule"], links),
                                      args.folds)
        gate, gate_table = cart.choose_gate(Xtr, Ttr, oof_tree, oof_forest, args.tree_ns, args.forest_ns, links)
        cand = cart.fit_forest(Xtr, Ttr, boot_for(Xtr.shape[0]), best["H"], best["L"], best["leaf_rule"], links)
        fpred = cand.predict(Xte)
        forest_held = {"accuracy": cart.accuracy(fpred, cart.labels_from_table(Tte)), "dtpr": cart.dtpr(Tte, fpred, links),
                       "geomean": cart.geomean_ratio(Tte, fpred, links)}
        fst = cand.stats()
        print(f"forest of {args.forest_trees} trees: cv geomean {forest_cv:.4f} (single tree {best['cv_geomean']:.4f}); "
              f"held-out accuracy {100 * forest_held['accuracy']:.1f}%  DTPR {forest_held['dtpr']:.4f}  "
              f"geomean {forest_held['geomean']:.4f}  leaves {fst['leaves']}")
        print(f"gate on M*N*K (tree below, forest at or above; {args.tree_ns:.0f} / {args.forest_ns:.0f} ns per evaluation "
              "charged to every out-of-fold prediction):")
        for r in gate_table:
            print(f"  gate {r['gate']:>20d}  geomean incl. selector cost {r['geomean_with_cost']:.4f}  "
                  f"({r['rows_by_tree']} of {Xtr.shape[0]} rows by the tree){'  <-- chosen' if r['gate'] == gate else ''}")
        if gate < cart.INT64_MAX:
            forest = cand
            gpred = cart.gated_predict(Xte, gate, pred, fpred)
            gated_held = {"accuracy": cart.accuracy(gpred, cart.labels_from_table(Tte)), "dtpr": cart.dtpr(Tte, gpred, links),
                          "geomean": cart.geomean_ratio(Tte, gpred, links)}
            print(f"gated model on the held-out set: accuracy {100 * gated_held['accuracy']:.1f}%  DTPR {gated_held['dtpr']:.4f}  "
                  f"geomean {gated_held['geomean']:.4f}")

    d_tiled, d_direct, d_thr = (meta[0]["id"], 0, 512.0 ** 3)
    if os.path.exists(args.cfg1):
        d_tiled, d_direct, d_thr = default_dispatch(load_table(args.cfg1), meta)
    print(f"default dispatch: tiled={meta[d_tiled]['name']} direct={meta[d_direct]['name']} threshold={d_thr:.3g}")

    if not args.no_write:
        name = f"{best['name']}/{best['leaf_rule']}"
        nested = tree.to_nested()
        forest_nested = forest.to_nested() if forest is not None else None
        if forest is None:  # the tree alone, as nested if-then-else
            shipped, style, st_ship = nested, "branches", st
        elif gate == 0:
            name = f"forest{args.forest_trees}-{name}"
            shipped, style, st_ship = forest_nested, "branches", forest.stats()
        else:
            name = f"gate2^{gate.bit_length() - 1}-forest{args.forest_trees}-{name}"
            shipped, style = {"gate": gate, "tree": nested, "forest": forest_nested}, "branches"
            st_ship = {"leaves": st["leaves"] + forest.stats()["leaves"], "height": max(st["height"], forest.stats()["height"])}
        codegen.write_header(shipped, name, variant_names=tab["variants"], style=style,
                             default_tiled=d_tiled, default_direct=d_direct, default_threshold=d_thr,
                             provenance=f"model {name}, trained on {Xtr.shape[0]} inputs ("
                                        + ", ".join(f"{src.count(n)} {n}" for n in dict.fromkeys(sorted(src))) + "); "
                                        f"{st_ship['leaves']} leaves, height {st_ship['height']}")
        os.makedirs(RESULTS, exist_ok=True)
        with open(os.path.join(RESULTS, "model.json"), "w") as f:
            json.dump({"name": name, "H": best["H"], "L": best["L"], "leaf_rule": best["leaf_rule"],
                       "training_set": {n: src.count(n) for n in dict.fromkeys(sorted(src))},
                       "cv_geomean": best["cv_geomean"], "heldout_at_training_time": held, "stats": st,
                       "variants": tab["variants"], "tree": nested, "forest": forest_nested,
                       "forest_trees": args.forest_trees if forest is not None else 0,
                       "gate": gate if forest is not None else None, "gate_table": gate_table,
                       "selector_ns_assumed": {"tree": args.tree_ns, "forest": args.forest_ns},
                       "heldout_rows_excluded_from_extra_tables": True,
                       "forest_cv_geomean": forest_cv, "forest_heldout_at_training_time": forest_held,
                       "default_dispatch": {"tiled": d_tiled, "direct": d_direct, "threshold": d_thr},
                       "sweep_on_heldout": report,
                       "cv_table": cv_table}, f, separators=(",", ":"))
        print(f"wrote {codegen.GENERATED_HEADER} and results/model.json -- rebuild the library")


if __name__ == "__main__":
    main()
