"""Off-line phase, step 1: build the dataset D by timing every variant on every input.

Section 4.1 of the paper builds each dataset entry by running the tuner over
the whole search space of both kernels for a triple (M, N, K) and keeping the
best; here the search space is the library's variant table and the *whole row*
of times is kept (the ratio metrics of Section 5.2 need the time of the
predicted variant, not only the label).  Unlike the paper's tuner, which
reports kernel time only, a time here is the whole call: the kernel plus any
pass the variant needs (split-K reduce).

Protocol per (input, variant), all through the library's own event-timing
entry point (mdg_time_calls):
  1. one probe call (after one warm-up) estimates the time t;
  2. if t exceeds `prune` x the best time seen so far for this input the
     estimate is recorded and the variant is not measured further (it cannot
     be the label and, being that slow, is priced well enough by one call);
  3. otherwise `spans` spans of `reps` back-to-back calls, reps chosen so a
     span lasts about `span_ms`; the median span is recorded.
Calls rotate through several operand sets so that inputs are not served from
cache left by the previous call (as many sets as fit 600 MB, at most 32).

Writes a CSV, one row per input: index, name, M, N, K, tA, tB, alpha, beta,
then seconds per variant (inf = illegal).  Rows already in the file are
skipped, so a run can be continued.
"""
import argparse
import csv
import math
import os
import sys
import time

import numpy as np

from .. import binding as mdg
from .. import workloads as wl

POOL_BYTES = 640 << 20
MAX_SETS = 32


def _align(n, a=64):
    return (n + a - 1) // a * a


class Pools:
    """Device pools for A, B, C (seeded U[-1,1] data; timing does not depend on the values)."""

    def __init__(self, torch, floats_each):
        g = torch.Generator(device="cuda")
        g.manual_seed(wl.BASE_SEED)
        self.torch = torch
        self.n = floats_each
        self.A = torch.rand(floats_each, device="cuda", generator=g) * 2 - 1
        self.B = torch.rand(floats_each, device="cuda", generator=g) * 2 - 1
        self.C = torch.rand(floats_each, device="cuda", generator=g) * 2 - 1

    def layout(self, case):
        c = case.resolved()
        na = wl.buffer_len(c.layout, c.a_shape(), c.lda)
        nb = wl.buffer_len(c.layout, c.b_shape(), c.ldb)
        nc = wl.buffer_len(c.layout, c.c_shape(), c.ldc)
        sa, sb, sc = _align(na), _align(nb), _align(nc)
        if max(sa, sb, sc) > self.n:
            raise ValueError(f"{c.name}: an operand of {max(sa, sb, sc)} floats does not fit the {self.n}-float pool")
        foot = 4 * (na + nb + nc)
        n_sets = max(1, min(MAX_SETS, math.ceil(600e6 / max(foot, 1)), self.n // max(sa, sb, sc)))
        return n_sets, sa, sb, sc


def time_variant(v, case, pools, n_sets, sa, sb, sc, stream, warmup, reps, spans):
    c = case
    st, ms = mdg.mdg_time_calls(v, c.tA(), c.tB(), c.M, c.N, c.K, c.alpha, pools.A.data_ptr(), c.lda,
                                pools.B.data_ptr(), c.ldb, c.beta, pools.C.data_ptr(), c.ldc, n_sets, sa, sb, sc,
                                warmup, reps, spans, stream)
    if st != 0:
        raise RuntimeError(f"variant {v} on {c.name}: {mdg.mdg_status_string(st)}")
    return float(np.median(ms)) * 1e-3


def measure_case(case, pools, stream, variants, span_ms=1.0, spans=3, prune=6.0, max_reps=200, known=None):
    """Seconds of every variant on one column-major case (inf where illegal).

    `known` maps variant ids to times measured earlier (same protocol): those are kept, not re-measured.
    """
    c = case.resolved()
    assert c.layout == wl.COL_MAJOR
    n_sets, sa, sb, sc = pools.layout(c)
    out = np.full(len(variants), np.inf)
    best = np.inf
    for v, t in (known or {}).items():
        out[v] = t
        best = min(best, t)
    # likely-good variants first so that pruning bites early
    order = sorted(range(len(variants)), key=lambda v: (variants[v]["family"] != mdg.FAMILY_TILED, v))
    for v in order:
        if known is not None and v in known:
            continue
        if mdg.mdg_variant_legal(v, c.tA(), c.tB(), c.M, c.N, c.K, c.lda, c.ldb, c.ldc, pools.A.data_ptr(),
                                 pools.B.data_ptr(), pools.C.data_ptr()) != 1:
            continue
        t = time_variant(v, c, pools, n_sets, sa, sb, sc, stream, 1, 1, 1)
        if t > prune * best and t < 1e-3:
            # a single cold call can be an outlier (first launch of a kernel symbol): ask once more before pruning
            t = min(t, time_variant(v, c, pools, n_sets, sa, sb, sc, stream, 1, 1, 1))
        if t <= prune * best:
            reps = int(min(max_reps, max(3, math.ceil(span_ms * 1e-3 / max(t, 1e-7)))))
            t = time_variant(v, c, pools, n_sets, sa, sb, sc, stream, 1, reps, spans)
        out[v] = t
        best = min(best, t)
    return out


def verify_case(case, pools, stream, variants):
    """Run every legal variant once on the first operand set of the pools and hold its C to variant 0's (the
    universal direct kernel, itself held to the oracle by the tests): |C_v - C_0| <= 2e-6 K max|a| max|b| +
    2e-6 |beta C0| (two results that each meet the library's tolerance differ by at most twice that).  Returns
    (pairs checked, worst error / bound).  A timing of a kernel that computes the wrong thing is worthless; this
    is the tuning run's own guard, not a parity test."""
    torch = pools.torch
    c = case.resolved()
    na = wl.buffer_len(c.layout, c.a_shape(), c.lda)
    nb = wl.buffer_len(c.layout, c.b_shape(), c.ldb)
    nc = wl.buffer_len(c.layout, c.c_shape(), c.ldc)
    C0 = pools.C[:nc].clone()

    def run(v):
        out = C0.clone()
        st = mdg.mdg_sgemm_variant(v, c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, pools.A.data_ptr(), c.lda,
                                   pools.B.data_ptr(), c.ldb, c.beta, out.data_ptr(), c.ldc, stream)
        if st != 0:
            raise RuntimeError(f"variant {v} on {c.name}: {mdg.mdg_status_string(st)}")
        return out

    ref = run(0)
    bound = 2e-6 * c.K * float(pools.A[:na].abs().max()) * float(pools.B[:nb].abs().max()) + 2e-6 * abs(c.beta) * C0.abs()
    bound = torch.clamp(bound, min=1e-30)
    worst, n = 0.0, 0
    for v in range(1, len(variants)):
        if mdg.mdg_variant_legal(v, c.tA(), c.tB(), c.M, c.N, c.K, c.lda, c.ldb, c.ldc, pools.A.data_ptr(),
                                 pools.B.data_ptr(), C0.data_ptr()) != 1:
            continue
        ratio = float(((run(v) - ref).abs() / bound).max()) if nc else 0.0
        if not ratio <= 1.0:
            raise RuntimeError(f"{variants[v]['name']} on {c.name} ({c.M}x{c.N}x{c.K}, tA={c.tA()}, tB={c.tB()}): result "
                               f"differs from variant 0 by {ratio:.2f} x the bound")
        worst, n = max(worst, ratio), n + 1
    return n, worst


def recheck_case(case, pools, stream, variants, times, span_ms=1.0, spans=3, prune=6.0, max_reps=200, below=1e-3):
    """Second look at entries that were recorded from one probe call (slower than prune x the row's best) and are
    short enough (< `below` seconds) for a cold first launch to have distorted them: probe again, and measure
    fully if the new probe no longer says prune.  Returns the corrected row and the number of entries changed."""
    c = case.resolved()
    n_sets, sa, sb, sc = pools.layout(c)
    out = np.array(times, dtype=np.float64)
    best = np.min(out)
    changed = 0
    for v in range(len(variants)):
        if not np.isfinite(out[v]) or out[v] <= prune * best or out[v] >= below:
            continue
        t = time_variant(v, c, pools, n_sets, sa, sb, sc, stream, 2, 3, 1)
        if t <= prune * best:
            reps = int(min(max_reps, max(3, math.ceil(span_ms * 1e-3 / max(t, 1e-7)))))
            t = time_variant(v, c, pools, n_sets, sa, sb, sc, stream, 1, reps, spans)
        if t < 0.8 * out[v]:
            out[v] = t
            changed += 1
    return out, changed


def load_done(path):
    done = {}
    if os.path.exists(path):
        with open(path) as f:
            r = csv.reader(f)
            header = next(r, None)
            for row in r:
                if row:
                    done[int(row[0])] = row
        return header, done
    return None, done


def cases_for(config):
    if config == 1:
        return [c.resolved() for c in wl.config1()]
    if config == 2:
        return [c.resolved() for c in wl.config2()]
    if config == 3:
        return [c.resolved() for c in wl.config3()]
    if config == 4:
        return [c.resolved() for c in wl.config4()]
    if config == 0:
        return [c.resolved() for c in wl.config0()]
    if config == 5:
        return [c.resolved() for c in wl.config_go2()]
    if config == 6:
        return [c.resolved() for c in wl.config_po2()]
    if config == 7:
        return [c.resolved() for c in wl.config_wide()]
    if config == 8:
        return [c.resolved() for c in wl.config_big()]
    if config == 9:
        return [c.resolved() for c in wl.config_large_grid()]
    if config == 10:
        return [c.resolved() for c in wl.config_thin()]
    if config == 11:
        return [c.resolved() for c in wl.config_flat()]
    if config == 12:
        return [c.resolved() for c in wl.config_thin_grid()]
    if config == 13:
        return [c.resolved() for c in wl.config_flat_grid()]
    if config == 14:
        return [c.resolved() for c in wl.config_sweep2()]
    if config == 15:
        return [c.resolved() for c in wl.config_thin2()]
    if config == 16:
        return [c.resolved() for c in wl.config_flat2()]
    if config == 17:
        return [c.resolved() for c in wl.config_sweep3()]
    if config == 18:
        return [c.resolved() for c in wl.config_thin3()]
    if config == 19:
        return [c.resolved() for c in wl.config_flat3()]
    if config == 20:
        return [c.resolved() for c in wl.config_thin_grid2()]
    raise ValueError(config)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=4,
                    help="0-4: the five workload configurations; 5: go2 grid; 6: po2 grid; 7: wide random sweep; 8: large products; 9: coarse grid of the largest sizes; 10: thin (few columns); 11: flat (few rows); 12 / 13: geometric grids over the thin / flat corners; 14 / 17: second and third random sweep; 15, 18 / 16, 19: more thin / flat shapes; 20: denser grid over the thin corner")
    ap.add_argument("--out", default=None, help="the table to write (required unless --verify-every)")
    ap.add_argument("--start", type=int, default=0)
    ap.add_argument("--limit", type=int, default=10 ** 9)
    ap.add_argument("--budget-s", type=float, default=1e9, help="stop cleanly after this many seconds")
    ap.add_argument("--span-ms", type=float, default=1.0)
    ap.add_argument("--spans", type=int, default=3)
    ap.add_argument("--prune", type=float, default=6.0)
    ap.add_argument("--verify-every", type=int, default=0, metavar="N",
                    help="instead of timing: for every N-th input run every legal variant once and hold its result "
                         "to variant 0's (see verify_case); prints a summary, writes no table")
    ap.add_argument("--recheck-from", default=None, metavar="CSV",
                    help="a finished table of the same inputs and variants: re-measure only the short entries that "
                         "were recorded from a single probe call, write the corrected table to --out")
    ap.add_argument("--remeasure-prefix", default=None, metavar="NAME",
                    help="with --extend-from: variants whose name starts with NAME are measured again instead of "
                         "copied (after a change to that kernel family)")
    ap.add_argument("--extend-from", default=None, metavar="CSV",
                    help="a table of the same inputs written for an older variant table: times of variants it "
                         "already holds (matched by name) are copied, only the new variants are measured")
    args = ap.parse_args(argv)

    if args.out is None and args.verify_every <= 0:
        ap.error("--out is required")
    import torch
    assert torch.cuda.is_available(), "the tuning run needs a GPU"
    mdg.lib()
    variants = mdg.variants()
    cases = cases_for(args.config)
    pools = Pools(torch, POOL_BYTES // 4)
    ws = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    assert mdg.mdg_set_workspace(ws.data_ptr(), ws.numel() * 4) == 0
    stream = torch.cuda.current_stream().cuda_stream

    if args.verify_every > 0:
        t0, pairs, worst, shapes = time.time(), 0, 0.0, 0
        for i, c in enumerate(cases):
            if i % args.verify_every or i < args.start or i >= args.start + args.limit:
                continue
            n, w = verify_case(c, pools, stream, variants)
            pairs, worst, shapes = pairs + n, max(worst, w), shapes + 1
            if shapes % 20 == 0:
                print(f"[{time.time() - t0:7.1f}s] {shapes} inputs, {pairs} (input, variant) results verified, worst "
                      f"error / bound {worst:.3f}", flush=True)
        mdg.mdg_set_workspace(0, 0)
        print(f"verified: {shapes} inputs of config {args.config}, {pairs} (input, variant) results against variant 0, "
              f"worst error / bound {worst:.3f}, {time.time() - t0:.1f}s", flush=True)
        return
    os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
    header, done = load_done(args.out)
    want_header = ["index", "name", "M", "N", "K", "tA", "tB", "alpha", "beta"] + [v["name"] for v in variants]
    if header is not None and header != want_header:
        raise SystemExit(f"{args.out} was written for a different variant table; move it away first")
    if args.recheck_from:
        rc_header, rc_rows = load_done(args.recheck_from)
        if rc_header != want_header:
            raise SystemExit(f"{args.recheck_from} was written for a different variant table")
        t0, total = time.time(), 0
        with open(args.out, "w", newline="") as f:
            w = csv.writer(f)
            w.writerow(want_header)
            for i, c in enumerate(cases):
                if i not in rc_rows:
                    continue
                r = rc_rows[i]
                assert (int(r[2]), int(r[3]), int(r[4]), int(r[5]), int(r[6])) == (c.M, c.N, c.K, c.tA(), c.tB()), r[:7]
                times, changed = recheck_case(c, pools, stream, variants, [float(x) for x in r[9:]], args.span_ms,
                                              args.spans, args.prune)
                total += changed
                w.writerow(r[:9] + [repr(float(t)) for t in times])
                if (i + 1) % 200 == 0:
                    f.flush()
                    print(f"[{time.time() - t0:7.1f}s] {i + 1}/{len(cases)} rechecked, {total} entries corrected", flush=True)
        mdg.mdg_set_workspace(0, 0)
        print(f"done: {total} entries corrected in {time.time() - t0:.1f}s -> {args.out}", flush=True)
        return
    old_rows, old_names = {}, []
    if args.extend_from:
        old_header, old_rows = load_done(args.extend_from)
        old_names = old_header[9:]
        name_to_id = {v["name"]: v["id"] for v in variants}
    t0 = time.time()
    with open(args.out, "a", newline="") as f:
        w = csv.writer(f)
        if header is None:
            w.writerow(want_header)
        n_new = 0
        for i, c in enumerate(cases):
            if i < args.start or i >= args.start + args.limit or i in done:
                continue
            if time.time() - t0 > args.budget_s:
                break
            known = None
            if i in old_rows:
                r = old_rows[i]
                assert (int(r[2]), int(r[3]), int(r[4]), int(r[5]), int(r[6])) == (c.M, c.N, c.K, c.tA(), c.tB()), r[:7]
                known = {name_to_id[n]: float(x) for n, x in zip(old_names, r[9:]) if n in name_to_id
                         and not (args.remeasure_prefix and n.startswith(args.remeasure_prefix))}
            times = measure_case(c, pools, stream, variants, args.span_ms, args.spans, args.prune, known=known)
            w.writerow([i, c.name, c.M, c.N, c.K, c.tA(), c.tB(), repr(c.alpha), repr(c.beta)] +
                       [repr(float(t)) for t in times])
            f.flush()
            n_new += 1
            if n_new % 25 == 0:
                b = int(np.argmin(times))
                print(f"[{time.time() - t0:7.1f}s] {i + 1}/{len(cases)} {c.name} {c.M}x{c.N}x{c.K} "
                      f"best={variants[b]['name']} {times[b] * 1e6:.1f}us", flush=True)
    mdg.mdg_set_workspace(0, 0)
    print(f"done: {n_new} new rows in {time.time() - t0:.1f}s -> {args.out}", flush=True)


if __name__ == "__main__":
    main()
