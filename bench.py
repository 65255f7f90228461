#!/usr/bin/env python3
"""Benchmark of the on-line hot path on one MI355X.

A step is one pass of the whole path -- validation, decision-tree selection,
legality check, kernel launch(es) -- over the square sweep: M = N = K in
{256 ... 8192}, all four transpose combinations, alpha = 1, beta = 0.5 (24
SGEMM calls through mdg_sgemm).  Operands are seeded synthetic data, resident
in HBM before the timed region.  Prints ONE JSON line.

  value        geometric mean over the 24 shapes of 2MNK / (time per call of that shape), TFLOP/s.  A shape's
               time per call is measured by the library's event-timing core: the K calls of the K timed steps
               issued back to back through the same dispatch path, bracketed by one event pair, operands
               rotating over several sets so they are not served from cache, after about 3 ms of untimed
               calls of the same shape (clock ramp-up).  (Events around every single
               call, as the interleaved pass below uses for the roofline, cost 4-5 us per call on this
               stack, which would distort the 10 us shapes; both figures are printed per shape.)
  ms_per_step  wall time of the K interleaved steps / K
  roofline     for the kernel symbol that takes the most time: algorithmic flops / measured duration
               of its launches (HIP events on the launch stream, inside the timed steps) vs the MI355X
               fp32 matrix peak
  cpu_baseline the CPU oracle timed on a bounded sample of the same workload (reported, not a target)
  selector_measured   (extra leg, bounded) on a seeded sample of the held-out random-sweep shapes plus the 24
               squares: every legal variant timed with the tuning protocol, and mdg_sgemm itself (selector,
               legality, kernel) timed the same way; pct_exhaustive_best_measured = geomean of t_best / t_mdg_sgemm,
               and the same with the measured cost of a fresh-shape model evaluation added to t_mdg_sgemm
  per_config   (extra leg, bounded) geomean TFLOP/s and roofline fraction of mdg_sgemm on samples of the skinny and
               convolution-lowered workloads; empty_launch_us = the smallest call that launches a kernel
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_MATRIX_PEAK_TFLOPS = 157.3  # MI355X datasheet, dense fp32 matrix
HBM_PEAK_GBS = 8000.0


def geomean(xs):
    xs = list(xs)
    return math.exp(sum(math.log(x) for x in xs) / len(xs)) if xs else float("nan")


def kernel_symbol(desc, tA, tB):
    """Name of the GPU kernel a variant launches for these transposes (matches the rocprofv3 kernel trace)."""
    b = lambda x: "true" if x else "false"
    if desc["family"] == 3:  # indirect: the tiled kernel on packed operands (A as stored untransposed, B transposed)
        tA, tB = 0, 1
    if desc["family"] in (1, 3):
        wgm, wgn = desc["tile_m"] // desc["sub_m"], desc["tile_n"] // desc["sub_n"]
        wgk = desc["threads"] // (64 * wgm * wgn)
        return (f"tiled_kernel<{desc['tile_m']}, {desc['tile_n']}, {desc['tile_k']}, {wgm}, {wgn}, {wgk}, {b(tA)}, {b(tB)}, "
                f"{b(desc['lds'] == 2)}, {2 if '_km' not in desc['name'] else desc['name'].split('_km')[1][0]}>")
    if desc["family"] == 0:
        return f"direct_kernel<{desc['sub_m']}, {desc['sub_n']}, {b(desc['lds'])}, {b(tA)}, {b(tB)}>"
    if desc["name"].startswith("skinny_mfma"):  # last argument: 16-byte loads, the case for aligned operands
        return f"thin_mfma_kernel<{b(tA)}, {b(tB)}, {desc['sub_n'] // 16}, true>"
    return f"skinny_{'t' if tA else 'n'}_kernel<{desc['sub_n']}, {b(tB)}>"


def cpu_baseline(sample_n=4096):
    """The oracle, as it stands, on a bounded sample of the sweep: the n = sample_n cases NN and TN (the two the
    oracle's loop order streams through memory; NT and TT take eight times as long)."""
    import numpy as np  # noqa: F401
    from oracle import gemm_oracle as go
    from paper_1806_07060_amd import workloads as wl
    flops, secs = 0.0, 0.0
    for case in wl.config1(sizes=(sample_n,)):
        if case.name[-2:] not in ("NN", "TN"):
            continue
        c = case.resolved()
        A, B, C0 = wl.make_operands(c, poison=False)
        t0 = time.perf_counter()
        st = go.sgemm(c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, A, c.lda, B, c.ldb, c.beta, C0, c.ldc)
        secs += time.perf_counter() - t0
        assert st == 0
        flops += c.flops()
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": go.max_threads(), "kind": "oracle",
            "sample": f"square sweep cases with M=N=K={sample_n}, NN and TN, full matrices "
                      f"({secs:.1f} s wall on {go.max_threads()} threads)"}


def extra_legs(torch, mdg, wl, sptr, heldout_sample=64, skinny_sample=24, conv_sample=15):
    """The bounded side measurements: selector quality measured end to end, secondary workloads, launch floor."""
    import numpy as np
    from paper_1806_07060_amd.tuning import harness
    variants = mdg.variants()
    pools = harness.Pools(torch, harness.POOL_BYTES // 4)
    out = {}

    def sgemm_seconds(c, span_ms=1.0, spans=3):
        n_sets, sa, sb, sc = pools.layout(c)
        t = harness.time_variant(-1, c, pools, n_sets, sa, sb, sc, sptr, 1, 1, 1)
        reps = int(min(200, max(3, math.ceil(span_ms * 1e-3 / max(t, 1e-7)))))
        return harness.time_variant(-1, c, pools, n_sets, sa, sb, sc, sptr, 1, reps, spans)

    # -- selector, measured: exhaustive search over the variant table against what mdg_sgemm does by itself
    _, held = wl.split_train_heldout(wl.config4())
    pick = np.random.Generator(np.random.PCG64(wl.case_seed(41, 0))).choice(len(held), heldout_sample, replace=False)
    sample = [held[i].resolved() for i in sorted(pick.tolist())] + [c.resolved() for c in wl.config1()]
    fresh = wl.fresh_shapes(50000, 2)
    select_ns = mdg.mdg_time_select_ns(fresh[:, 3], fresh[:, 4], fresh[:, 0], fresh[:, 1], fresh[:, 2], iters=2)
    rows = []
    for c in sample:
        times = harness.measure_case(c, pools, sptr, variants)
        t_sel = sgemm_seconds(c)
        rows.append((c, float(np.min(times)), t_sel, int(np.argmin(times))))
    r = np.array([tb / ts for _, tb, ts, _ in rows])
    rc = np.array([tb / (ts + select_ns * 1e-9) for _, tb, ts, _ in rows])
    nh = heldout_sample
    gm = lambda x: float(np.exp(np.mean(np.log(np.minimum(x, 1.0)))))  # noqa: E731  (a ratio above 1 is timing noise)
    out["selector_measured"] = {
        "n": len(rows), "n_heldout": nh, "n_square": len(rows) - nh,
        "pct_exhaustive_best_measured": 100.0 * gm(r),
        "pct_exhaustive_best_measured_heldout": 100.0 * gm(r[:nh]),
        "pct_exhaustive_best_measured_square": 100.0 * gm(r[nh:]),
        "pct_exhaustive_best_measured_with_selector_cost": 100.0 * gm(rc),
        "pct_exhaustive_best_measured_with_selector_cost_heldout": 100.0 * gm(rc[:nh]),
        "fresh_shape_selector_ns": float(select_ns),
        "worst": [{"case": c.name, "shape": [c.M, c.N, c.K, c.tA(), c.tB()], "ratio": float(tb / ts),
                   "best": variants[b]["name"]} for c, tb, ts, b in sorted(rows, key=lambda x: x[1] / x[2])[:3]],
        "protocol": "every legal variant and mdg_sgemm timed by the library's event core on rotating operand sets: "
                    "probe call, then the median of 3 spans of about 1 ms",
    }

    # -- secondary workloads through mdg_sgemm (bounded samples)
    per_config = {}
    for key, every, n_pick, stream_id in (("skinny_fc", wl.config2(), skinny_sample, 1), ("conv_lowered", wl.config3(), conv_sample, 2)):
        pick = np.random.Generator(np.random.PCG64(wl.case_seed(41, stream_id))).choice(len(every), n_pick, replace=False)
        tf, fr, gbs = [], [], []
        for i in sorted(pick.tolist()):
            c = every[i].resolved()
            t = sgemm_seconds(c)
            tf.append(c.flops() / t / 1e12)
            fr.append(max(c.flops() / (FP32_MATRIX_PEAK_TFLOPS * 1e12), c.algorithmic_bytes() / (HBM_PEAK_GBS * 1e9)) / t)
            gbs.append(c.algorithmic_bytes() / t / 1e9)
        per_config[key] = {"n": n_pick, "of": len(every), "geomean_tflops": geomean(tf), "geomean_roofline_frac": geomean(fr),
                           "best_gb_per_s": max(gbs)}
    out["per_config"] = per_config

    # -- launch floor: K = 0 on a 1 x 1 C is one tiny scaling kernel and nothing else
    tiny = wl.GemmCase(1, 1, 0, beta=0.5).resolved()
    n_sets, sa, sb, sc = pools.layout(tiny)
    out["empty_launch_us"] = 1e6 * harness.time_variant(-1, tiny, pools, n_sets, sa, sb, sc, sptr, 20, 500, 5)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU oracle timing (profiling runs)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the bounded side legs (measured selector quality, secondary workloads, launch floor)")
    ap.add_argument("--sizes", type=str, default="256,512,1024,2048,4096,8192")
    ap.add_argument("--workload", choices=("square", "skinny", "conv"), default="square",
                    help="square = the headline sweep (default); skinny = the fully-connected-like shapes "
                         "(HBM-bound for small N); conv = the convolution-lowered shapes.  The secondary workloads "
                         "exist for profiling evidence; the benchmark line the driver reads is the default one")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="instead of the benchmark, launch 5 plain device copies of BYTES (read BYTES + write BYTES "
                         "each) and exit: the known-size kernel against which the FETCH_SIZE / WRITE_SIZE counters "
                         "are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (a call shards over GPUs by column blocks "
              "of B and C without communication, but nothing here uses a second GPU)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1806_07060_amd import binding as mdg
    from paper_1806_07060_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        n = args.copy_calibration // 4
        src = torch.rand(n, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": n * 4, "launches": 5}))
        return
    mdg.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    sizes = tuple(int(s) for s in args.sizes.split(","))
    if args.workload == "square":
        cases = [c.resolved() for c in wl.config1(sizes=sizes)]
        workload_text = ("square fp32 SGEMM sweep M=N=K in {" + ",".join(map(str, sizes)) + "}, column-major, "
                         "NN/NT/TN/TT, alpha=1, beta=0.5, U[-1,1] operands, tight leading dimensions")
    elif args.workload == "skinny":
        cases = [c.resolved() for c in wl.config2()]
        workload_text = ("skinny fp32 SGEMM shaped like fully-connected layers at small batch: M in {1024,2048,4096,7680}, "
                         "N in {1,4,16,32,64,128}, K in {1024,2048,4096}, transA in {N,T}, alpha=1, beta=0, N(0,1/sqrt(K)) operands")
    else:
        cases = [c.resolved() for c in wl.config3()]
        workload_text = ("convolution-lowered fp32 SGEMM: M in {32..512}, N in {3136,12544,50176}, K in {27..2304}, NN, "
                         "alpha=1, beta=0, U[-1,1] operands")
    variants = mdg.variants()

    ws = torch.empty(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB of split-K workspace
    assert mdg.mdg_set_workspace(ws.data_ptr(), ws.numel() * 4) == 0

    # per case: n_sets copies of the seeded operands laid out back to back (set 0 is what the interleaved
    # steps use); as many sets as fit 600 MB, at most 8
    dev, sets = [], []
    for c in cases:
        A, B, C0 = wl.make_operands(c, poison=False)
        n_sets = int(max(1, min(8, math.ceil(600e6 / (4.0 * (A.size + B.size + C0.size))))))
        dev.append(tuple(torch.from_numpy(x).cuda().repeat(n_sets) for x in (A, B, C0)))
        sets.append((n_sets, A.size, B.size, C0.size))
        del A, B, C0
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    sptr = stream.cuda_stream

    def one_step(events=None):
        for i, (c, (dA, dB, dC)) in enumerate(zip(cases, dev)):
            if events is not None:
                events[i][0].record(stream)
            st = mdg.mdg_sgemm(c.layout, c.transA, c.transB, c.M, c.N, c.K, c.alpha, dA.data_ptr(), c.lda,
                               dB.data_ptr(), c.ldb, c.beta, dC.data_ptr(), c.ldc, sptr)
            if st != 0:
                raise RuntimeError(f"{c.name}: {mdg.mdg_status_string(st)}")
            if events is not None:
                events[i][1].record(stream)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in cases]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(ev[s])
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0

    per_case_ms = np.array([[ev[s][i][0].elapsed_time(ev[s][i][1]) for i in range(len(cases))]
                            for s in range(args.steps)])
    med_ms = np.median(per_case_ms, axis=0)  # per call, one event pair around every call

    # the same K calls per shape, back to back between one event pair (selector and legality included)
    b2b_ms = []
    for i, (c, (dA, dB, dC), (n_sets, na, nb, nc)) in enumerate(zip(cases, dev, sets)):
        # untimed calls of the same shape for about 3 ms first: a run of launch-bound small shapes leaves the
        # GPU clocks near idle, and the first milliseconds of the next shape would be timed while they ramp up
        warm = int(min(500, max(1, math.ceil(3.0 / max(float(med_ms[i]), 1e-3)))))
        st, ms = mdg.mdg_time_calls(-1, c.tA(), c.tB(), c.M, c.N, c.K, c.alpha, dA.data_ptr(), c.lda, dB.data_ptr(),
                                    c.ldb, c.beta, dC.data_ptr(), c.ldc, n_sets, na, nb, nc, warmup=warm,
                                    reps=args.steps, spans=1, stream=sptr)
        if st != 0:
            raise RuntimeError(f"{c.name}: {mdg.mdg_status_string(st)}")
        b2b_ms.append(ms[0])
    b2b_ms = np.array(b2b_ms)
    tflops = np.array([c.flops() / (m * 1e-3) / 1e12 for c, m in zip(cases, b2b_ms)])

    # which kernel each call ran (selector, then fallback to variant 0 if illegal), grouped by kernel symbol
    groups = {}
    chosen = []
    for i, c in enumerate(cases):
        v = mdg.mdg_select(c.tA(), c.tB(), c.M, c.N, c.K)
        for _ in range(len(variants)):  # the dispatch's fallback chain
            if v == 0 or mdg.mdg_variant_legal(v, c.tA(), c.tB(), c.M, c.N, c.K, c.lda, c.ldb, c.ldc,
                                               dev[i][0].data_ptr(), dev[i][1].data_ptr(), dev[i][2].data_ptr()) == 1:
                break
            v = variants[v]["fallback"]
        chosen.append(v)
        sym = kernel_symbol(variants[v], c.tA(), c.tB())
        g = groups.setdefault(sym, {"ms": 0.0, "flops": 0.0, "launches": 0, "bytes": 0.0})
        g["ms"] += float(per_case_ms[:, i].sum())
        g["flops"] += float(c.flops()) * args.steps
        g["bytes"] += float(c.algorithmic_bytes()) * args.steps
        g["launches"] += args.steps
    dom_sym, dom = max(groups.items(), key=lambda kv: kv[1]["ms"])
    achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12

    # the launches of the dominant kernel sit below or above the ridge (157.3 TFLOP/s / 8 TB/s = 19.7 flop/byte)?
    hbm_bound = dom["flops"] / dom["bytes"] < FP32_MATRIX_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and args.workload == "square" and args.sizes == ap.get_default("sizes"):
        try:
            traffic = json.load(open(tpath)).get(dom_sym, {}).get("bytes_per_launch")
        except Exception:
            traffic = None

    if hbm_bound:
        gbs = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": float(gbs), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": float(gbs / HBM_PEAK_GBS)}
    else:
        roofline = {"bound": "mfma", "achieved": float(achieved), "peak": FP32_MATRIX_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": float(achieved / FP32_MATRIX_PEAK_TFLOPS)}
    roofline.update({"traffic": traffic, "kernel": dom_sym, "launches": dom["launches"],
                     "avg_launch_ms": dom["ms"] / dom["launches"],
                     "algorithmic_flops_per_launch": dom["flops"] / dom["launches"],
                     "algorithmic_bytes_per_launch": dom["bytes"] / dom["launches"]})
    large = [t for c, t in zip(cases, tflops) if c.M >= 4096 and args.workload == "square"]
    sel_eval = None
    epath = os.path.join(ROOT, "paper_1806_07060_amd", "tuning", "results", "selector_eval.json")
    if os.path.exists(epath):
        try:
            sel_eval = json.load(open(epath))
        except Exception:
            sel_eval = None

    out = {
        "metric": "SGEMM TFLOP/s geomean over shape sweep; % of exhaustive-best; % FP32 peak",
        "value": float(geomean(tflops)),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": total_s * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": workload_text + f" ({len(cases)} calls per step through mdg_sgemm)",
                   "selector": mdg.mdg_selector_name()},
        "aggregate_tflops": float(sum(c.flops() for c in cases) * args.steps / total_s / 1e12),
        "pct_fp32_peak_large": float(100.0 * geomean(large) / FP32_MATRIX_PEAK_TFLOPS) if large else None,
        "pct_exhaustive_best_heldout_stored_table": (sel_eval or {}).get("heldout_geomean_pct"),
        "pct_exhaustive_best_heldout_stored_table_with_selector_cost":
            (sel_eval or {}).get("heldout_geomean_with_selector_cost_pct"),
        "per_shape": [{"case": c.name, "variant": variants[v]["name"], "ms": float(m), "tflops": float(t),
                       "ms_single_call_events": float(e),
                       "roofline_frac": float(max(c.flops() / (FP32_MATRIX_PEAK_TFLOPS * 1e12),
                                                  c.algorithmic_bytes() / (HBM_PEAK_GBS * 1e9)) / (m * 1e-3)),
                       "gb_per_s": float(c.algorithmic_bytes() / (m * 1e-3) / 1e9)}
                      for c, v, m, t, e in zip(cases, chosen, b2b_ms, tflops, med_ms)],
        "roofline": roofline,
    }
    if not args.no_extras and args.workload == "square":
        del dev  # the side legs bring their own operand pools
        torch.cuda.empty_cache()
        out.update(extra_legs(torch, mdg, wl, sptr))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    mdg.mdg_set_workspace(0, 0)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
