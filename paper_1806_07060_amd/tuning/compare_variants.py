"""Time a handful of named variants against each other in one process (same box, same clocks, alternating rounds).

  python -m paper_1806_07060_amd.tuning.compare_variants --variants NAME[,NAME...] [--sizes 8192,4096] [--rounds 3]

For every square case of the given sizes (all four transpose combinations, alpha = 1, beta = 0.5) each listed
variant that is legal is timed with the library's event core on rotating operand sets, `--rounds` times in turn;
the best round is printed as TFLOP/s and as microseconds per call.  Differences between boxes and between runs are 1-2 %, larger than many
kernel effects, so design choices inside a kernel family (lane arrangements, direct-to-LDS loads, tile shapes)
are compared here rather than across runs of the benchmark.
"""
import argparse

from . import harness
from .. import binding as mdg
from .. import workloads as wl


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--variants", required=True, help="comma-separated variant names (mdg_variant_info().name)")
    ap.add_argument("--sizes", default="8192,4096")
    ap.add_argument("--shapes", default="", help="further cases MxNxK[,MxNxK...] (tight leading dimensions, all four "
                                                 "transpose combinations, alpha = 1, beta = 0.5)")
    ap.add_argument("--rounds", type=int, default=3)
    args = ap.parse_args(argv)
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    table = mdg.variants()
    by_name = {v["name"]: v["id"] for v in table}
    ids = [by_name[n] for n in args.variants.split(",")]
    pools = harness.Pools(torch, harness.POOL_BYTES // 4)
    ws = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    assert mdg.mdg_set_workspace(ws.data_ptr(), ws.numel() * 4) == 0
    stream = torch.cuda.current_stream().cuda_stream
    cases = [c for n in (int(x) for x in args.sizes.split(",") if x) for c in wl.config1(sizes=(n,))]
    for spec in (x for x in args.shapes.split(",") if x):
        M, N, K = (int(v) for v in spec.split("x"))
        cases += [wl.GemmCase(M, N, K, ta, tb, 1.0, 0.5, name=f"{spec}/{'NT'[ta != wl.NO_TRANS]}{'NT'[tb != wl.NO_TRANS]}")
                  for ta in (wl.NO_TRANS, wl.TRANS) for tb in (wl.NO_TRANS, wl.TRANS)]
    for case in cases:
        if True:
            c = case.resolved()
            n = max(c.M, c.N, c.K)
            n_sets, sa, sb, sc = pools.layout(c)
            best = {}
            for _ in range(args.rounds):
                for i in ids:
                    if mdg.mdg_variant_legal(i, c.tA(), c.tB(), c.M, c.N, c.K, c.lda, c.ldb, c.ldc, pools.A.data_ptr(),
                                             pools.B.data_ptr(), pools.C.data_ptr()) != 1:
                        continue
                    reps = 6 if n >= 8192 else 20 if n >= 2048 else 100
                    t = harness.time_variant(i, c, pools, n_sets, sa, sb, sc, stream, 2, reps, 3)
                    best[i] = min(best.get(i, t), t)
            print(c.name, " | ".join(f"{table[i]['name']} {c.flops() / t / 1e12:.1f} ({t * 1e6:.1f} us)" for i, t in best.items()), flush=True)
    mdg.mdg_set_workspace(0, 0)


if __name__ == "__main__":
    main()
