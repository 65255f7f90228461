"""bench.py contract checks that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_kernel_symbols_match_the_compiled_template_names():
    sys.path.insert(0, ROOT)
    import bench
    from paper_1806_07060_amd import binding as mdg
    names = set()
    for d in mdg.variants():
        for tA in (0, 1):
            for tB in (0, 1):
                names.add(bench.kernel_symbol(d, tA, tB))
    syms = subprocess.run(["nm", "-C", "--defined-only", mdg.LIB_PATH], capture_output=True, text=True).stdout
    # host-side launch stubs carry the kernels' demangled names
    for n in sorted(names):
        assert n in syms, n
