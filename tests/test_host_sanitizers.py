"""Host-only sanitizer build (CPU, no GPU runtime): the library's host translation unit -- variant table, validation,
legality, workspace arithmetic, the generated selector and its memo -- and the C oracle are compiled with
AddressSanitizer and UndefinedBehaviorSanitizer, linked with a driver that walks them
(tests/host_sanitize_main.cpp), and run.  Any report ends the run with a non-zero status."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def test_host_code_and_oracle_run_clean_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_1806_07060_amd", "csrc")
    objs = []
    for compiler, src, flags in (("g++", os.path.join(csrc, "mdg_dispatch.cpp"), ["-std=c++17"]),
                                 ("g++", os.path.join(ROOT, "tests", "host_sanitize_main.cpp"), ["-std=c++17"]),
                                 ("gcc", os.path.join(ROOT, "oracle", "gemm_oracle.c"), ["-std=c11", "-fopenmp"])):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([compiler] + SAN + flags + ["-Wall", "-c", src, "-o", obj], check=True)
        objs.append(obj)
    exe = str(tmp_path / "host_sanitize")
    # the sanitizer runtimes are linked statically: a preloaded library in the environment cannot get in front of them
    subprocess.run(["g++"] + SAN + ["-static-libasan", "-static-libubsan", "-fopenmp", "-o", exe] + objs, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0 and r.stdout.startswith("ok:"), (r.stdout[-2000:], r.stderr[-4000:])
