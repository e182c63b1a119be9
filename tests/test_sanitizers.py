"""CPU builds with -fsanitize=address,undefined: the whole oracle on small exact-size buffers, and the
host-side GEMM launch planner over a sweep of shapes (coverage invariant).  No GPU, no HIP."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="2")
ENV.pop("LD_PRELOAD", None)           # the sanitizer runtime must come first in the initial library list


def _build_and_run(tmp_path, compiler, sources, extra):
    exe = str(tmp_path / "driver")
    subprocess.check_call([compiler] + SAN + sources + ["-o", exe] + extra)
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=ENV, timeout=600)
    assert proc.returncode == 0, proc.stdout[-4000:]
    assert "runtime error" not in proc.stdout and "AddressSanitizer" not in proc.stdout, proc.stdout[-4000:]
    assert proc.stdout.strip().splitlines()[-1].startswith("ok"), proc.stdout[-2000:]


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    _build_and_run(tmp_path, "gcc", [os.path.join(HERE, "sanitize", "oracle_driver.c"),
                                     os.path.join(ROOT, "oracle", "nvfp4_oracle.c")],
                   ["-ffp-contract=off", "-fopenmp", "-lm"])


def test_gemm_launch_planner_under_sanitizers(tmp_path):
    _build_and_run(tmp_path, "g++", ["-std=c++17", os.path.join(HERE, "sanitize", "plan_driver.cpp")], [])
