"""Host check of the launch plans (tasks, segments of split rows, combine lists) that klay_build
uploads: tests/host_plan_check.cpp layerizes random DAGs under many option sets and executes every
plan in plain C++ the way the kernels walk it, against sums over the plain index vectors.  Compiled
with the address and undefined-behaviour sanitizers, so it also sweeps the layerizer for memory
errors.  No GPU needed."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_launch_plans_execute_to_the_plain_sums(tmp_path):
    exe = str(tmp_path / "host_plan_check")
    # the sanitizer runtimes are linked statically, so they come first whatever else the process preloads
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan", "-fno-omit-frame-pointer", "-o", exe,
           os.path.join(ROOT, "tests", "host_plan_check.cpp"),
           os.path.join(ROOT, "paper_2410_11415_amd", "csrc", "layerize.cpp")]
    subprocess.run(cmd, check=True, cwd=ROOT)
    r = subprocess.run([exe, "120"], capture_output=True, text=True, timeout=600)
    sys.stdout.write(r.stdout[-2000:]); sys.stderr.write(r.stderr[-4000:])
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert r.stdout.strip().startswith("ok:")
