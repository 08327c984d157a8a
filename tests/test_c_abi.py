"""include/klay.h compiles as plain C and the library works without Python: tests/c_abi_check.c is
built with gcc against the in-tree library, builds the circuit of Figure 1(b) as a host-only handle
and checks Figure 2's layer sizes and the error reporting.  The program's "gpu" mode (the figure's
closed form and its derivative on device 0) is for running by hand: a GPU-using child process must
not run from the test process, whose own first use of the GPU then fails on the test machines."""
import os
import subprocess

from paper_2410_11415_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build(tmp_path):
    exe = str(tmp_path / "c_abi_check")
    lib = binding.library_path()
    binding.load()                                  # raises if the library is missing
    cmd = ["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-o", exe, os.path.join(ROOT, "tests", "c_abi_check.c"),
           lib, "-L/opt/rocm/lib", "-lamdhip64", "-lm", "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True, cwd=ROOT)
    return exe


def test_c_program_builds_and_inspects_a_circuit(tmp_path):
    r = subprocess.run([_build(tmp_path)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr

