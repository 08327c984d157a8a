"""include/klay.h compiles as plain C and the library works without Python: tests/c_abi_check.c is
built with gcc against the in-tree library, builds the circuit of Figure 1(b), checks Figure 2's
layer sizes on a host-only handle and, on the GPU, the figure's closed form and its derivative."""
import os
import subprocess

import pytest

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


@pytest.mark.gpu
def test_c_program_evaluates_on_the_gpu(tmp_path):
    r = subprocess.run([_build(tmp_path), "gpu"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "gpu ok" in r.stdout, r.stdout + r.stderr
