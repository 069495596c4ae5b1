"""A C99 program (tests/c_caller.c), compiled with gcc and linked against
libh2o_hip.so, calls the library with no C++ or Python in between: the host-side
argument checks here (no GPU), and on a GPU a whole small run."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "c_caller.c")
OUT_DIR = os.path.join(ROOT, "tests", "_build")
EXE = os.path.join(OUT_DIR, "c_caller")
LIB_DIR = os.path.join(ROOT, "paper_2306_14048_amd")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build_c_caller(force: bool = False) -> str:
    lib = os.path.join(LIB_DIR, "libh2o_hip.so")
    if not os.path.exists(lib):
        from paper_2306_14048_amd import build
        build.build(verbose=False)
    newest = max(os.path.getmtime(SRC), os.path.getmtime(os.path.join(ROOT, "include", "h2o.h")))
    if force or not os.path.exists(EXE) or os.path.getmtime(EXE) < newest:
        os.makedirs(OUT_DIR, exist_ok=True)
        tmp = EXE + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-O1", "-D__HIP_PLATFORM_AMD__",
             "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(ROCM, "include"), SRC, "-o", tmp,
             "-L", LIB_DIR, "-lh2o_hip", "-L", os.path.join(ROCM, "lib"), "-lamdhip64", "-lm",
             "-Wl,-rpath," + LIB_DIR, "-Wl,-rpath," + os.path.join(ROCM, "lib")])
        os.replace(tmp, EXE)
    return EXE


def run(mode: str) -> str:
    res = subprocess.run([build_c_caller(), mode], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, "c_caller %s failed (%d):\n%s\n%s" % (mode, res.returncode, res.stdout, res.stderr)
    return res.stdout.strip().splitlines()[-1]


def test_c_program_links_and_walks_the_host_side_checks():
    assert run("host") == "host ok"


@pytest.mark.gpu
def test_c_program_runs_the_path_on_the_device():
    assert run("gpu") == "gpu ok"
