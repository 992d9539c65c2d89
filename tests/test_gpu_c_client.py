"""The boundary from the other side: a program in plain C (no Python, no PyTorch) that calls
libxbq.so with device memory from the HIP runtime and checks itself against the C oracle."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "abi_client")
BINARY = os.path.join(HERE, "client")


def build_client() -> str:
    """gcc only: the client holds no device code (about a second)."""
    from oracle import scale as oracle_scale
    oracle_lib = oracle_scale.build()
    pkg = os.path.join(ROOT, "paper_2008_02002_amd")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-O1", "-std=c11", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"),
           "-o", BINARY, os.path.join(HERE, "client.c"),
           os.path.join(pkg, "libxbq.so"), oracle_lib, "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath," + pkg, "-Wl,-rpath," + os.path.dirname(oracle_lib), "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.run(cmd, check=True)
    return BINARY


def test_plain_c_caller_matches_the_oracle():
    src = os.path.join(HERE, "client.c")
    if not os.path.exists(BINARY) or os.path.getmtime(BINARY) < os.path.getmtime(src):
        build_client()
    print("running the C client", flush=True)
    r = subprocess.run([BINARY], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.stdout + r.stderr)[-2000:]
    assert "abi client ok" in r.stdout
