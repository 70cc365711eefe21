"""The boundary from plain C: tests/c/abi_driver.c is compiled with gcc against include/bdr_mx.h,
linked with libbdr_mx.so, the oracle's library and the HIP runtime (no Python, no PyTorch in the
process), and run on the GPU.  It checks planes, dequantized values, the fused round trip (both
axes, a ragged shape) and the QSNR sweep against the oracle and exits non-zero on any difference."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def test_a_c_program_drives_the_library(tmp_path):
    lib_dir = os.path.join(ROOT, "paper_2302_08007_amd")
    ora_dir = os.path.join(ROOT, "oracle")
    assert os.path.exists(os.path.join(lib_dir, "libbdr_mx.so")), "build the library first"
    assert os.path.exists(os.path.join(ora_dir, "libbdr_ref.so")), "build the oracle first"
    exe = str(tmp_path / "abi_driver")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-Wno-unused-parameter",
           "-D_POSIX_C_SOURCE=200809L", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", ora_dir, "-isystem", os.path.join(ROCM, "include"),
           os.path.join(ROOT, "tests", "c", "abi_driver.c"), "-o", exe,
           "-L", lib_dir, "-lbdr_mx", "-L", ora_dir, "-lbdr_ref", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           "-lm", "-Wl,-rpath," + lib_dir, "-Wl,-rpath," + ora_dir, "-Wl,-rpath," + os.path.join(ROCM, "lib")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert r.stdout.startswith("ok:"), r.stdout
