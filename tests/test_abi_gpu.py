"""The C ABI from a plain C99 program on a real GPU: no Python and no PyTorch between the caller and the library."""
import os
import shutil
import subprocess

import pytest

import paper_2411_09009_amd as L

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_program_calls_the_plain_entry_points_on_the_gpu(cce, tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None or not os.path.exists("/opt/rocm/include/hip/hip_runtime_api.h"):
        pytest.skip("no C compiler or no HIP headers")
    libdir = os.path.dirname(L.LIB_PATH)
    exe = str(tmp_path / "run_on_gpu")
    subprocess.run([gcc, "-std=c99", "-O1", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
                    os.path.join(ROOT, "tests", "abi_c", "run_on_gpu.c"), "-L", libdir, "-lcce", "-L", "/opt/rocm/lib",
                    "-lamdhip64", "-lm", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True)
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    print(r.stdout)
    assert r.returncode == 0 and "gpu run ok" in r.stdout, r.stdout
