"""Compile the HIP sources into paper_2411_09009_amd/lib/libcce.so for gfx950.

hipcc cross-compiles without a GPU.  Objects go to a scratch directory outside
the package; only the shared library stays in-tree (git-ignored)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libcce.so")
SOURCES = ["cce_api.hip", "plain_kernels.hip", "fwd_mfma.hip", "bwd_mfma.hip", "sort_kernels.hip"]
# the benchmark's measurement probes: a shared object of their own, loaded by bench.py only
PROBE_LIB_PATH = os.path.join(LIB_DIR, "libcce_probe.so")
PROBE_SOURCES = [os.path.join("probe", "probe_kernels.hip")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep hipcc from forming packed-fp32 instructions on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False) -> str:
    """Compiles libcce.so (the product) and libcce_probe.so (bench.py's probes); returns the former's path."""
    os.makedirs(LIB_DIR, exist_ok=True)
    with tempfile.TemporaryDirectory(prefix="cce_build_") as tmp:
        every = SOURCES + PROBE_SOURCES
        objs = [os.path.join(tmp, os.path.basename(s).replace(".hip", ".o")) for s in every]
        cmds = [[HIPCC, *FLAGS, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(every, objs)]
        with ThreadPoolExecutor(max_workers=min(6, len(cmds))) as ex:
            for out in ex.map(_run, cmds):
                if verbose and out.strip():
                    print(out)
        for path, group in ((LIB_PATH, objs[:len(SOURCES)]), (PROBE_LIB_PATH, objs[len(SOURCES):])):
            tmp_lib = os.path.join(tmp, os.path.basename(path))
            _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *group, "-o", tmp_lib])
            staged = path + ".tmp"
            shutil.copyfile(tmp_lib, staged)
            os.replace(staged, path)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
