"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/*.h declares, sizes its workspaces as documented and rejects bad
arguments before launching anything."""
import ctypes
import os
import re

import pytest

import paper_2411_09009_amd as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for h in sorted(os.listdir(inc)):
        if h.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, h)).read(), flags=re.S)
            names |= set(re.findall(r"\b(cce_[a-z_]+)\s*\(", text))
    return sorted(names)


# The boundary: the two plain calls (cce_forward, cce_backward), their extended forms, the sizing / option / reporting helpers
# they need, the registration that lends the plain calls their scratch, and the allocation-free forward.
BOUNDARY = {"cce_forward", "cce_backward", "cce_forward_ex", "cce_backward_ex", "cce_workspace_bytes",
            "cce_block_max_bytes", "cce_strerror", "cce_default_opts", "cce_filter_block",
            "cce_backward_filter_stats", "cce_forward_target_stats", "cce_set_workspace",
            "cce_forward_noalloc", "cce_noalloc_scratch_bytes"}


def test_library_exports_exactly_the_declared_boundary():
    import subprocess
    lib = L.load()
    names = declared_symbols()
    assert set(names) == BOUNDARY
    for n in names:
        assert hasattr(lib, n), n
    # and nothing else with the library's prefix: measurement probes live in a shared object of their own
    out = subprocess.run(["nm", "-D", "--defined-only", L.LIB_PATH], stdout=subprocess.PIPE, text=True, check=True).stdout
    exported = {line.split()[-1] for line in out.splitlines() if line.split()[-1].startswith("cce_")}
    assert exported == BOUNDARY, exported ^ BOUNDARY


def test_the_library_never_allocates_frees_or_synchronises_the_device():
    src = os.path.join(ROOT, "paper_2411_09009_amd", "csrc")
    for f in sorted(os.listdir(src)):
        path = os.path.join(src, f)
        if os.path.isfile(path):
            text = open(path).read()
            for word in ("hipMalloc", "hipFree", "hipDeviceSynchronize", "hipHostMalloc", "hipMemset"):
                assert word not in text, (f, word)


def test_plain_entry_points_need_a_lent_workspace():
    lib = L.load()
    buf = (ctypes.c_char * 4096)()
    p = (ctypes.addressof(buf) + 255) // 256 * 256
    # argument errors first, nothing touches the device
    assert lib.cce_forward(None, p, p, 4, 64, 8, 0.0, -100, p, p) == -1
    assert lib.cce_backward(p, p, p, 4, 64, 8, -1.0, -100, p, p, p, p) == -1
    assert lib.cce_set_workspace(p + 8, 1024) == -1          # misaligned
    assert lib.cce_set_workspace(None, 1024) == -1           # pointer / size inconsistent
    assert lib.cce_set_workspace(p, 0) == -1


def test_binding_exposes_the_same_names():
    for n in declared_symbols():
        assert hasattr(L, n), n


def test_default_opts_and_error_strings():
    o = L.cce_default_opts(L.CCE_BF16)
    assert o.flags == (L.CCE_FILTER_DE | L.CCE_FILTER_DC) and o.filter_eps == 2.0 ** -12
    o = L.cce_default_opts(L.CCE_F32)
    assert o.flags == 0 and o.filter_eps == 0.0
    for st in (0, -1, -2, -3, -4, -99):
        assert isinstance(L.cce_strerror(st), str) and L.cce_strerror(st)


def test_forward_workspace_is_linear_in_tokens_and_independent_of_vocabulary():
    o = L.cce_default_opts(L.CCE_BF16)
    a = L.cce_workspace_bytes(L.CCE_OP_FORWARD, 8192, 2304, 256000, o)
    b = L.cce_workspace_bytes(L.CCE_OP_FORWARD, 8192, 2304, 128000, o)
    c = L.cce_workspace_bytes(L.CCE_OP_FORWARD, 16384, 2304, 256000, o)
    assert a == b                          # no O(V) term
    assert a <= 8192 * 8 * 8 + 512         # at most 8 (max, sum) pairs per token, plus the counters
    assert c <= 2 * a + 256
    logits_bytes = 8192 * 256000 * 4
    assert a < logits_bytes / 10000


def test_backward_workspace_is_bounded_by_the_slab_not_the_vocabulary():
    o = L.cce_default_opts(L.CCE_BF16)
    N, D = 8192, 2304
    rec = L.cce_workspace_bytes(L.CCE_OP_BACKWARD, N, D, 256000, o)
    rec2 = L.cce_workspace_bytes(L.CCE_OP_BACKWARD, N, D, 1024000, o)
    mn = L.cce_workspace_bytes(L.CCE_OP_BACKWARD_MIN, N, D, 256000, o)
    # the only |V|-dependent part is one 4-byte filter flag per 256 x 64 and per 64 x 256 block of logits
    assert 0 <= rec2 - rec <= N * (1024000 - 256000) // 2048 + 4096 and 0 < mn < rec
    assert rec < N * 256000 * 2 / 5        # far below even a bf16 logit matrix
    # a larger workspace buys slabs up to four times as wide, never more
    wide = L.cce_workspace_bytes(L.CCE_OP_BACKWARD_WIDE, N, D, 256000, o)
    assert rec < wide <= 4 * rec
    # small vocabulary: one slab already holds all of it, so there is nothing to widen
    assert (L.cce_workspace_bytes(L.CCE_OP_BACKWARD_WIDE, N, D, 4096, o)
            == L.cce_workspace_bytes(L.CCE_OP_BACKWARD, N, D, 4096, o))
    # the widest slab stays addressable with 32-bit element offsets at the largest benchmark shape
    big = L.cce_workspace_bytes(L.CCE_OP_BACKWARD_WIDE, 65536, 5120, 131072, o)
    assert big <= 65536 * 5120 * 4 + 2 * 2 * 2 ** 30 + 64 * 2 ** 20
    assert L.cce_workspace_bytes(99, N, D, 256000, o) == 0
    assert L.cce_workspace_bytes(L.CCE_OP_FORWARD, 0, D, 256000, o) == 0


def test_bad_arguments_are_rejected_without_a_gpu():
    lib = L.load()
    o = L.cce_default_opts(L.CCE_BF16)
    buf = (ctypes.c_char * 4096)()
    p = (ctypes.addressof(buf) + 255) // 256 * 256
    args = dict(E=p, C=p, t=p, N=4, D=64, V=8, cap=0.0, ign=-100, loss=p, lse=p)

    def fwd(**kw):
        a = dict(args, **kw)
        return lib.cce_forward_ex(a["E"], a["C"], a["t"], a["N"], a["D"], a["V"], a["cap"], a["ign"],
                                  a["loss"], a["lse"], ctypes.byref(kw.get("opts", o)))
    assert fwd(E=None) == -1
    assert fwd(N=0) == -1 and fwd(V=-3) == -1 and fwd(D=0) == -1
    assert fwd(cap=-1.0) == -1 and fwd(cap=float("nan")) == -1
    assert fwd(E=p + 2) == -1                       # misaligned
    assert fwd(loss=None) == -1
    assert fwd() == -2                              # no workspace
    bad = L.cce_default_opts(L.CCE_BF16)
    bad.dtype = 7
    assert fwd(opts=bad) == -3
    bad = L.cce_default_opts(L.CCE_BF16)
    bad.flags = 1 << 9
    assert fwd(opts=bad) == -3
    bad = L.cce_default_opts(L.CCE_BF16)
    bad.filter_eps = -0.5
    assert fwd(opts=bad) == -1
    r = lib.cce_backward_ex(p, p, p, 4, 64, 8, 0.0, -100, None, p, p, p, ctypes.byref(o))
    assert r == -1
    r = lib.cce_backward_ex(p, p, p, 4, 64, 8, 0.0, -100, p, p, p, p, ctypes.byref(o))
    assert r == -2


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2411_09009_amd.binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libcce.so")
    with pytest.raises(FileNotFoundError):
        B.load()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2411_09009_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no CPU or eager", ""), (f, "mentions the oracle")


def test_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    """include/cce.h is C99 (no C++ needed), and a C program linked against libcce.so can call it."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    L.load()
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    for h in sorted(os.listdir(inc)):
        subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(inc, h)], check=True)
    libdir = os.path.dirname(L.LIB_PATH)
    exe = str(tmp_path / "use_from_c")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-I", inc, os.path.join(root, "tests", "abi_c", "use_from_c.c"),
                    "-L", libdir, "-lcce", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True)
    r = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
    assert r.returncode == 0, r.stdout
    assert r.stdout.startswith("forward ")


def test_host_code_under_address_and_undefined_sanitizers(tmp_path):
    """The dispatcher's host code (argument checks, workspace layouts, slab fitting) built with the address and
    undefined-behaviour sanitizers (host side only: device code is compiled as usual) and driven by a C program
    that sweeps shapes from 1 to the ABI's limits over every layout-changing flag.  No call reaches the GPU."""
    import glob
    import shutil
    import subprocess
    from paper_2411_09009_amd import build as B
    clang = "/opt/rocm/lib/llvm/bin/clang"
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not (os.path.exists(B.HIPCC) and os.path.exists(clang) and rt):
        pytest.skip("no ROCm clang with sanitizer runtimes")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = [f for f in B.FLAGS if f != "-O3"] + ["-O1", "-g"]
    objs = []
    procs = []
    for src in B.SOURCES:
        obj = str(tmp_path / src.replace(".hip", ".o"))
        objs.append(obj)
        procs.append(subprocess.Popen([B.HIPCC, *flags, *san, "-c", os.path.join(B.CSRC, src), "-o", obj],
                                      stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    for pr in procs:
        out, _ = pr.communicate()
        assert pr.returncode == 0, out
    lib = str(tmp_path / "libcce_san.so")
    subprocess.run([B.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-shared-libsan", *objs, "-o", lib], check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    exe = str(tmp_path / "host_sweep")
    subprocess.run([clang, "-std=c99", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
                    "-shared-libsan", "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "abi_c", "host_sweep.c"),
                    "-L", str(tmp_path), "-lcce_san", "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath,/opt/rocm/lib",
                    "-Wl,-rpath," + os.path.dirname(rt[0]), "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env)
    if r.returncode != 0 and "ASan runtime does not come first" in r.stdout:
        pytest.skip("another preloaded library precedes the sanitizer runtime in this environment")
    assert r.returncode == 0 and "host sweep ok" in r.stdout, r.stdout
    shutil.rmtree(str(tmp_path), ignore_errors=True)
