"""The library's host-side logic (argument checks, layouts, workspace sizes, launch planning up to the first HIP call)
rebuilt with the undefined-behaviour sanitizer and driven through the C ABI without a GPU.

Only `api.hip` is recompiled (its host half with -fsanitize=undefined, aborting on the first report) and linked against
the objects of the regular build; a child process loads that library and sweeps the host-only entry points over
ordinary, degenerate and extreme descriptors, comparing every result with the regular library's.  Signed overflow in a
size computation, a shift past the width or a misaligned access in the checks would end the child with a report.
"""
import glob
import os
import subprocess
import sys
import textwrap

import pytest

from paper_2410_08661_amd import build as qbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = textwrap.dedent('''
    import ctypes as C, itertools, sys
    from paper_2410_08661_amd import binding as B
    san = C.CDLL(sys.argv[1])
    for name, (res, args) in B.EXPORTS.items():
        fn = getattr(san, name)
        fn.restype, fn.argtypes = res, args
    n = 0
    big = 2**31 - 1
    dims = [0, 1, 7, 8, 64, 129, 4096, 11008, 28672, 2**20, 2**30, big]
    ks = [0, 8, 21, 128, 256, 4096, big]
    for oc, ic, k, bits, g, layout in itertools.product(dims, dims, ks, (3, 4, 5), (0, 32, 100, 128, 2**20), (0, 1, 7)):
        d = B.make_desc(oc, ic, k, bits, g, layout)
        la, lb = B.qeft_layout_t(), B.qeft_layout_t()
        ra, rb = B.raw.qeft_layout(C.byref(d), C.byref(la)), san.qeft_layout(C.byref(d), C.byref(lb))
        assert ra == rb and bytes(la) == bytes(lb), (oc, ic, k, bits, g, layout)
        for op in range(-1, 8):
            for m in (-1, 0, 1, 16, 17, 300, 4096, 2**31, 2**40):
                assert B.raw.qeft_workspace_bytes(C.byref(d), op, m) == san.qeft_workspace_bytes(C.byref(d), op, m), (oc, ic, k, bits, g, layout, op, m)
                n += 1
    for dd in (0, 8, 4096, big):
        for t in (-1, 0, 1, 4096, 2**40):
            assert B.raw.qeft_sensitivity_workspace(dd, t) == san.qeft_sensitivity_workspace(dd, t)
    # argument checks of the compute entry points: every call below must return before a launch
    w = B.qeft_weight_t(0x10000, 0x20000, 0x30000, 0x40000)
    X, Y, WS = 0x100000, 0x200000, 0x4000000
    for oc, ic, k in ((64, 256, 128), (4096, 4096, 128), (28672, 8192, 256), (big, big, 0)):
        d = B.make_desc(oc, ic, k, 4)
        for m in (-5, 0):
            for fn in (B.raw, san):
                fn.qeft_linear_fwd(C.byref(d), C.byref(w), X, m, ic, Y, oc, None, 0, None)
                fn.qeft_linear_bwd_dx(C.byref(d), C.byref(w), Y, m, oc, X, ic, None, 0, None)
                fn.qeft_weak_grad(C.byref(d), Y, m, oc, X, max(k, 8), WS, 1, 0, None, 0, None)
                fn.qeft_linear_bwd(C.byref(d), C.byref(w), Y, m, oc, X, ic, X, max(k, 8), WS, 1, 0, None, 0, None)
        for fn in (B.raw, san):   # misaligned, too-small and missing operands
            assert fn.qeft_linear_fwd(C.byref(d), C.byref(w), X + 2, 4, ic, Y, oc, None, 0, None) == B.raw.qeft_linear_fwd(C.byref(d), C.byref(w), X + 2, 4, ic, Y, oc, None, 0, None)
            assert fn.qeft_linear_fwd(C.byref(d), None, X, 4, ic, Y, oc, None, 0, None) != B.QEFT_OK
            assert fn.qeft_linear_bwd(C.byref(d), C.byref(w), Y, 4096, oc, X, ic, None, 8, WS, 1, 0, None, 0, None) != B.QEFT_OK
    for s in range(-3, 12):
        assert B.raw.qeft_status_string(s) == san.qeft_status_string(s)
    print("calls compared:", n)
''')


@pytest.mark.skipif(not os.path.exists(qbuild.HIPCC), reason="needs hipcc")
def test_host_logic_under_ubsan(tmp_path):
    objs = [os.path.join(qbuild.BUILD_DIR, f[:-4] + ".o") for f in qbuild.SOURCES if f != "api.hip"]
    if not all(os.path.exists(o) for o in objs):
        pytest.skip("regular build objects are missing: run `python -m paper_2410_08661_amd.build` first")
    api_o, lib = str(tmp_path / "api_ubsan.o"), str(tmp_path / "libqeft_ubsan.so")
    san = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = [f for f in qbuild.FLAGS if f != "-O3"]
    subprocess.run([qbuild.HIPCC, *flags, "-O1", "-g", *san, "-c", os.path.join(qbuild.CSRC, "api.hip"), "-o", api_o], check=True, capture_output=True)
    # a shared library does not get the sanitizer's runtime by itself: link the toolchain's shared one, found beside
    # the compiler's other runtime libraries, and let the child find it through the library's run path
    rt_dirs = glob.glob(os.path.join(os.path.dirname(os.path.realpath(qbuild.HIPCC)), "..", "lib", "llvm", "lib", "clang", "*", "lib", "linux"))
    rt = [d for d in rt_dirs if os.path.exists(os.path.join(d, "libclang_rt.ubsan_standalone-x86_64.so"))]
    if not rt:
        pytest.skip("the toolchain ships no shared UBSan runtime")
    subprocess.run([qbuild.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, api_o, *objs, "-L", rt[0],
                    "-l:libclang_rt.ubsan_standalone-x86_64.so", f"-Wl,-rpath,{os.path.realpath(rt[0])}"], check=True, capture_output=True)
    r = subprocess.run([sys.executable, "-c", CHILD, lib], cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "runtime error" not in r.stderr, r.stderr[-3000:] + r.stdout[-500:]
    assert "calls compared:" in r.stdout
