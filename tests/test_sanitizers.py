"""Host-side sanitizer runs (AddressSanitizer + UndefinedBehaviorSanitizer; no GPU involved, device code untouched).

1. The CPU oracle: oracle/sparsek_oracle.c compiled under the sanitizers together with a C driver that calls every
   oracle routine on small ragged inputs and checks invariants (tests/san/oracle_san.c).
2. The boundary: the argument validation of every C-ABI entry point (csrc/api.hip, csrc/mask_static.hip, host side
   compiled under the sanitizers) called with null pointers and zero / negative / overflowing sizes
   (tests/san/abi_san.cpp); every call must return its error code before anything touches a GPU.
"""
import os
import subprocess
import tempfile

import paper_2406_16747_amd as spk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-3000:], r.stderr[-3000:])
    return r.stdout


def test_oracle_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_san")
        run(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-Wall"] + SAN + ["-o", exe,
             os.path.join(ROOT, "tests", "san", "oracle_san.c"), os.path.join(ROOT, "oracle", "sparsek_oracle.c"), "-lm"])
        out = run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=1"))
        assert "oracle_san ok" in out


def test_boundary_argument_checks_under_asan_and_ubsan():
    from paper_2406_16747_amd import build

    objdir = build.OBJ
    need = [s[:-4] + ".o" for s in build.sources()]
    if not os.path.exists(spk.lib_path()) or not all(os.path.exists(os.path.join(objdir, o)) for o in need):
        build.build()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    host_san = []
    for f in SAN:
        host_san += ["-Xarch_host", f]
    with tempfile.TemporaryDirectory() as tmp:
        objs = []
        for src in build.sources():
            if src in ("api.hip", "mask_static.hip"):  # the translation units that validate arguments
                o = os.path.join(tmp, src[:-4] + ".o")
                run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-fPIC", "-std=c++17"] + host_san +
                    ["-c", os.path.join(build.CSRC, src), "-o", o])
            else:
                o = os.path.join(objdir, src[:-4] + ".o")
            objs.append(o)
        drv = os.path.join(tmp, "abi_san.o")
        run([clangxx, "-O1", "-g", "-std=c++17"] + SAN + ["-c", os.path.join(ROOT, "tests", "san", "abi_san.cpp"), "-o", drv])
        exe = os.path.join(tmp, "abi_san")
        run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe,
             drv] + objs)
        out = run([exe], env=ENV)
        assert "abi_san ok" in out
