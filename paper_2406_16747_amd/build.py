"""Builds libsparsek.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to build.

Besides the library the build writes libsparsek.toolchain.json: the compiler it used and the result of a check of
the generated code.  Three kernels (attention forward, mask backward, dK/dV) issue direct-to-LDS loads from inline
assembly that sets the M0 register itself; that is only sound while the compiler keeps no value of its own in M0
inside those kernels.  The check reads the device assembly of every translation unit and accepts a mention of M0
only in the three-instruction pattern of those loads.
"""
import json
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsparsek.so")
OBJ = os.path.join(HERE, "_build")
SIDECAR = os.path.join(HERE, "libsparsek.toolchain.json")

# The compiler the kernels' hand-written M0 handling was validated with (GPU parity tests green).  Another version
# is not wrong by itself -- check_m0 below looks at the code it generates -- but the tests ask for a fresh validation.
VALIDATED_HIPCC = "HIP version: 7.2.26015"

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-result",
    # packed-fp32 VALU forms are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def check_m0(asm_path):
    """Per kernel of a device assembly file: the mentions of M0 are either all inside inline-assembly regions (the
    hand-written direct-to-LDS loads of attn_tiles.hpp, which set M0 themselves) or all outside (M0 managed by the
    compiler, e.g. for the builtin form of the same loads).  A kernel with both would let the hand-written loads
    clobber a value the compiler keeps in M0.  Returns {kernel: number of hand-written loads}; raises on a mix."""
    found = {}
    name, in_asm, ours, theirs = None, False, 0, []
    for raw in open(asm_path, errors="replace"):
        ln = raw.strip()
        if ln.startswith(";;#ASMSTART"):
            in_asm = True
        elif ln.startswith(";;#ASMEND"):
            in_asm = False
        elif ln.startswith(".Lfunc_end"):
            if ours and theirs:
                raise RuntimeError("%s: kernel %s sets M0 by hand (%d loads) while the compiler uses it too: `%s`"
                                   % (os.path.basename(asm_path), name, ours, theirs[0]))
            if ours:
                found[name] = ours
            name, ours, theirs = None, 0, []
        elif re.match(r"^[A-Za-z_][\w$.]*:", ln) and not ln.startswith(".L"):
            name = ln.split(":")[0]
        else:
            code = ln.split(";")[0]
            if re.search(r"\bm0\b", code):
                if in_asm:
                    ours += 1 if code.startswith("s_mov_b32 m0") else 0
                else:
                    theirs.append(code)
    return found


def build(verbose=False):
    """Compiles every .hip file and links the shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)

    def one(src):
        obj = os.path.join(OBJ, src[:-4] + ".o")
        cmd = [hipcc] + FLAGS + ["-save-temps=obj", "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stderr[-4000:]))
        if verbose and r.stderr.strip():
            print(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(one, sources()))
    tmp = LIB + ".tmp%d" % os.getpid()
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr[-4000:])
    os.replace(tmp, LIB)
    version = subprocess.run([hipcc, "--version"], capture_output=True, text=True).stdout.strip()
    loads = {}
    for src in sources():
        asm = os.path.join(OBJ, src[:-4] + "-hip-amdgcn-amd-amdhsa-gfx950.s")
        n = check_m0(asm)
        if n:
            loads[src] = sum(n.values())
    with open(SIDECAR, "w") as f:
        json.dump({"hipcc_version": version.splitlines(), "flags": FLAGS,
                   "m0_check": "ok", "untracked_direct_to_lds_loads": loads}, f, indent=1)
    keep = {src[:-4] + ".o" for src in sources()}
    for name in os.listdir(OBJ):   # the intermediate files of -save-temps
        if name not in keep:
            os.remove(os.path.join(OBJ, name))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
