"""Builds libmmaemu.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libmmaemu.so")

COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          "-Wall", "-Wno-unused-function",
          # packed-FP32 VALU forms are not to be generated on the test machines
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the NORMAL generator is defined as a fixed sequence of IEEE operations: no fused multiply-add
PER_FILE = {"gen.hip": ["-ffp-contract=off"], "emulate_addmul.hip": ["-ffp-contract=off"]}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src):
    obj = os.path.join(OBJ, src[:-4] + ".o")
    cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj] + COMMON + PER_FILE.get(src, [])
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, obj, r


def _stale(src):
    """True when the object of `src` is older than the source or than any header."""
    obj = os.path.join(OBJ, src[:-4] + ".o")
    if not os.path.exists(obj):
        return True
    deps = [os.path.join(CSRC, src)] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    deps += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    return any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps)


def build_library(verbose=True, jobs=8, only_stale=False):
    """Compiles every source (only_stale: those whose object is out of date) and links the library."""
    os.makedirs(OBJ, exist_ok=True)
    todo = [s for s in sources() if not only_stale or _stale(s)]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(_compile, todo))
    objs = [os.path.join(OBJ, s[:-4] + ".o") for s in sources() if s not in todo]
    for src, obj, r in results:
        warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stderr))
        if verbose and warn:
            print("[%s]\n%s" % (src, warn), file=sys.stderr)
        objs.append(obj)
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(only_stale="--stale" in sys.argv[1:]))
