"""Builds libcleave.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcleave.so")

SOURCES = ["plan.cpp", "scheduler.cpp", "api.cpp", "execute.hip", "execute_direct.hip", "reduce.hip", "verify.hip", "subset.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # the host-side planners compare doubles the oracle must reproduce: no fused multiply-adds
    "-Xarch_host", "-ffp-contract=off",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
    # no packed-fp32 instructions in device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _compile(src):
    obj = os.path.join(OBJ_DIR, src + ".o")
    cmd = [HIPCC] + COMMON + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    return src, obj, res


def build(verbose=True, extra=None):
    """Compiles every source (always; the call is the build check) and links."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    if extra:
        COMMON.extend(extra)
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_compile, SOURCES))
    objs = []
    for src, obj, res in results:
        text = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                         if "packed-fp32-ops" not in l and l.strip())
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, text))
        if verbose and text:
            print(text, file=sys.stderr)
        objs.append(obj)
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


def ensure_built(verbose=False):
    """Builds the library only if none is there (tests, the smoke check and the
    benchmark use what is built; after a change to a source, build again)."""
    if not os.path.exists(LIB):
        build(verbose=verbose)
    return LIB


if __name__ == "__main__":
    print(build(extra=sys.argv[1:]))
