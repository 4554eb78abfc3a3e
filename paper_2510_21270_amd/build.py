"""Build libpbs.so (the C-ABI library of hand-written HIP kernels) for gfx950, in-tree.

Usage: python -m paper_2510_21270_amd.build [--force]
hipcc cross-compiles without a GPU.  Every .hip file is compiled to an object in parallel, then linked.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libpbs.so")
SOURCES = ["status.hip", "key_scores.hip", "permute.hip", "block_mask.hip", "attn_fwd.hip", "attn_wide.hip",
           "mfma_probe.hip", "coverage.hip", "query_permute.hip"]
HEADERS = ["pbs_device.h", "pbs_host.h", os.path.join("..", "..", "include", "pbs.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-array-bounds",
         # packed fp32 instructions are kept off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _newest(paths):
    return max(os.path.getmtime(p) for p in paths)


def _compile(src, force):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    deps = [os.path.join(CSRC, src)] + [os.path.join(CSRC, h) for h in HEADERS]
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= _newest(deps):
        return obj, ""
    cmd = ["hipcc"] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stdout))
    return obj, res.stdout


def build(force=False, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        results = list(ex.map(lambda s: _compile(s, force), SOURCES))
    objs = [r[0] for r in results]
    if verbose:
        for _, out in results:
            lines = [l for l in out.splitlines() if "not a recognized feature" not in l]
            if lines:
                print("\n".join(lines))
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < _newest(objs):
        tmp = LIB + ".tmp.%d" % os.getpid()
        res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                             stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stdout)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
