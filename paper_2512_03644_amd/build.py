"""Builds libffsnap.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libffsnap.so")
SOURCES = ["api.hip", "kernels.hip", "fused.hip", "layout.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Wno-align-mismatch",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]
_NOISE = ("packed-fp32-ops", "target feature")


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stderr)
    return "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in _NOISE))


def build(verbose=False):
    """Always recompiles every source (one hipcc process per file, side by side), then links;
    returns the path of the library."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    cmds = [["hipcc"] + FLAGS + ["-c", "-o", o, os.path.join(CSRC, s)]
            for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(len(cmds)) as ex:
        errs = list(ex.map(_run, cmds))
    errs.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs))
    if verbose:
        for e in errs:
            if e.strip():
                print(e)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
