"""Build libgspc.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgspc.so")

SOURCES = ["gspc_api.cpp", "pack_kernels.hip", "chain_kernels.hip",
           "direct_kernels.hip", "mfma_kernels.hip", "mfma4_kernels.hip", "mfmab_kernels.hip",
           "mfmaw_kernels.hip", "fused_kernels.hip", "dw_kernels.hip", "dwpw_kernels.hip", "wino_kernels.hip", "rowb_kernels.hip", "gpw_kernels.hip", "tune_table.cpp"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]
if os.environ.get("GSPC_PHASE_TIMING"):      # developer aid: per-phase timestamps
    FLAGS.append("-DGSPC_PHASE_TIMING")


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _deps_mtime():
    paths = [os.path.join(ROOT, "include", "gspc.h")]
    paths += [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    return max(os.path.getmtime(p) for p in paths)


def _compile(src):
    obj = os.path.join(OBJ, src + ".o")
    cmd = [_hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines()
                     if "packed-fp32-ops" not in l and l.strip())
    return obj, warn


def build(force=True, verbose=False):
    """Compiles every source and links libgspc.so.  With force=False an
    up-to-date library is reused."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= _deps_mtime():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = [o for o, _ in results]
    if verbose:
        for _, w in results:
            if w:
                print(w, file=sys.stderr)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
