"""Builds librad_hip.so (gfx950) from csrc/ with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librad_hip.so")
SOURCES = ["api.hip", "plan.hip", "small.hip", "gemm_f32.hip", "gemm_bf16.hip", "gemm_bf16_fwd.hip",
           "gemm_bf16_dx.hip", "gemm_bf16_dwd.hip", "gemm_bf16_sparse.hip", "gemm_bf16_sparse3.hip",
           "gemm_bf16_sparse7.hip", "optim.hip", "project.hip", "pde.hip", "paths.hip", "ceilings.hip", "conv.hip", "gemm_f32_ks.hip"]
# packed fp32 VALU forms are switched off: hipcc -O3 otherwise forms them on its own
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _stale(src, obj):
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    deps = [os.path.join(CSRC, src)] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    deps.append(os.path.join(HERE, "..", "include", "rad.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src, force=True):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    if not force and not _stale(src, obj):
        return obj, ""
    cmd = [_hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(ln for ln in r.stderr.splitlines() if "not a recognized feature" not in ln)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    return obj, err


def build(verbose=False, jobs=10, force=True):
    """force=False recompiles only sources older than their object (developer loop)."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if verbose:
        for _, err in results:
            if err.strip():
                print(err, file=sys.stderr)
    objs = [o for o, _ in results]
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, force="--incremental" not in sys.argv))
