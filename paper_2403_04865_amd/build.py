"""Build libslide.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2403_04865_amd.build            # incremental
    python -m paper_2403_04865_amd.build --force    # recompile everything
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libslide.so")
SOURCES = ["slide_lib.hip", "misc.hip", "ln.hip", "gemm.hip", "gemm_mfma.hip", "gemm_nt_mfma.hip", "gemm_nt_big.hip", "gemm_nt_gelu.hip", "gemm_tn_big.hip", "attn.hip", "attn_mfma.hip", "cls_lane.hip", "pool.hip", "pool_mfma.hip", "pool_bwd_mfma.hip", "optim.hip",
           "conv.hip", "bn_pool.hip", "resnet_lib.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if p and (os.path.isabs(p) and os.path.exists(p) or not os.path.isabs(p)):
            return p
    raise RuntimeError("hipcc not found")


def _newer(src_files, target):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(s) > t for s in src_files)


def build(force: bool = False, verbose: bool = True, extra_flags=()):
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers += [os.path.join(HERE, "..", "include", h) for h in ("slide.h", "slide_prof.h", "resnet.h")]
    hipcc = _hipcc()
    jobs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", ".o"))
        if force or _newer([s] + headers, o):
            jobs.append((s, o))

    def compile_one(job):
        s, o = job
        cmd = [hipcc, *FLAGS, *extra_flags, *os.environ.get("SLIDE_HIPCC_FLAGS", "").split(), "-c", s, "-o", o]
        p = subprocess.run(cmd, capture_output=True, text=True)
        # the host pass does not know the gfx-only feature flag and says so: not an error
        err = "\n".join(l for l in p.stderr.splitlines() if "packed-fp32-ops" not in l)
        return s, p.returncode, err

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        results = list(ex.map(compile_one, jobs))
    for s, rc, err in results:
        if verbose and err.strip():
            print(f"[hipcc] {os.path.basename(s)}:\n{err}", file=sys.stderr)
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {s}")
    objs = [os.path.join(OBJ, src.replace(".hip", ".o")) for src in SOURCES]
    if force or jobs or _newer(objs, LIB):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        p = subprocess.run(cmd, capture_output=True, text=True)
        if p.returncode != 0:
            print(p.stderr, file=sys.stderr)
            raise RuntimeError("link failed")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
