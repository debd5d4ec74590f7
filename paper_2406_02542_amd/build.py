"""Builds the HIP library (libloki.so) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libloki.so")
SOURCES = ["api.hip", "score.hip", "select.hip", "attend.hip", "attend_mfma.hip", "fused.hip", "fused_gqa.hip", "fused_gqa_cluster.hip", "rotate.hip", "calibrate.hip"]
HEADERS = ["common.h", "launch.h", "score_impl.h", "select_impl.h", "attend_impl.h", "score_mfma_impl.h", "attend_mfma_impl.h", "fused_gqa_impl.h", "cluster_impl.h", os.path.join("..", "..", "include", "loki.h")]

# -packed-fp32-ops is switched off on purpose: the compiler must not form v_pk_*_f32.
HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def find_hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found (looked at $HIPCC, /opt/rocm/bin/hipcc and PATH)")


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > built for d in deps)


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    return proc.returncode, proc.stdout, err


def build(verbose: bool = True) -> str:
    """Compiles every HIP source into paper_2406_02542_amd/libloki.so (always recompiles):
    one object per source, compiled in parallel, then one link."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = find_hipcc()
    obj_dir = os.path.join(PKG_DIR, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]

    def compile_one(src):
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + flags + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print("[build]", " ".join(cmd), flush=True)
        return (src, obj) + _run(cmd)

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 4)) as ex:
        results = list(ex.map(compile_one, SOURCES))
    for src, obj, rc, out, err in results:
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {src} ({rc}):\n{out}\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH + ".tmp"] + \
        [r[1] for r in results]
    if verbose:
        print("[build]", " ".join(link), flush=True)
    rc, out, err = _run(link)
    if rc != 0:
        raise RuntimeError(f"link failed ({rc}):\n{out}\n{err}")
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
