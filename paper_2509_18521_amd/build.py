"""Builds the HIP library (libapril.so) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libapril.so")
OBJ_DIR = os.path.join(PKG, "_build")
SOURCES = ["engine.hip", "kernels_basic.hip", "kernels_gemm.hip", "kernels_gemm_tile.hip", "kernels_attn.hip", "kernels_moe.hip", "kernels_sample.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-unused-value", "-Wno-unused-result"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose=True, incremental=False):
    """Compiles every source and links.  incremental: only the sources whose object is older than
    the source or than any header (development shortcut; the default compiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = {s: os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES}
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(PKG), "include", "april.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)

    def stale(s):
        if not incremental or not os.path.exists(objs[s]):
            return True
        t = os.path.getmtime(objs[s])
        return t < os.path.getmtime(os.path.join(CSRC, s)) or t < newest_header
    todo = [s for s in SOURCES if stale(s)]
    with ThreadPoolExecutor(max_workers=min(8, len(todo) or 1)) as ex:
        list(ex.map(lambda s: _run([hipcc] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", objs[s]], verbose), todo))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [objs[s] for s in SOURCES] + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv[1:])
    print("built", LIB)
