"""Compile the HIP sources into paper_2401_12522_amd/libbita.so (gfx950 only)."""
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libbita.so")
SOURCES = ["api.hip", "gemm.hip", "attention.hip", "misc.hip", "tree.hip", "prefill.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # kernel arguments arrive in SGPRs with the wave instead of through a scalar load at
         # the head of every kernel (267 launches per step)
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wno-unused-command-line-argument"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose=False, extra_flags=(), lib_path=LIB_PATH):
    """Every source is compiled to an object of its own (side by side, one process each: no
    device symbol crosses a file), then linked."""
    from concurrent.futures import ThreadPoolExecutor
    obj_dir = os.path.join(PKG_DIR, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    tag = os.path.splitext(os.path.basename(lib_path))[0]
    objs = [os.path.join(obj_dir, tag + "_" + s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[HIPCC] + FLAGS + list(extra_flags) + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(len(cmds), os.cpu_count() or 1)) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib_path], verbose)
    return lib_path


if __name__ == "__main__":
    print(build_library(verbose=True))
