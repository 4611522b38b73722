"""Compile the HIP sources into paper_2401_12522_amd/libbita.so (gfx950 only)."""
import json
import os
import re
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
         # registers, scratch and occupancy of every kernel, as remarks on stderr (parsed below)
         "-Rpass-analysis=kernel-resource-usage",
         "-Wno-unused-command-line-argument"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    lines = [l for l in res.stderr.splitlines() if noise not in l]
    remarks = [l for l in lines if "[-Rpass-analysis=kernel-resource-usage]" in l]
    err = "\n".join(_without_remarks(lines))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return remarks


def _without_remarks(lines):
    """Drop the resource-usage remarks and the two source-echo lines that follow each."""
    out, skip = [], 0
    for l in lines:
        if "[-Rpass-analysis=kernel-resource-usage]" in l:
            skip = 2
            continue
        if skip and (re.match(r"^\s*\d+ \|", l) or re.match(r"^\s*\|\s*\^", l)):
            skip -= 1
            continue
        skip = 0
        out.append(l)
    return out


def _kernel_resources(remarks):
    """{mangled kernel name: {"vgprs", "agprs", "scratch", "occupancy"}} from the compiler's remarks."""
    res, cur = {}, None
    keys = {"VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch", "Occupancy [waves/SIMD]": "occupancy"}
    for l in remarks:
        m = re.search(r"remark:\s+(.*?):\s+(\S+) \[-Rpass", l)
        if not m:
            continue
        k, v = m.group(1).strip(), m.group(2)
        if k == "Function Name":
            cur = res.setdefault(v, {})
        elif cur is not None and k in keys:
            cur[keys[k]] = int(v)
    return res


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
        remarks = list(pool.map(lambda c: _run(c, verbose), cmds))
    resources = {}
    for r in remarks:
        resources.update(_kernel_resources(r))
    with open(os.path.join(obj_dir, tag + "_kernel_resources.json"), "w") as f:
        json.dump(resources, f, indent=1, sort_keys=True)
    # The skinny GEMM is written to fit its register budget in every instantiation: a spill inside
    # its loop is silent and costs percents of a step (scratch traffic shares the vector-memory
    # path and its wait counter with the weight stream), so it fails the build instead.
    spilled = sorted(k for k, v in resources.items() if "gemm_skinny_kernel" in k and v.get("scratch", 0) > 0)
    if spilled:
        raise RuntimeError("gemm_skinny_kernel instantiations that spill registers to scratch:\n  " + "\n  ".join(spilled))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib_path], verbose)
    return lib_path


if __name__ == "__main__":
    print(build_library(verbose=True))
