"""Builds ``librocketkv.so`` (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librocketkv.so")
SOURCES = ["api.hip", "summaries.hip", "select.hip", "attend.hip", "attend_tok.hip", "decode.hip", "decode_tok.hip", "snapkv.hip", "probe.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Rpass-analysis=kernel-resource-usage",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Wall", "-Wno-unused-function"]
# what the compiler reports per kernel (registers, scratch, LDS, occupancy), one line each: a kernel
# that starts to spill costs HBM traffic without any test failing, so the CPU tests read this file
RESOURCES = os.path.join(HERE, "kernel_resources.txt")


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _resource_lines(src, remarks):
    """One line per kernel from the compiler's resource-usage remarks of one source file."""
    out, cur = [], None

    def val(line):
        return line.split("]:")[-1].split(":")[-1].replace("[-Rpass-analysis=kernel-resource-usage", "").strip().split()[0]

    for l in remarks:
        if "Function Name:" in l:
            if cur:
                out.append(cur)
            cur = {"name": l.split("Function Name:")[1].split()[0]}
        elif cur is not None:
            for key, tag in (("vgpr", " VGPRs:"), ("agpr", " AGPRs:"), ("sgpr", "TotalSGPRs:"), ("scratch", "ScratchSize"),
                             ("lds", "LDS Size"), ("occ", "Occupancy")):
                if tag in l:
                    cur[key] = val(l)
    if cur:
        out.append(cur)
    return [f"{src} {k['name']} {k.get('vgpr', '?')} {k.get('agpr', '?')} {k.get('sgpr', '?')} {k.get('scratch', '?')} "
            f"{k.get('lds', '?')} {k.get('occ', '?')}" for k in out]


def build(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library. Always recompiles."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        lines = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l]
        remarks = [l for l in lines if "-Rpass-analysis=kernel-resource-usage" in l]
        err = "\n".join(l for l in lines if "-Rpass-analysis=kernel-resource-usage" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj, _resource_lines(src, remarks)

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        done = list(ex.map(compile_one, SOURCES))
    objs = [d[0] for d in done]
    with open(RESOURCES, "w") as f:
        f.write("# source kernel(mangled) VGPRs AGPRs SGPRs scratch_bytes_per_lane LDS_bytes occupancy_waves_per_SIMD\n")
        for d in done:
            f.writelines(l + "\n" for l in d[1])
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
