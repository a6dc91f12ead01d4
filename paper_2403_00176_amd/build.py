"""Builds libsod2.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsod2.so")
SOURCES = ["expr.cpp", "rdp.cpp", "plan.cpp", "bind.cpp", "api.cpp", "kernels.hip", "gemm.hip", "attention.hip", "run.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def build(verbose: bool = False) -> str:
    out_dir = os.path.join(HERE, "_build")
    os.makedirs(out_dir, exist_ok=True)
    cc = _hipcc()

    def compile_one(src):
        obj = os.path.join(out_dir, src + ".o")
        cmd = [cc] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if src.endswith(".hip"):
            cmd.append("-Rpass-analysis=kernel-resource-usage")
        r = subprocess.run(cmd, capture_output=True, text=True)
        remarks = [l for l in r.stderr.splitlines() if "[-Rpass-analysis=kernel-resource-usage]" in l]
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and
                        "-Rpass-analysis=kernel-resource-usage" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"{' '.join(cmd)}\n{err}")
        # No kernel may keep data in scratch (private) memory: an array the compiler could not hold in
        # registers turns every access into a global memory round trip (this once cost the attention
        # kernel 2 us per launch without any warning).
        name = None
        for l in remarks:
            if "Function Name:" in l:
                name = l.split("Function Name:")[1].split("[")[0].strip()
            for key in ("ScratchSize [bytes/lane]:", "VGPRs Spill:"):
                if key in l and int(l.split(key)[1].split("[")[0].strip()) != 0:
                    raise RuntimeError(f"{src}: kernel {name} uses scratch memory ({l.split('remark:')[1].strip()})")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
