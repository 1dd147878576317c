"""Builds librelax_mi355.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librelax_mi355.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC] + os.environ.get("RELAX_EXTRA_HIPCC_FLAGS", "").split()


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


# Sources whose kernels stream from HBM with their working set in registers: a variant that the register allocator
# spills to scratch memory still computes the right values, several times slower (measured: 4 x on a one-row matvec), so
# the build refuses it.  {source: substring of the mangled kernel names it applies to}
NO_SCRATCH = {"gemv_q4_reg.hip": "gemv_q4_reg_kernel", "gemv_reg_f16.hip": "gemv_q4_reg_kernel", "gemv_reg_q3.hip": "gemv_q4_reg_kernel", "gemv_q4_long.hip": "gemv_q4_long_kernel",
              "gemv_q3.hip": "gemv_q3", "attn_decode.hip": "attn_"}
REMARK = "-Rpass-analysis=kernel-resource-usage"


def scratch_users(remarks: str, name_part: str):
    """(kernel, bytes per lane) of every kernel in the compiler's resource-usage remarks that uses scratch memory."""
    bad, name = [], None
    for line in remarks.splitlines():
        if "remark: Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line and name is not None:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if size > 0 and name_part in name:
                bad.append((name, size))
    return bad


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src[:-4] + ".o")
    guarded = src in NO_SCRATCH
    cmd = [HIPCC] + FLAGS + ([REMARK] if guarded else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    if guarded:
        bad = scratch_users(res.stderr, NO_SCRATCH[src])
        if bad:
            raise RuntimeError("%s: kernels that spill to scratch memory: %s" % (src, ", ".join("%s (%d B/lane)" % b for b in bad)))
        res.stderr = "\n".join(l for l in res.stderr.splitlines() if REMARK not in l and not l.lstrip().startswith(("|", "^", "In file included from")) and
                               not (l.strip()[:1].isdigit() and "|" in l))
    warn = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as pool:
        objs = list(pool.map(_compile, sources()))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
