"""Build liboccult.so (HIP, gfx950 only) next to this file.

    python -m paper_2505_13345_amd.build

Every translation unit under csrc/ is compiled with hipcc for gfx950 and linked into one shared
library with a C ABI (include/occult.h).  Objects go to _build/ (ignored by git)."""
from __future__ import annotations

import concurrent.futures
import os
import re
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(ROOT, "_build", "occult")
LIB_PATH = os.path.join(HERE, "liboccult.so")

SOURCES = ["api.hip", "route.hip", "plan.hip", "dispatch.hip", "ffn.hip", "combine.hip", "combine_atomic.hip", "coact.hip", "backward.hip",
           "ffn_backward.hip", "wgrad.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed-fp32 instruction forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    # per-kernel register and scratch figures, checked below
    "-Rpass-analysis=kernel-resource-usage",
    "-I" + os.path.join(ROOT, "include"),
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the occult library cannot be built")
    return exe


# Kernels that must not touch scratch memory: in the persistent 256-row GEMM every reload of a spilled
# register waits for all outstanding loads, the next tile's prefetch included (a one-register change in
# its epilogue has cost 20 % before).  Matched against the mangled kernel names.
NO_SCRATCH = ("t256",)


def _resource_usage(stderr: str):
    """(kernel name, scratch bytes per lane) from the compiler's resource remarks, and the other lines."""
    usage, rest, name = [], [], None
    for line in stderr.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" in line:
            text = line.split("remark:", 1)[1].strip()
            if text.startswith("Function Name:"):
                name = text.split(":", 1)[1].split()[0]
            elif text.startswith("ScratchSize") and name:
                usage.append((name, int(text.split(":")[1].split()[0])))
            continue
        rest.append(line)
    # the remark's source excerpt (the kernel's signature line and a caret) follows each remark
    rest = [l for l in rest if not re.match(r"^\s*\d*\s*\|", l)]
    return usage, rest


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{res.stdout}\n{res.stderr}")
    usage, rest = _resource_usage(res.stderr)
    noise = "packed-fp32-ops"
    warn = "\n".join(l for l in rest if noise not in l and l.strip() and "warning generated" not in l)
    if warn:
        sys.stderr.write(f"[{src}]\n{warn}\n")
    spilled = [(n, b) for n, b in usage if b > 0 and any(tag in n for tag in NO_SCRATCH)]
    if spilled:
        raise RuntimeError(f"{src}: kernels that must stay in registers use scratch memory: {spilled}")
    return obj


def build(jobs: int = 8) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(_compile, SOURCES))
    tmp = LIB_PATH + ".tmp"
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
