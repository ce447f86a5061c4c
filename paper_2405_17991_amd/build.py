"""Build libvelora.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2405_17991_amd.build [--force]

hipcc cross-compiles for gfx950 without a GPU.  The shared library lands next
to this file so that it travels with the source tree.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys
from typing import List

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libvelora.so")
SOURCES = ["api.hip", "compress.hip", "init_v.hip", "wgrad.hip", "adamw.hip", "swiglu.hip", "rmsnorm.hip", "linear.hip", "probe.hip"]
HEADERS = [os.path.join(CSRC, "common.h"), os.path.join(CSRC, "kernels.h"),
           os.path.join(os.path.dirname(HERE), "include", "velora.h")]

HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _stale(target: str, deps: List[str]) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


# Kernels whose loops count outstanding vector-memory operations by hand (s_waitcnt vmcnt(n)): a register
# spill inside them would add scratch loads and stores to that count, which makes every wait cover more
# than it needs and serialises the load streams, so the build fails if the compiler reports any spill or
# scratch use for them.
NO_SPILL = {"linear.hip": "linear_mfma_kernel", "wgrad.hip": "wgrad_partial_ws"}


def _check_no_spill(src: str, remarks: str) -> None:
    name, bad = None, []
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif name and NO_SPILL[src] in name:
            for key in ("VGPRs Spill:", "SGPRs Spill:", "ScratchSize [bytes/lane]:"):
                if key in line and int(line.split(key)[1].split()[0]) != 0:
                    bad.append(f"{name}: {key} {line.split(key)[1].split()[0]}")
    if bad:
        raise RuntimeError(f"{src}: kernels with hand-counted waits are built without spills:\n" + "\n".join(bad))


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if force or _stale(obj, [path] + HEADERS):
        cmd = [HIPCC] + FLAGS + ["-c", path, "-o", obj]
        if src in NO_SPILL:
            cmd.append("-Rpass-analysis=kernel-resource-usage")
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if src in NO_SPILL and r.returncode == 0:
            _check_no_spill(src, r.stdout)
        kept, skip = [], 0
        for l in r.stdout.splitlines():        # drop the resource remarks with their two source-context lines
            if "-Rpass-analysis=kernel-resource-usage" in l:
                skip = 2
            elif skip:
                skip -= 1
            elif "packed-fp32-ops" not in l:
                kept.append(l)
        out = "\n".join(kept)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{out}")
        if out.strip():
            print(out, file=sys.stderr)
    return obj


def build(force: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or _stale(LIB_PATH, objs):
        cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB_PATH] + objs
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}")
    return LIB_PATH


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
