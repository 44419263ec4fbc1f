"""Compile the HIP sources in csrc/ for gfx950 into paper_2501_05408_amd/lib/libtempo.so.

Run as `python -m paper_2501_05408_amd.build` (always recompiles) or call
build(force=False) to compile only when a source is newer than the library.
hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIBDIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIBDIR, "libtempo.so")
OBJDIR = os.path.join(HERE, "_build")

SOURCES = ["tempo_api.hip", "kv_store.hip", "attn_partial_bf16.hip", "attn_partial_f32.hip",
           "attn_combine.hip", "stream_read.hip", "rope.hip", "attn_prefill_bf16.hip", "worklist.hip", "discounted_sum.hip"]
HEADERS = [os.path.join(CSRC, "tempo_internal.h"), os.path.join(CSRC, "attn_bf16_common.h"),
           os.path.join(CSRC, "attn_combine.h"), os.path.join(ROOT, "include", "tempo.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Rpass-analysis=kernel-resource-usage",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _stale() -> bool:
    if not os.path.exists(LIB):
        return True
    lib_m = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > lib_m for d in deps)


def _drop_remarks(lines):
    """Remove the resource-usage remarks (and their source excerpts) from hipcc's stderr."""
    out, skip = [], 0
    for l in lines:
        if "[-Rpass-analysis=kernel-resource-usage]" in l:
            skip = 2 if "Function Name" in l else 0   # the excerpt and caret lines follow the first remark
            continue
        if skip and (re.match(r"\s*\d+ \| ", l) or re.match(r"\s*\|\s*\^", l)):
            skip -= 1
            continue
        skip = 0
        out.append(l)
    return out


# Kernels whose speed depends on how many wavefronts fit a SIMD: (mangled-name
# fragment, minimum "Occupancy [waves/SIMD]").  A source change that pushes the
# register count over the edge fails the build instead of silently costing 30%.
MIN_OCCUPANCY = [
    ("attn_partial_bf16ILi128E", 3),           # decode kernel, D = 128: <= 170 VGPRs
    ("attn_prefill_bf16ILi128ELi8ELb", 4),   # prompt kernel, D = 128: two workgroups of 8 per compute unit
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    lines = [l for l in r.stderr.splitlines() if noise not in l]
    # Resource remarks: a kernel that falls back to scratch memory (a register array
    # the compiler could not keep in registers) is several times slower; refuse it.
    kernel, spilled, crowded = None, [], []
    for l in lines:
        m = re.search(r"remark: Function Name: (\S+)", l)
        if m:
            kernel = m.group(1)
        m = re.search(r"remark:\s+ScratchSize \[bytes/lane\]: (\d+)", l)
        if m and int(m.group(1)) > 0:
            spilled.append(f"{kernel}: {m.group(1)} bytes/lane of scratch")
        m = re.search(r"remark:\s+Occupancy \[waves/SIMD\]: (\d+)", l)
        if m:
            for frag, need in MIN_OCCUPANCY:
                if frag in kernel and int(m.group(1)) < need:
                    crowded.append(f"{kernel}: occupancy {m.group(1)} waves/SIMD, needs {need}")
    err = "\n".join(_drop_remarks(lines))
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if spilled:
        raise RuntimeError(f"{src}: kernels must not use scratch memory:\n  " + "\n  ".join(spilled))
    if crowded:
        raise RuntimeError(f"{src}: register use went over an occupancy edge:\n  " + "\n  ".join(crowded))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force: bool = True) -> str:
    """Compile every HIP source and link libtempo.so; returns the library path."""
    if not force and not _stale():
        return LIB
    os.makedirs(OBJDIR, exist_ok=True)
    os.makedirs(LIBDIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
