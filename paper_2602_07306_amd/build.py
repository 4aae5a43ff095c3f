"""Builds libpt.so (the HIP library, gfx950) in-tree with hipcc.

    python -m paper_2602_07306_amd.build [--force]

Object files go to paper_2602_07306_amd/_build/, the library to paper_2602_07306_amd/libpt.so.
"""
from __future__ import annotations

import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpt.so")
CEILINGS_LIB = os.path.join(HERE, "libpt_ceilings.so")   # bench.py --ceilings only
CEILINGS_SOURCES = ["bench_ceilings.hip", "bench_gemm_tiles.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

SOURCES = [
    "pt_api.cpp",
    "kernels_elementwise.hip",
    "kernels_weights.hip",
    "kernels_gemm_generic.hip",
    "kernels_gemm_mfma.hip",
    "kernels_gemm_mfma_store.hip",
    "kernels_gemm_mfma_residual.hip",
    "kernels_gemm_mfma_swiglu.hip",
    "kernels_gemm_mfma_qkv_a.hip",
    "kernels_gemm_mfma_qkv_b.hip",
    "kernels_gemm_mfma_qkv_c.hip",
    "kernels_gemm_mfma_qkv_d.hip",
    "kernels_gemm_skinny.hip",
    "kernels_attn_generic.hip",
    "kernels_attn_prefill_mfma.hip",
    "kernels_attn_decode.hip",
    "kernels_moe.hip",
]

COMMON = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-x", "hip", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wno-unused-command-line-argument",
]
PER_FILE = {
    # the weight generator must not contract a*b+c into a fused multiply-add
    "kernels_weights.hip": ["-ffp-contract=off"],
}


def _headers_mtime() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(ROOT, "include", "pt.h"))
    return max(os.path.getmtime(h) for h in hs)


def resources_path(src: str) -> str:
    """Where the compiler's per-kernel resource report of a source file is kept (tests read it)."""
    return os.path.join(BUILD, os.path.splitext(src)[0] + ".resources.json")


def _kernel_resources(remarks: str) -> dict:
    """{mangled kernel name: {"VGPRs", "AGPRs", "ScratchSize", "VGPRs Spill", "Occupancy", ...}} from the remarks of
    -Rpass-analysis=kernel-resource-usage."""
    out, cur = {}, None
    for line in remarks.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\S+) \[-Rpass", line)
        if m and cur is not None:
            v = m.group(2)
            cur[m.group(1).strip()] = int(v) if v.isdigit() else v
    return out


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    is_kernel_source = src.endswith(".hip")
    if (not force and os.path.exists(obj) and (not is_kernel_source or os.path.exists(resources_path(src)))
            and os.path.getmtime(obj) > max(os.path.getmtime(path), _headers_mtime())):
        return obj
    cmd = [HIPCC] + COMMON + PER_FILE.get(src, []) + ["-Rpass-analysis=kernel-resource-usage", "-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    if is_kernel_source:
        with open(resources_path(src), "w") as f:
            json.dump(_kernel_resources(r.stderr), f, indent=1, sort_keys=True)
    return obj


def build(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        all_objs = list(ex.map(lambda s: _compile(s, force), SOURCES + CEILINGS_SOURCES))
    objs, cobjs = all_objs[:len(SOURCES)], all_objs[len(SOURCES):]
    for lib, olist, extra in ((LIB, objs, ["-Wl,--version-script=" + os.path.join(CSRC, "libpt.map")]),
                              (CEILINGS_LIB, cobjs, [])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + extra + ["-o", lib] + olist
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
