"""Builds libsol_mi355.so (the HIP library behind the C ABI in include/sol.h) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsol_mi355.so")
SOURCES = ["conv_igemm.hip", "conv_dma.hip", "conv_halo.hip", "conv_gemm8.hip", "conv_stem.hip", "conv_pair.hip", "conv_block.hip", "conv_xr.hip", "fusion.hip", "dwconv.hip", "linear.hip", "train.hip", "probe.hip", "api.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage"]
RESOURCES = os.path.join(HERE, "kernel_resources.json")     # per kernel: VGPRs, scratch bytes per lane, LDS bytes (written by build())


def _compile(src: str):
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    lines = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l]
    # the compiler's per-kernel resource remarks (device pass): registers, scratch (spill) bytes per lane, LDS
    res, cur, rest = {}, None, []
    for l in lines:
        if "-Rpass-analysis=kernel-resource-usage" in l:
            body = l.split("remark:", 1)[1].replace("[-Rpass-analysis=kernel-resource-usage]", "").strip()
            if body.startswith("Function Name:"):
                cur = res.setdefault(body.split(":", 1)[1].strip(), {"source": src})
            elif cur is not None and ":" in body:
                k, v = body.rsplit(":", 1)
                key = {"VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch_bytes_per_lane",
                       "LDS Size [bytes/block]": "lds_bytes", "Occupancy [waves/SIMD]": "waves_per_simd"}.get(k.strip())
                if key:
                    cur[key] = int(v)
        elif not l.lstrip().startswith(("|", "^")) and "remark" not in l and "__global__" not in l:
            rest.append(l)
    err = "\n".join(rest)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n" + "\n".join(lines))
    if err.strip():
        print(err, file=sys.stderr)
    return obj, res


def build(verbose: bool = True) -> str:
    import json

    with ThreadPoolExecutor(max_workers=4) as ex:
        done = list(ex.map(_compile, SOURCES))
    objs = [o for o, _ in done]
    resources = {}
    for _, res in done:
        resources.update(res)
    with open(RESOURCES, "w") as f:
        json.dump(resources, f, indent=0, sort_keys=True)
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
