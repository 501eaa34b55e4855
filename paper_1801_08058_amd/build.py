"""Builds libngconv.so (gfx950 only) from csrc/ with hipcc.  In-tree, no JIT cache."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libngconv.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "layout.hip", "conv_direct.hip", "conv_igemm.hip", "conv_strip.hip", "conv_rows.hip", "conv_strip3.hip", "conv_stem.hip", "wgrad.hip", "wgrad_strip.hip", "wgrad_stem.hip", "wgrad_gemm.hip", "conv_gemm1x1.hip", "bias_grad.hip", "softmax.hip", "conv3d_direct.hip", "api3d.hip", "static_scratch.hip", "switches.hip", "bwd1x1_fused.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the compiler's per-kernel resource report: kept out of the output, except that a kernel which uses scratch
    # memory (a register array that was not promoted, or spilled registers) is named - none of them should
    err_lines, held, kernel, in_remark = [], [], "?", False
    for l in r.stderr.splitlines():
        if "packed-fp32-ops" in l:
            continue
        if l.startswith("In file included from"):
            held.append(l)                        # belongs to the diagnostic that follows
            continue
        if in_remark and (l.split("|")[0].strip().isdigit() or l.lstrip().startswith("|")):
            continue                              # the source line and caret printed under a remark
        in_remark = "-Rpass-analysis=kernel-resource-usage" in l
        if in_remark:
            held = []
            if "Function Name:" in l:
                kernel = l.split("Function Name:")[1].split("[-Rpass")[0].strip()
            elif "ScratchSize [bytes/lane]:" in l:
                n = int(l.split("ScratchSize [bytes/lane]:")[1].split()[0])
                if n:
                    err_lines.append(f"warning: {src}: kernel {kernel} uses {n} bytes of scratch memory per lane")
            continue
        err_lines += held + [l]
        held = []
    err = "\n".join(err_lines)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link libngconv.so next to this file."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
