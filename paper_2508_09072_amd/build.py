"""Build libreader_hip.so for gfx950 with hipcc (no torch involved).

    python -m paper_2508_09072_amd.build

The library is written in-tree next to this file so that it travels with the
source tree; it is not installed anywhere else.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libreader_hip.so")
# the same library with per-workgroup time stamps in the 128-row attention kernel (python -m ...build --stamps;
# used by wg_timeline.py only)
STAMPS_LIB = os.path.join(HERE, "libreader_hip_stamps.so")
SOURCES = ["reader_api.hip", "trie_drafter.cpp", "tree_shape.cpp", "accept_compact.hip", "kv_compact_layers.hip", "kv_rearrange.hip", "target_argmax.hip", "target_sample.hip", "tree_attn_scalar.hip", "tree_attn_mfma.hip", "tree_attn_wide.hip", "peak_probes.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall",
    # the LDS-copy inline asm names m0 as clobbered on purpose
    "-Wno-inline-asm",
    # the wide attention kernel manages the accumulation registers by hand: the compiler must not park values there
    "-mllvm", "-amdgpu-spill-vgpr-to-agpr=0",
    # per-kernel register and scratch usage as compiler remarks: checked below
    "-Rpass-analysis=kernel-resource-usage",
]


def spilled_kernels(compiler_output: str):
    """(kernel, spilled VGPRs, scratch bytes per lane) for every kernel the compiler had to spill vector
    registers to memory in.

    The attention kernels are written against the register file (256 registers per lane with two
    wavefronts per SIMD, 512 with one): a change that makes them spill to scratch memory costs a
    factor of two and shows in no test, so the build refuses it.  (Values parked in the other
    half of the register file do not count: they use no memory.)"""
    import re
    found, name, scratch = [], None, 0
    for line in compiler_output.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name, scratch = m.group(1), 0
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m:
            scratch = int(m.group(1))
        m = re.search(r"VGPRs? Spill: (\d+)", line)
        if m and name and int(m.group(1)) > 0 and scratch > 0:
            found.append((name, int(m.group(1)), scratch))
    return found


def foreign_agpr_uses(asm_text: str):
    """Lines of compiler-generated code (outside inline-asm blocks) that touch an accumulation register.

    tree_attn_wide.hip keeps its output accumulators and query fragments in accumulation registers it names
    by number in inline asm; the register allocator does not know that, so it must never put anything
    there itself (a value parked in one would be overwritten, and an overwritten address faults the GPU)."""
    import re
    bad, inside = [], False
    for line in asm_text.splitlines():
        if "#ASMSTART" in line:
            inside = True
        elif "#ASMEND" in line:
            inside = False
        elif not inside and not line.lstrip().startswith((";", ".")) and re.search(r"(^|[\s,\[])a(\d+|\[\d+:\d+\])", line):
            bad.append(line.strip())
    return bad


def check_wide_kernel(hipcc: str, verbose: bool) -> None:
    cmd = [hipcc] + [f for f in FLAGS if f not in ("-fPIC", "-shared", "-Rpass-analysis=kernel-resource-usage")]
    cmd += ["--cuda-device-only", "-S", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
            os.path.join(CSRC, "tree_attn_wide.hip"), "-o", "-"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc -S of tree_attn_wide.hip failed")
    bad = foreign_agpr_uses(res.stdout)
    if bad:
        raise RuntimeError("the compiler uses accumulation registers of its own in tree_attn_wide.hip: %s" % bad[:5])
    if verbose:
        print("tree_attn_wide.hip: accumulation registers are touched by hand-written instructions only")


def build(verbose: bool = False, stamps: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    lib = STAMPS_LIB if stamps else LIB
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + FLAGS + (["-DREADER_WG_STAMPS"] if stamps else []) + ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    spilled = spilled_kernels(res.stdout)
    kept, after_remark = [], False
    for l in res.stdout.splitlines():
        if "remark:" in l:
            after_remark = True
            continue
        if after_remark and l.lstrip()[:1] in "|0123456789":    # the source line and the caret under a remark
            continue
        after_remark = False
        if "not a recognized feature" not in l:
            kept.append(l)
    out = "\n".join(kept)
    if res.returncode != 0 or spilled:
        if os.path.exists(tmp):
            os.remove(tmp)
        if spilled:
            raise RuntimeError("kernels spill vector registers: %s" % spilled)
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    try:
        check_wide_kernel(hipcc, verbose)
    except Exception:
        os.remove(tmp)
        raise
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, stamps="--stamps" in sys.argv))
