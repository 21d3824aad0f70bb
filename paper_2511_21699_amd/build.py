"""Build libcacheback_verify.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import glob
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcacheback_verify.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # every atomic here is issued by one thread; the wave-aggregation pass would only add a
         # wait for the result right behind the atomic, where the kernels want it in flight
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    subprocess.run(["hipcc", *FLAGS, "-c", src, "-o", obj], check=True)
    return obj


def device_asm(src: str) -> str:
    """The gfx950 assembly hipcc makes of one source file, with the library's flags."""
    os.makedirs(OBJ, exist_ok=True)
    out = os.path.join(OBJ, os.path.basename(src) + ".s")
    flags = [f for f in FLAGS if f not in ("-fPIC",)]
    subprocess.run(["hipcc", *flags, "-S", "--offload-device-only", src, "-o", out], check=True,
                   stderr=subprocess.DEVNULL)
    with open(out) as f:
        return f.read()


_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def untracked_load_violations(asm: str) -> list:
    """The attention kernel issues some loads as inline assembly the compiler does not know to be
    loads, and waits for them itself before their first use.  That is only right while the compiler
    leaves the destination registers alone in between (a copy or a spill would read them before
    the data is there).  For every such load (a global_load_dwordx4 inside an inline-assembly
    block) this walks down the listing to the first instruction that names one of its registers
    and reports the load if no vmcnt wait and no branch (where the walk cannot follow) came
    before it.  Returns a list of (line number, text) pairs, empty if all is well."""
    lines = asm.split("\n")
    bad = []
    in_asm = False
    for i, line in enumerate(lines):
        if "ASMSTART" in line:
            in_asm = True
            continue
        if "ASMEND" in line:
            in_asm = False
            continue
        # (every register-returning load spelling: the query rows' and the logits item's 16-byte loads today)
        m = re.search(r"(?:global|buffer|flat)_load_dword(?:x[234])? v\[(\d+):(\d+)\]", line) if in_asm else None
        if not m:
            continue
        lo, hi = int(m.group(1)), int(m.group(2))
        covered = False
        for j in range(i + 1, len(lines)):
            code = lines[j].split(";")[0]
            if "s_waitcnt vmcnt" in code or re.search(r"\bs_(c?branch|endpgm)", code):
                covered = True
                break
            touched = False
            for r in _REG.finditer(code):
                a, b = (int(r.group(1)), int(r.group(2))) if r.group(1) else (int(r.group(3)),) * 2
                touched |= a <= hi and b >= lo
            if touched:
                break
        if not covered:
            bad.append((i + 1, line.strip()))
    return bad


def kernel_resources(asm: str) -> dict:
    """{kernel symbol: (vgpr_count, vgpr_spill_count, private_segment_fixed_size)} from the listing's metadata."""
    out, name, cur = {}, None, {}
    for line in asm.split("\n"):
        m = re.match(r"\s*(?:- )?\.(name|vgpr_count|vgpr_spill_count|private_segment_fixed_size):\s*(\S+)", line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "name":
            name = val
        else:
            cur[key] = int(val)
        if name and len(cur) == 3:
            out[name] = (cur["vgpr_count"], cur["vgpr_spill_count"], cur["private_segment_fixed_size"])
            name, cur = None, {}
    return out


def scratch_violations(asm: str) -> list:
    """Kernels of the listing that spill registers or use scratch memory.  In the attention kernel a spill
    reload inside the K/V ring phase would be a compiler-generated load, and with it a wait for every load in
    flight, in a loop whose waits are counted by hand."""
    return [(k, v) for k, v in kernel_resources(asm).items() if v[1] != 0 or v[2] != 0]


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    asm = device_asm(os.path.join(CSRC, "cb_attn_mfma.hip"))
    bad = untracked_load_violations(asm)
    if bad:
        raise RuntimeError(f"cb_attn_mfma.hip: registers of untracked loads are touched before their wait: {bad[:4]}")
    bad = scratch_violations(asm)
    if bad:
        raise RuntimeError(f"cb_attn_mfma.hip: kernels that spill or use scratch memory: {bad[:4]}")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print(LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
