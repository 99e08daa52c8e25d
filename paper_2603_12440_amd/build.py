"""Builds libmi355gemm.so (HIP, gfx950 only) next to this file with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmi355gemm.so")
SOURCES = [os.path.join(CSRC, f) for f in
           ("gemm_api.hip", "mfma_bf16_inst.hip", "mfma_f16_inst.hip", "mfma_f8_inst.hip",
            "mfma16_bf16_inst.hip", "mfma16_f16_inst.hip", "mfma16p_bf16_inst.hip", "mfma16p_f16_inst.hip", "rope_api.hip", "probe_api.hip")]
OBJ_DIR = os.path.join(os.path.dirname(HERE), "_build")


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the GEMM library cannot be built")


def sources_newer_than_lib() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "gemm.h"))
    deps.append(os.path.join(os.path.dirname(HERE), "include", "rope.h"))
    deps.append(os.path.join(os.path.dirname(HERE), "include", "probe.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(verbose: bool = False, only: tuple = ()) -> str:
    """Compile every kernel instantiation for gfx950 (one object per translation unit, side by
    side) and link them into one shared library.  `only`: source file names to recompile (the
    other objects are taken as they are; for development, when a change touches one unit)."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OBJ_DIR, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             # packed-fp32 VALU forms stay off
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-function", "-Rpass-analysis=kernel-resource-usage",
             # keep the generated device assembly next to the object: it is scanned below
             "-save-temps=obj"]
    noise = ("is not a recognized feature for this target", "-Rpass-analysis=kernel-resource-usage")

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        if only and os.path.basename(src) not in only and os.path.exists(obj):
            return src, obj, subprocess.CompletedProcess([], 0, "", "")
        res = subprocess.run([_hipcc()] + flags + ["-c", src, "-o", obj], capture_output=True, text=True)
        return src, obj, res

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        results = list(pool.map(compile_one, SOURCES))
    objs, remarks = [], []
    for src, obj, res in results:
        err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {os.path.basename(src)}:\n" + err)
        if verbose and err.strip():
            print(err)
        objs.append(obj)
        remarks.append(res.stderr)
    bad = kernels_with_scratch("\n".join(remarks))
    if bad:
        if os.path.exists(LIB):
            os.remove(LIB)
        raise RuntimeError("kernels that keep data in scratch memory (the hand-scheduled kernels place their own "
                           "waits for asynchronous LDS reads and matrix-core results; a register the compiler "
                           "moves to memory in between breaks that):\n  " + "\n  ".join(bad))
    hazards = []
    for src in SOURCES:
        asm = os.path.join(OBJ_DIR, os.path.splitext(os.path.basename(src))[0] + "-hip-amdgcn-amd-amdhsa-gfx950.s")
        if os.path.exists(asm):
            with open(asm) as f:
                hazards += [f"{os.path.basename(asm)}:{h}" for h in lds_load_hazards(f.read())]
    if hazards:
        if os.path.exists(LIB):
            os.remove(LIB)
        raise RuntimeError("a direct-to-LDS load reads a scalar register fewer than 5 wait states after a vector-ALU "
                           "instruction wrote it:\n  " + "\n  ".join(hazards[:20]))
    res = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC",
                          "-Wl,--version-script=" + os.path.join(CSRC, "exports.map"), "-o", LIB] + objs,
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("linking failed:\n" + res.stderr)
    return LIB


def lds_load_hazards(asm: str) -> list:
    """Lines of generated assembly where a `global_load_lds_*` takes its scalar base address from a register
    that a `v_readlane` / `v_readfirstlane` wrote fewer than 5 wait states earlier.  The kernels issue these
    loads from inline assembly, which the compiler's hazard recogniser does not see into; a vector-memory
    instruction may not read a scalar register that soon after a vector-ALU write of it."""
    import re
    lines = [l.strip() for l in asm.splitlines()]
    ins = [(i, l) for i, l in enumerate(lines)
           if l and not l.startswith((";", ".", "//")) and not l.endswith(":")]
    bad = []
    for k, (i, l) in enumerate(ins):
        if not l.startswith("global_load_lds"):
            continue
        m = re.search(r"s\[(\d+):(\d+)\]", l)
        if not m:
            continue
        regs = {int(m.group(1)), int(m.group(2))}
        dist = 0
        for kk in range(k - 1, max(k - 12, -1), -1):
            prev = ins[kk][1]
            w = re.match(r"v_read(?:first)?lane_b32\s+s(\d+)", prev)
            if w and int(w.group(1)) in regs and dist < 5:
                bad.append(f"{i + 1}: {l}   (after line {ins[kk][0] + 1}: {prev})")
            n = re.match(r"s_nop\s+(\d+)", prev)
            dist += (int(n.group(1)) + 1) if n else 1
            if dist >= 5:
                break
    return bad


def kernels_with_scratch(remarks: str) -> list:
    """Names of kernels whose resource-usage remarks show scratch memory or vector-register spills
    (scalar registers spilled into vector-register lanes stay in registers and are fine)."""
    bad, name = [], None
    for line in remarks.splitlines():
        if "remark:" not in line:
            continue
        text = line.split("remark:", 1)[1].strip()
        if text.startswith("Function Name:"):
            name = text.split(":", 1)[1].split("[")[0].strip()
        elif name and text.split(":")[0] in ("ScratchSize [bytes/lane]", "VGPRs Spill"):
            if int(text.split(":")[1].split("[")[0]) != 0 and name not in bad:
                bad.append(name)
    return bad


if __name__ == "__main__":
    print(build_library(verbose=True))
