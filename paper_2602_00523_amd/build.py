"""Build libsage_hip.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2602_00523_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsage_hip.so")

SOURCES = ["entropy_topk.hip", "build_tree.hip", "tree_attention.hip", "tree_attention_f32.hip",
           "tree_attention_bf16.hip", "verify_accept.hip", "commit_history.hip", "lm_head_topk.hip", "fused_steps.hip"]
# packed-fp32 instructions are switched off for every translation unit; the tree rule additionally forbids
# contraction so that its fp32 decisions are reproducible bit for bit.
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wno-unused-command-line-argument",
          # leading scalar kernel arguments arrive in registers at wave launch instead of through a first memory fetch:
          # these kernels are short and launched in dependent chains, where that round trip is a visible share
          "-mllvm", "-amdgpu-kernarg-preload-count=16"]
EXTRA = {"build_tree.hip": ["-ffp-contract=off"]}
# Kernels that keep their own count of vector-memory operations in flight (s_waitcnt vmcnt(N) around LDS-direct loads):
# a register spill adds scratch loads and stores to that counter and silently breaks the count, so these translation
# units are compiled with the resource-usage remarks on and the build fails if any of their kernels uses scratch memory.
NO_SCRATCH = {"tree_attention_bf16.hip": ("tree_attention_bf16_kernel", "tree_attention_plan_kernel"),
              "lm_head_topk.hip": ("lm_head_kernel",)}


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, verbose: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    guarded = NO_SCRATCH.get(src, ())
    remarks = ["-Rpass-analysis=kernel-resource-usage"] if guarded else []
    cmd = [hipcc(), *COMMON, *EXTRA.get(src, []), *remarks, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    lines = [l for l in res.stderr.splitlines() if noise not in l]
    if guarded:
        lines = _check_no_scratch(src, lines, guarded)
    err = "\n".join(lines)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return obj


def _check_no_scratch(src: str, lines: list, kernels: tuple) -> list:
    """Read the resource-usage remarks of one translation unit: raise if a guarded kernel spills to scratch memory;
    return the compiler output without the remarks."""
    rest, name, seen = [], None, set()
    skip = 0
    for l in lines:
        if skip:                                   # the two source-echo lines that follow a remark
            skip -= 1
            continue
        if "-Rpass-analysis=kernel-resource-usage" not in l:
            if "|" in l and l.lstrip()[:1].isdigit() or l.strip().startswith("|"):
                continue
            rest.append(l)
            continue
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in l and name:
            size = int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            for k in kernels:
                if k in name:
                    seen.add(k)
                    if size != 0:
                        raise RuntimeError(f"{src}: kernel {name} uses {size} bytes of scratch per lane (register spills); "
                                           "its counted waits on the vector-memory counter would be wrong")
    missing = [k for k in kernels if k not in seen]
    if missing:
        raise RuntimeError(f"{src}: no resource-usage remark for {missing}: cannot verify the absence of scratch")
    return rest


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(lambda s: _compile(s, verbose), SOURCES))
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
