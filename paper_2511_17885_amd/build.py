"""Compile the HIP library (csrc/*.hip) for gfx950 into paper_2511_17885_amd/libfmoe.so.

hipcc cross-compiles without a GPU.  Packed-fp32 instruction selection is disabled for all
device code; the router and pruning kernels are additionally built with floating-point
contraction off because their operation order is part of their contract.
"""
import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
OUT = os.path.join(HERE, "libfmoe.so")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-fast-math",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]
SOURCES = {
    "api.hip": [],
    "route.hip": ["-ffp-contract=off"],
    "prune.hip": ["-ffp-contract=off"],
    "permute.hip": [],
    "ffn.hip": [],
    "combine.hip": [],
    "diag.hip": [],
    "stack.hip": [],
    "noalloc.hip": [],
}


def check_accumulation_registers(asm_path):
    """The dense-shape expert GEMM kernels (ffn_dense_kernel) keep their accumulators in accumulation
    registers that the kernel names itself, which the compiler's register allocator does not see.  This
    reads the device assembly the compiler wrote for ffn.hip and fails if, inside those kernels, the
    compiler placed anything of its own in an accumulation register (any a<N> operand outside the
    kernel's own inline-assembly blocks)."""
    import re
    inside = in_asm = False
    kernels = 0
    for n, line in enumerate(open(asm_path), 1):
        if re.match(r"^_ZN\S*ffn_dense_kernel\S*:", line):
            inside, in_asm = True, False
            kernels += 1
            name = line.split(":")[0]
            continue
        if not inside:
            continue
        if line.startswith(".Lfunc_end"):   # not s_endpgm: a kernel has one per early exit
            inside = False
        elif "ASMSTART" in line:
            in_asm = True
        elif "ASMEND" in line:
            in_asm = False
        elif not in_asm and re.search(r"\ba\[?\d", line.split(";")[0]):
            raise RuntimeError(f"{asm_path}:{n}: the compiler uses an accumulation register inside {name}, which "
                               f"keeps hand-placed accumulators there: {line.strip()}")
    if kernels == 0:
        raise RuntimeError(f"{asm_path}: no ffn_dense_kernel found to check")
    return kernels


def _compile(name, extra, verbose):
    src = os.path.join(CSRC, name)
    obj = os.path.join(OBJ, name.replace(".hip", ".o"))
    cmd = ["hipcc", "-c", src, "-o", obj] + COMMON + extra
    if name == "ffn.hip":
        cmd.append("-save-temps=obj")   # keeps the device assembly beside the object, for the check below
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature; that is expected
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {name}:\n{err}")
    if err.strip() and verbose:
        print(err, flush=True)
    if name == "ffn.hip":
        check_accumulation_registers(os.path.join(OBJ, "ffn-hip-amdgcn-amd-amdhsa-gfx950.s"))
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(lambda kv: _compile(kv[0], kv[1], verbose), SOURCES.items()))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", OUT] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
