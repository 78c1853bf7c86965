"""Builds the HIP library in-tree: paper_2411_11217_amd/libmoe_hip.so (gfx950)."""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoe_hip.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-pthread", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# Kernels whose inline assembly owns the accumulator registers a0 .. a255 by NAME (the MFMA accumulators of the expert
# GEMMs).  The register allocator does not know that they are taken: when it runs out of vector registers it parks
# values in accumulator registers, where the kernel's MFMAs then overwrite them (seen once, in an experimental variant
# of the kernel: a pointer came back as accumulator bits and the kernel faulted).  The kernels are written so that it
# has no need to; this check of the assembly the compiler generates makes a build fail if it ever does, or if such a
# kernel spills to scratch memory.  The kernels' own uses print as a[N] or a[N:M], the allocator's as aN.
ACCUMULATOR_OWNERS = {"moe_ffn_bf16.hip"}


def check_kernel_assembly(asm_path: str) -> None:
    found = []
    in_kernel = False
    with open(asm_path) as f:
        for line in f:
            code = line.split(";")[0]
            if re.match(r"^_Z\w*ffn_gemm_bf16\w*:", code):
                in_kernel = True
            elif code.startswith(".Lfunc_end"):
                in_kernel = False
            if not in_kernel:
                m = re.match(r"^\s+\.amdhsa_private_segment_fixed_size\s+(\d+)", code)
                if m and int(m.group(1)) != 0:
                    found.append("a kernel of this file spills to scratch memory (%s bytes)" % m.group(1))
            elif not code.lstrip().startswith(".") and re.search(r"(?<![\w\[])a\d+\b", code):
                found.append("accumulator register used by the compiler: " + code.strip())
    if found:
        raise RuntimeError("%s:\n  %s" % (asm_path, "\n  ".join(found[:10])))


def sources():
    """The .hip files (device code, compiled by hipcc) and the .cpp files (host only, compiled by the host compiler)."""
    return sorted(glob.glob(os.path.join(CSRC, "*.hip"))) + sorted(glob.glob(os.path.join(CSRC, "*.cpp")))


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(ROOT, "include", "moe.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    """Compile every .hip file and link the shared library.  Returns its path.

    ``extra_flags`` / ``out`` build an experimental variant next to the default library."""
    if not force and not is_stale():
        return LIB
    build_dir = BUILD if out == LIB else os.path.join(os.path.dirname(os.path.abspath(out)), "_build_" + os.path.basename(out).replace(".", "_"))
    os.makedirs(build_dir, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "hipcc")

    def compile_one(src):
        obj = os.path.join(build_dir, os.path.basename(src)[:-4] + ".o")
        checked = os.path.basename(src) in ACCUMULATOR_OWNERS
        if src.endswith(".cpp"):
            cmd = [os.environ.get("CXX", "g++")] + HOST_FLAGS + ["-c", src, "-o", obj]
        else:
            cmd = [hipcc] + FLAGS + list(extra_flags) + (["-save-temps=obj"] if checked else []) + ["-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True, cwd=build_dir)
        if r.returncode != 0:
            raise RuntimeError("compiler failed for %s:\n%s" % (src, r.stderr[-8000:]))
        if checked:
            check_kernel_assembly(os.path.join(build_dir, os.path.basename(src)[:-4] + "-hip-amdgcn-amd-amdhsa-gfx950.s"))
        if verbose and r.stderr.strip():
            sys.stderr.write(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(sources())))) as pool:
        objs = list(pool.map(compile_one, sources()))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr[-8000:])
    return out


if __name__ == "__main__":
    flags = [a for a in sys.argv[1:] if a.startswith("-D")]
    outs = [a for a in sys.argv[1:] if a.endswith(".so")]
    print(build(force=True, verbose="-v" in sys.argv, extra_flags=flags, out=outs[0] if outs else LIB))
