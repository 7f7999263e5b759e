"""Build libround_attention.so (HIP, gfx950 only) in-tree with hipcc.

Usage: python -m paper_2502_15294_amd.build [--force]
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libround_attention.so")
EXAMPLE_SRC = os.path.join(HERE, "examples", "decode_step.c")
EXAMPLE = os.path.join(HERE, "ra_decode_step")  # plain C program driving the library through the C boundary alone
SOURCES = ["context.hip", "decode.hip", "attn_mfma.hip", "attn_prefill_mfma.hip", "scores.hip", "scores_mfma.hip", "scores_prefill_mfma.hip", "select.hip", "prefill.hip", "kv_store.hip", "monitor.hip"]
# packed-fp32 instruction selection is switched off for every device translation unit
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr[-4000:]}")
    return obj


def build(force: bool = True, jobs: int = 6) -> str:
    """Compile every translation unit and link the shared library.  Always recompiles when
    `force` is set; otherwise only when a source or header is newer than the library."""
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "round_attention.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(d) <= os.path.getmtime(LIB) for d in deps):
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr[-4000:]}")
    build_example()
    return LIB


def build_example() -> str:
    """The C example, compiled as C11 by the host C compiler (it includes round_attention.h as C)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.environ.get("CC", "gcc"), "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"), EXAMPLE_SRC, "-o", EXAMPLE,
           "-L", HERE, "-lround_attention", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"C example failed to build:\n{r.stderr[-4000:]}")
    return EXAMPLE


# ---- the same sources under other instruction schedules ------------------------------------------------------
# Results must not depend on how the compiler orders instructions.  A wait state the hardware leaves to software
# and the source forgets (an instruction hidden from the compiler, a missing barrier) shows up as outputs that differ
# in their last bits between builds that differ only in the scheduling strategy, so the GPU tests compare such
# builds with the product build bit by bit (tests/test_gpu_schedule_independence.py).  They are optional: built by
# `python -m paper_2502_15294_amd.build --alt-schedules`, skipped by the test when absent or stale.
ALT_STRATEGIES = ("iterative-ilp", "iterative-minreg")
ALT_DIR = os.path.join(HERE, "_alt")


def sources_digest() -> str:
    """sha1 over the kernel sources and the boundary header: names a build's inputs."""
    import hashlib
    h = hashlib.sha1()
    for path in sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC)) + [os.path.join(ROOT, "include", "round_attention.h")]:
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()


def alt_library(strategy: str) -> str:
    return os.path.join(ALT_DIR, f"libround_attention.{strategy}.so")


def build_alt_schedules(jobs: int = 6) -> list:
    """The whole library once per strategy in ALT_STRATEGIES, each with a stamp file holding sources_digest()."""
    libs = []
    for strategy in ALT_STRATEGIES:
        obj_dir = os.path.join(OBJ, "alt_" + strategy)
        os.makedirs(obj_dir, exist_ok=True)
        os.makedirs(ALT_DIR, exist_ok=True)

        def compile_one(src, obj_dir=obj_dir, strategy=strategy):
            obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
            cmd = [_hipcc(), *FLAGS, "-mllvm", f"-amdgpu-sched-strategy={strategy}", "-c", os.path.join(CSRC, src), "-o", obj]
            r = subprocess.run(cmd, capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc ({strategy}) failed on {src}:\n{r.stderr[-4000:]}")
            return obj

        with ThreadPoolExecutor(max_workers=jobs) as ex:
            objs = list(ex.map(compile_one, SOURCES))
        lib = alt_library(strategy)
        r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link ({strategy}) failed:\n{r.stderr[-4000:]}")
        with open(lib + ".stamp", "w") as f:
            f.write(sources_digest())
        libs.append(lib)
    return libs


if __name__ == "__main__":
    print(build(force=True))
    if "--alt-schedules" in sys.argv:
        for lib in build_alt_schedules():
            print(lib)
