"""Builds the HIP library in-tree (gfx950 only): paper_2311_12023_amd/liblq_hip.so, the product, and
liblq_hip_testing.so, the same sources compiled with -DLQ_TESTING_HOOKS plus csrc/lq_testing_hooks.cpp (the entry
points of include/lq_testing.h, which only the test-suite loads)."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblq_hip.so")
TEST_LIB = os.path.join(HERE, "liblq_hip_testing.so")
HOOKS = "lq_testing_hooks.cpp"
# sources whose code differs in the testing build (they contain #ifdef LQ_TESTING_HOOKS sections)
HOOKED = ("lq_api_decomp.cpp",)

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result",
         "-Wno-inline-asm"]   # the direct-to-LDS loads set M0 in inline assembly and say so in their clobber list


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.cpp")) + glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False) -> str:
    """Compiles every source under csrc/ with hipcc and links the two shared libraries."""
    objs, test_objs, procs = [], [], []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)

    def compile_one(src, obj, extra=()):
        cmd = ["hipcc", "-x", "hip"] + [f for f in FLAGS if f != "-shared"] + list(extra) + ["-c", src, "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))

    for src in sources():
        base = os.path.basename(src)
        obj = os.path.join(HERE, "_build", base + ".o")
        if base == HOOKS:
            compile_one(src, obj, ["-DLQ_TESTING_HOOKS"])
            test_objs.append(obj)
            continue
        compile_one(src, obj)
        objs.append(obj)
        if base in HOOKED:
            tobj = os.path.join(HERE, "_build", base + ".testing.o")
            compile_one(src, tobj, ["-DLQ_TESTING_HOOKS"])
            test_objs.append(tobj)
        else:
            test_objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], check=True)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + test_objs + ["-o", TEST_LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
