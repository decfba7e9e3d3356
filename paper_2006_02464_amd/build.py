"""Builds libclockwork_exec.so for gfx950 with hipcc, in-tree.

``python -m paper_2006_02464_amd.build`` compiles unconditionally; the binding
loads what is built and only calls :func:`build` when nothing is.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libclockwork_exec.so")
SOURCES = ["clockwork_exec.hip", "plan.cpp", "kernels_conv.hip", "kernels_conv_dlds.hip", "kernels_resident.hip", "kernels_misc.hip", "worker.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fno-gpu-rdc",
    # never let the compiler form packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-result",
]
# The direct-to-LDS convolution kernel takes its hottest arguments as leading scalars, the small
# kernels all of theirs; with this option the hardware has them in SGPRs when a wave starts (at most
# 14 dwords: every user SGPR beside the argument pointer).  The compiler keeps a prologue that loads them the ordinary way for firmware
# without the feature.
EXTRA_FLAGS = {"kernels_conv_dlds.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=10"],
               "kernels_misc.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=11"]}


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    """Compiles every source to an object (in parallel) and links the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, s + ".%d.o" % os.getpid()) for s in SOURCES]
    cmds = [["hipcc"] + FLAGS + EXTRA_FLAGS.get(s, []) + ["-x", "hip", "-c", os.path.join(CSRC, s), "-o", o]
            for s, o in zip(SOURCES, objs)]
    try:
        with ThreadPoolExecutor(max_workers=min(len(cmds), 8)) as ex:
            list(ex.map(lambda c: _run(c, verbose), cmds))
        tmp = LIB + ".tmp%d" % os.getpid()
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + objs + ["-o", tmp], verbose)
        os.replace(tmp, LIB)
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    return LIB


if __name__ == "__main__":
    print("built", build(verbose=True))
