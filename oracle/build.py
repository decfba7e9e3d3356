"""Compile the C oracle with gcc into two shared libraries (fp32 and fp64 builds).

Test infrastructure: building the checker is not using it.  Run as
``python -m oracle.build``; the wrapper in :mod:`oracle.network` also calls
:func:`build` on first use when a library is missing or older than the source.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle.c")
LIBS = {
    "f32": (os.path.join(HERE, "liboracle_f32.so"), "float"),
    "f64": (os.path.join(HERE, "liboracle_f64.so"), "double"),
}


def build(force: bool = False) -> None:
    for _, (lib, real) in LIBS.items():
        if (not force and os.path.exists(lib)
                and os.path.getmtime(lib) >= os.path.getmtime(SRC)):
            continue
        tmp = lib + ".tmp%d" % os.getpid()
        # -O2, no -ffast-math: the compiler may not reassociate the sums.
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-DREAL=" + real,
               "-o", tmp, SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, lib)


if __name__ == "__main__":
    build(force=True)
    print("built", ", ".join(v[0] for v in LIBS.values()))
