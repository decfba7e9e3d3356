"""Builds and runs the three stand-alone microbenchmarks of this folder on the GPU (needs an MI355X and
hipcc): per-CU limits that bound the convolution kernel -- the direct-to-LDS load rate, the LDS read
rate per wave and per CU, and the MFMA issue rate.

  python -m paper_2006_02464_amd.microbench [--out FILE]
"""
import argparse
import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
NAMES = ("dma_rate", "lds_rate", "mfma_rate")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    args = ap.parse_args()
    text = []
    with tempfile.TemporaryDirectory() as tmp:
        for name in NAMES:
            exe = os.path.join(tmp, name)
            subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                            "-o", exe, os.path.join(HERE, name + ".hip")], check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
            out = subprocess.run([exe], check=True, capture_output=True, text=True, timeout=120).stdout
            text.append("== %s\n%s" % (name, out))
            print(text[-1], flush=True)
    if args.out:
        with open(args.out, "w") as f:
            f.write("\n".join(text))


if __name__ == "__main__":
    sys.exit(main())
