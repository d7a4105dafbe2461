"""Builds and runs the stand-alone ceiling measurements (needs the GPU):

    python ceilings.py

Prints the HBM read bandwidth a plain streaming kernel and a plain row-gather kernel reach, and the
sustained bf16 MFMA rate by operand data (zeros, ones, random normal) and with vector / LDS work beside the
MFMAs, on the GPU at hand.  These are reported beside the published peaks as "achievable" denominators;
the library itself does not use this program.
"""
import os
import subprocess
import sys

here = os.path.dirname(os.path.abspath(__file__))
exe = os.path.join(here, "_build", "ceilings")
os.makedirs(os.path.dirname(exe), exist_ok=True)
src = os.path.join(here, "ceilings.hip")
if not os.path.exists(exe) or os.path.getmtime(exe) < os.path.getmtime(src):
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", "-Wno-inline-asm", src, "-o", exe], check=True)
sys.exit(subprocess.run([exe]).returncode)
