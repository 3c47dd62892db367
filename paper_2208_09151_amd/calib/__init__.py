"""Counter calibration for the traffic figures: a stand-alone plain-copy program.

Not part of libginex.so and not built by the library's build step.
``python -m paper_2208_09151_amd.calib`` compiles ``calib_copy.hip`` next to itself; running
the program under ``rocprofv3 --pmc FETCH_SIZE`` (then ``WRITE_SIZE``) shows what the
counters report for a copy of known size, which is the scale applied to the counter
readings of the library's kernels.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "calib_copy.hip")
EXE = os.path.join(HERE, "calib_copy")


def build() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "-O3", "--offload-arch=gfx950", SRC, "-o", EXE])
    return EXE
