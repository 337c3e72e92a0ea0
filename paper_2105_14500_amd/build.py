"""Compile the HIP library for gfx950 into paper_2105_14500_amd/libtesseract_hip.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtesseract_hip.so")
SOURCES = [os.path.join(CSRC, "tess_api.cpp"), os.path.join(CSRC, "tess_kernels.hip"),
           os.path.join(CSRC, "tess_layernorm.hip")]
HEADERS = [os.path.join(CSRC, "tess_internal.h"), os.path.join(ROOT, "include", "tesseract.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(force=True, extra=()):
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    cmd = ["hipcc"] + FLAGS + list(extra) + ["-x", "hip"] + SOURCES + ["-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
