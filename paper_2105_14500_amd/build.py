"""Compile the HIP library for gfx950 into paper_2105_14500_amd/libtesseract_hip.so."""
import glob
import os
import re
import shutil
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtesseract_hip.so")
SOURCES = [os.path.join(CSRC, "tess_api.cpp"), os.path.join(CSRC, "tess_kernels.hip"),
           os.path.join(CSRC, "tess_layernorm.hip")]
HEADERS = [os.path.join(CSRC, "tess_internal.h"), os.path.join(ROOT, "include", "tesseract.h"),
           os.path.join(ROOT, "include", "tesseract_diag.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-Wno-inline-asm",      # the loader's statements clobber M0 on purpose (see check_m0_writes)
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def check_m0_writes(asm_text):
    """The direct-to-LDS loader sets M0 once for a group of four requests that are issued
    at different points of the software pipeline (tess_kernels.hip, DmaLoader::request).
    That is only sound if nothing else writes M0 in between, which the compiler is not
    told.  Every instruction of the generated device code whose destination is M0 must
    therefore be one of the loader's own: `s_mov_b32 m0, <sgpr>` followed by `s_nop 0`.
    Returns the list of offending lines."""
    lines = [l.strip() for l in asm_text.splitlines()]
    insns = [l for l in lines if l and not l.startswith((".", ";", "/")) and not l.endswith(":")]
    bad = []
    for i, l in enumerate(insns):
        m = re.match(r"^(\S+)\s+m0\b", l)
        if not m:
            continue
        nxt = insns[i + 1] if i + 1 < len(insns) else ""
        if not (m.group(1) == "s_mov_b32" and re.match(r"^s_nop\s+0\b", nxt)):
            bad.append(l)
    return bad


def build(force=True, extra=()):
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    with tempfile.TemporaryDirectory(prefix="tess_build_") as tmp:
        out = os.path.join(tmp, "libtesseract_hip.so")
        cmd = ["hipcc"] + FLAGS + ["--save-temps"] + list(extra) + ["-x", "hip"] + SOURCES + ["-o", out]
        subprocess.run(cmd, check=True, cwd=tmp)
        found = glob.glob(os.path.join(tmp, "tess_kernels-hip-amdgcn*gfx950*.s"))
        if not found:
            raise RuntimeError("no device assembly of tess_kernels.hip was kept: cannot check M0 writes")
        for path in found:
            bad = check_m0_writes(open(path).read())
            if bad:
                raise RuntimeError("compiler-generated writes to M0 in the device code of tess_kernels.hip "
                                   "(they would redirect the direct-to-LDS requests): " + "; ".join(bad[:5]))
        shutil.move(out, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
