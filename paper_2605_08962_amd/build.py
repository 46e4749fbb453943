"""Builds libvarlen_attn.so from csrc/ with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvarlen_attn.so")
# (source, object name, extra flags).  va_bwd.hip is built in three parts: the head_dim 128 dK/dV and dQ
# kernels get their own instruction-scheduling strategy (measured faster there: dK/dV 7 %, the two-workgroup dQ
# kernel 1-7 %; slower for the other head sizes), and dK/dV at 128 is told to let MFMAs write S and dP into
# ordinary vector registers: it runs one wave per SIMD on more than 256 registers, and the default puts every
# MFMA result into the accumulation half of the register file, from where the vector ALU needs a copy per
# register (64 per step; 5 % of its time).
SOURCES = [("va_api.hip", "va_api.o", []), ("va_sched.hip", "va_sched.o", []), ("va_fwd.hip", "va_fwd.o", []),
           ("va_bwd.hip", "va_bwd.o", ["-DVA_BWD_PART=0"]),
           ("va_bwd.hip", "va_bwd_dkdv128.o", ["-DVA_BWD_PART=1", "-mllvm", "-amdgpu-sched-strategy=iterative-ilp",
                                               "-mllvm", "-amdgpu-mfma-vgpr-form=1"]),
           ("va_bwd.hip", "va_bwd_dq128.o", ["-DVA_BWD_PART=2", "-mllvm", "-amdgpu-sched-strategy=iterative-ilp"]),
           ("va_partition.hip", "va_partition.o", []), ("va_merge.hip", "va_merge.o", [])]
# -packed-fp32-ops is switched off on purpose: hipcc must not form v_pk_*_f32 from float code.
# -fno-honor-nans: the kernels never produce NaN from finite inputs (masked scores use a finite
# sentinel), and without it every fmaxf of an MFMA result costs an extra canonicalising v_max.
# -Wno-inline-asm: the direct-to-LDS load statements name M0 as clobbered (they overwrite it); clang remarks
# on every one of them that M0 is a reserved register it will not save, which is exactly what is meant.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         "-fno-honor-nans",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(item):
    src, objname, extra = item
    obj = os.path.join(CSRC, "_build", objname)
    cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build():
    os.makedirs(os.path.join(CSRC, "_build"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
