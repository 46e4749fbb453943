"""Builds libvarlen_attn.so from csrc/ with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvarlen_attn.so")
# (source, object name, extra flags).  va_bwd.hip is built in three parts: the head_dim 128 dK/dV and dQ
# kernels get their own instruction-scheduling strategy (measured faster there, slower elsewhere), and
# dK/dV at 128 is told to let MFMAs write S and dP into ordinary vector registers: it runs one wave per
# SIMD on more than 256 registers, and the default puts every MFMA result into the accumulation half of
# the register file, from where the vector ALU needs a copy per register (64 per step; 5 % of its time).
SOURCES = [("va_api.hip", "va_api.o", []), ("va_sched.hip", "va_sched.o", []), ("va_fwd.hip", "va_fwd.o", []),
           ("va_bwd.hip", "va_bwd.o", ["-DVA_BWD_PART=0"]),
           ("va_bwd.hip", "va_bwd_dkdv128.o", ["-DVA_BWD_PART=1", "-mllvm", "-amdgpu-sched-strategy=iterative-ilp",
                                               "-mllvm", "-amdgpu-mfma-vgpr-form=1"]),
           ("va_bwd.hip", "va_bwd_dq128.o", ["-DVA_BWD_PART=2", "-mllvm", "-amdgpu-sched-strategy=max-memory-clause"]),
           ("va_partition.hip", "va_partition.o", []), ("va_merge.hip", "va_merge.o", [])]
# -packed-fp32-ops is switched off on purpose: hipcc must not form v_pk_*_f32 from float code.
# -fno-honor-nans: the kernels never produce NaN from finite inputs (masked scores use a finite
# sentinel), and without it every fmaxf of an MFMA result costs an extra canonicalising v_max.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-fno-honor-nans",
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


UBENCH = os.path.join(HERE, "ubench_mfma_valu")
UBENCH_ATOMIC = os.path.join(HERE, "ubench_atomic_rate")


def build_ubench():
    """The stand-alone microbenchmarks: MFMA / vector-ALU overlap (csrc/ubench_mfma_valu.hip) and the fp32
    atomic-add rate that rules out a one-kernel backward (csrc/ubench_atomic_rate.hip)."""
    for src, out in (("ubench_mfma_valu.hip", UBENCH), ("ubench_atomic_rate.hip", UBENCH_ATOMIC)):
        cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               os.path.join(CSRC, src), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + r.stderr)
    return UBENCH


def build():
    os.makedirs(os.path.join(CSRC, "_build"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        ub = ex.submit(build_ubench)
        objs = list(ex.map(_compile, SOURCES))
        ub.result()
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
