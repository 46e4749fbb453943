"""Writes tests/golden/config1_fwd_samples.txt from the CPU oracle alone.

The paper prints no numeric attention example, so these are not paper values: they are the
oracle's own outputs on BASELINE config 1, stored so that an accidental change of the oracle's
arithmetic or of the input generator shows up.  Run: python tests/golden/make_golden.py
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402
from paper_2605_08962_amd import workloads as W  # noqa: E402

w = W.make(1)
o, lse = oracle.fwd(w.f32("q"), w.f32("k"), w.f32("v"), w.cu_seqlens, False, w.scale)
out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_fwd_samples.txt")
with open(out, "w") as f:
    f.write("# oracle outputs on BASELINE config 1 (seed 1001); kind token head dim value\n")
    f.write("# written by tests/golden/make_golden.py, which calls only oracle/\n")
    for t in (0, 15, 16, 52, 53, 116, 117, 245):
        for h in (0, 1):
            f.write(f"O {t} {h} 0 {float(o[t, h, 0])!r}\n")
            f.write(f"O {t} {h} 63 {float(o[t, h, 63])!r}\n")
            f.write(f"LSE {t} {h} 0 {float(lse[h, t])!r}\n")
print("wrote", out)
