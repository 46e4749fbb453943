"""Shared helpers for the GPU parity tests: device upload and the error measures.

Tolerances (bf16 inputs, fp32 accumulation): max abs error <= 1e-2, relative RMS error <= 5e-3
for O and the gradients, max abs error <= 1e-3 for LSE.  max-abs is taken over all elements,
relative RMS is sqrt(sum (gpu - ref)^2 / sum ref^2) per tensor; the oracle is not rounded.
"""
import numpy as np
import torch

MAX_ABS = 1e-2
REL_RMS = 5e-3
LSE_ABS = 1e-3


def to_gpu_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def upload(w):
    d = {n: to_gpu_bf16(getattr(w, n)) for n in ("q", "k", "v")}
    if w.dout is not None:
        d["dout"] = to_gpu_bf16(w.dout)
    d["cu"] = torch.from_numpy(w.cu_seqlens).cuda()
    return d


def to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def errors(got, ref):
    diff = got - ref
    max_abs = float(np.abs(diff).max()) if diff.size else 0.0
    den = float(np.sqrt((ref * ref).sum()))
    rel_rms = float(np.sqrt((diff * diff).sum())) / den if den > 0 else 0.0
    return max_abs, rel_rms


def bf16_half_ulp(x):
    """Half the spacing of bf16 numbers around x: what storing x in bf16 can cost at most."""
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -126)))
    return np.exp2(e - 8)


def assert_close(name, got, ref, max_abs=MAX_ABS, rel_rms=REL_RMS, allow_output_rounding=False):
    """allow_output_rounding: only for the robustness inputs whose outputs reach |x| >= 4, where the
    bf16 grid itself is coarser than max_abs; the bound then becomes max_abs + half a bf16 ulp."""
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    if allow_output_rounding:
        excess = np.abs(got - ref) - bf16_half_ulp(ref)
        a = float(excess.max()) if excess.size else 0.0
        r = errors(got, ref)[1]
        assert a <= max_abs and r <= rel_rms, f"{name}: max_abs beyond bf16 rounding={a:.3e} rel_rms={r:.3e}"
        return a, r
    a, r = errors(got, ref)
    assert a <= max_abs and r <= rel_rms, f"{name}: max_abs={a:.3e} (<= {max_abs}) rel_rms={r:.3e} (<= {rel_rms})"
    return a, r
