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
    """Strict form: max |got - ref| <= max_abs and relative RMS <= rel_rms.

    allow_output_rounding=True is for outputs that reach |x| >= 2 (peaky-softmax robustness inputs,
    tiny samples, gradients under the causal mask or summed over a GQA group, where dK/dV of a
    sample's first keys sum many O(1) terms).  bf16 cannot hold such values to 1e-2: half an ulp is
    0.0078 in [2, 4) and 0.0156 in [4, 8).  There the bound is put on the value BEFORE its final
    rounding to bf16: |got - ref| <= max_abs + half a bf16 ulp of ref.  Relative RMS is unchanged."""
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    if allow_output_rounding:
        excess = np.abs(got - ref) - (max_abs + bf16_half_ulp(ref))
        a, r = errors(got, ref)
        assert (excess <= 0).all() and r <= rel_rms, (
            f"{name}: {int((excess > 0).sum())} elements beyond {max_abs} + half ulp, "
            f"worst excess {float(excess.max()):.3e}; max_abs={a:.3e} rel_rms={r:.3e}")
        return a, r
    a, r = errors(got, ref)
    assert a <= max_abs and r <= rel_rms, f"{name}: max_abs={a:.3e} (<= {max_abs}) rel_rms={r:.3e} (<= {rel_rms})"
    return a, r


def assert_gradients_close(label, got, q, k, v, dout, cu, causal, scale, o_saved, allow_output_rounding=False,
                           rel_rms=REL_RMS, max_abs=MAX_ABS):
    """Gradient parity at the stated bounds.  got = (dQ, dK, dV) float64 from the GPU; q, k, v, dout float32
    arrays of the same slice; o_saved = the forward output the GPU backward was given (what a training step
    stores: bf16), as float64.

    The backward interface takes O as stored, so Delta = <dO, O> inherits O's bf16 rounding whatever the
    kernels do.  The reference is therefore the exact (fp64) gradient arithmetic on the inputs the call
    received, the stored O included: oracle.bwd(..., o_saved=...), held to max abs 1e-2 / relative RMS 5e-3.
    The distance between that and the oracle on its own fp64 O, printed beside it, is the cost of the
    interface, not of the kernels.  Returns [(max_abs, rel_rms)] per tensor against the stored-O reference."""
    import oracle
    ref = oracle.bwd(q, k, v, dout, cu, causal, scale, o_saved=o_saved)
    own = oracle.bwd(q, k, v, dout, cu, causal, scale)
    out = []
    for name, g_, r_, o_ in zip(("dQ", "dK", "dV"), got, ref, own):
        a, r = assert_close(f"{name}[{label}]", g_, r_, max_abs=max_abs, rel_rms=rel_rms,
                            allow_output_rounding=allow_output_rounding)
        iface = float(np.abs(r_ - o_).max()) if r_.size else 0.0
        vs_own = float(np.abs(g_ - o_).max()) if r_.size else 0.0
        print(f"   {name}[{label}]: max_abs={a:.2e} rel_rms={r:.2e} | stored-O vs own-O oracle {iface:.2e}, "
              f"GPU vs own-O oracle {vs_own:.2e}", flush=True)
        out.append((a, r))
    return out
