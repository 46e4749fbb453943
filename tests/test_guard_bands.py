"""Out-of-bounds canaries: every buffer the library WRITES (O, LSE, dQ, dK, dV and both workspaces) sits between
two poisoned margins inside a larger allocation; after forward + backward on ragged shapes at every head_dim the
margins must be untouched, bit for bit.  (The kernels issue surplus and clamped loads by design; this checks the
stores and the workspace carving.)"""
import numpy as np
import pytest
import torch

from paper_2605_08962_amd import workloads as W
from tests._util import upload

pytestmark = pytest.mark.gpu

MARGIN = 1 << 16          # bytes on either side
POISON = 0xA5


class Guarded:
    def __init__(self, nbytes):
        self.n = int(nbytes)
        self.pad = (-self.n) % 256
        self.buf = torch.full((MARGIN + self.n + self.pad + MARGIN,), POISON, dtype=torch.uint8, device="cuda")

    def view(self, dtype, shape):
        return self.buf[MARGIN:MARGIN + self.n].view(dtype).view(shape)

    def bytes_view(self):
        return self.buf[MARGIN:MARGIN + self.n]

    def intact(self):
        lo, hi = self.buf[:MARGIN], self.buf[MARGIN + self.n:]
        return bool((lo == POISON).all()) and bool((hi == POISON).all())


@pytest.mark.parametrize("D", [64, 80, 96, 128])
@pytest.mark.parametrize("causal,Hq,Hkv,kv_splits", [(False, 4, 4, 1), (True, 8, 2, 1), (False, 2, 2, 3)])
def test_margins_around_outputs_and_workspaces_stay_untouched(D, causal, Hq, Hkv, kv_splits):
    from paper_2605_08962_amd import binding
    lengths = [300, 1, 129, 64, 0, 513, 7, 128, 65, 1027, 63]
    w = W.make_custom(lengths, Hq, Hkv, D, causal, seed=900 + D, with_dout=True)
    print(f"lengths={lengths} Hq={Hq} Hkv={Hkv} D={D} causal={causal} kv_splits={kv_splits}", flush=True)
    d = upload(w)
    T = w.total_tokens
    p = binding.make_params(T, w.num_seqs, Hq, Hkv, D, causal, w.scale, kv_splits)
    g = {"o": Guarded(T * Hq * D * 2), "lse": Guarded(Hq * T * 4), "dq": Guarded(T * Hq * D * 2),
         "dk": Guarded(T * Hkv * D * 2), "dv": Guarded(T * Hkv * D * 2),
         "wsf": Guarded(binding.fwd_workspace_bytes(p)), "wsb": Guarded(binding.bwd_workspace_bytes(p))}
    o = g["o"].view(torch.bfloat16, (T, Hq, D))
    lse = g["lse"].view(torch.float32, (Hq, T))
    dq = g["dq"].view(torch.bfloat16, (T, Hq, D))
    dk = g["dk"].view(torch.bfloat16, (T, Hkv, D))
    dv = g["dv"].view(torch.bfloat16, (T, Hkv, D))
    binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], causal, w.scale, out=o, lse=lse,
                            workspace=g["wsf"].bytes_view(), kv_splits=kv_splits)
    binding.varlen_attn_bwd(d["dout"], d["q"], d["k"], d["v"], o, lse, d["cu"], causal, w.scale, dq=dq, dk=dk, dv=dv,
                            workspace=g["wsb"].bytes_view())
    torch.cuda.synchronize()
    for name, gb in g.items():
        assert gb.intact(), f"{name}: a margin was written"
    # the outputs themselves were fully written (no poison pattern left: 0xA5A5 is a bf16 around -7e-17)
    ref_o, ref_lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], causal, w.scale, kv_splits=kv_splits)
    ref = binding.varlen_attn_bwd(d["dout"], d["q"], d["k"], d["v"], ref_o, ref_lse, d["cu"], causal, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(o, ref_o) and torch.equal(lse, ref_lse)
    assert all(torch.equal(a, b) for a, b in zip((dq, dk, dv), ref))
