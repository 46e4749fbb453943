"""The forward entry point that takes no workspace (varlen_attn_fwd_static_scratch): its scratch is a static
device array inside the library, so it can be called where nothing may be allocated.  Called through the
C ABI and compared with varlen_attn_fwd, whose kernels it shares: the results must be identical bit for
bit (and so match the oracle exactly as varlen_attn_fwd's do), on two calls in a row, the second with a
smaller input, so that whatever the first call left in the shared array is in the way of the second."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2605_08962_amd import workloads as W
from tests._util import LSE_ABS, assert_close, to_f64, upload

pytestmark = pytest.mark.gpu


def _both(w, kv_splits):
    from paper_2605_08962_amd import binding
    d = upload(w)
    ref_o, ref_lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], w.causal, w.scale, kv_splits=kv_splits)
    o = torch.full_like(d["q"], float("nan"))
    lse = torch.full((w.num_q_heads, w.total_tokens), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.varlen_attn_fwd_static_scratch(d["q"], d["k"], d["v"], d["cu"], w.causal, w.scale, o, lse,
                                           kv_splits=kv_splits)
    assert torch.cuda.memory_allocated() == before            # (torch's allocator saw no request either)
    torch.cuda.synchronize()
    assert torch.equal(o, ref_o) and torch.equal(lse, ref_lse), f"{w.name}: differs from varlen_attn_fwd"
    return o, lse


@pytest.mark.parametrize("first,second", [
    # (lengths, Hq, Hkv, D, causal, kv_splits) of the first call, then of the smaller second call
    (([700, 129, 64, 1, 300], 4, 2, 64, False, 0), ([37, 16, 129], 2, 2, 64, False, 0)),
    (([1500, 260], 8, 2, 128, True, 0), ([300], 4, 1, 128, True, 0)),
    (([4096], 2, 2, 80, False, 4), ([1024], 2, 2, 80, False, 2)),     # keys split: partial results in the scratch
])
def test_static_scratch_forward_equals_the_workspace_forward(first, second):
    import oracle
    for i, (lengths, Hq, Hkv, D, causal, splits) in enumerate((first, second)):
        w = W.make_custom(lengths, Hq, Hkv, D, causal, seed=700 + i + D, with_dout=False)
        print(f"call {i}: lengths={lengths} Hq={Hq} Hkv={Hkv} D={D} causal={causal} kv_splits={splits}", flush=True)
        o, lse = _both(w, splits)
        ro, rlse = oracle.fwd(w.f32("q"), w.f32("k"), w.f32("v"), w.cu_seqlens, causal, w.scale)
        assert_close("O", to_f64(o), ro, allow_output_rounding=True)
        assert float(np.abs(to_f64(lse) - rlse).max()) <= LSE_ABS


def test_static_scratch_limit_and_argument_errors():
    from paper_2605_08962_amd import binding
    lib = binding.load()
    # needs more than the static array: 8 splits of 200000 tokens x 16 heads x 64 fp32 -- rejected on the host,
    # before any pointer is looked at
    p = binding.make_params(200000, 4, 16, 16, 64, False, 0.125, 8)
    assert binding.fwd_workspace_bytes(p) > binding.STATIC_SCRATCH_BYTES
    rc = lib.varlen_attn_fwd_static_scratch(ctypes.byref(p), 16, 16, 16, 16, 16, 16, None)
    assert rc == binding.VA_ERR_SCRATCH_LIMIT and "scratch" in binding.status_string(rc)
    # the same sizes unsplit fit
    p1 = binding.make_params(200000, 4, 16, 16, 64, False, 0.125, 1)
    assert binding.fwd_workspace_bytes(p1) <= binding.STATIC_SCRATCH_BYTES
    # argument errors as in varlen_attn_fwd
    ok = binding.make_params(8, 1, 2, 2, 64, False, 0.125, 1)
    assert lib.varlen_attn_fwd_static_scratch(ctypes.byref(ok), None, 16, 16, 16, 16, 16, None) == 1
    assert lib.varlen_attn_fwd_static_scratch(ctypes.byref(ok), 16, 24, 16, 16, 16, 16, None) == 7
    bad = binding.make_params(8, 1, 2, 2, 72, False, 0.125, 1)
    assert lib.varlen_attn_fwd_static_scratch(ctypes.byref(bad), 16, 16, 16, 16, 16, 16, None) == 3
    assert lib.varlen_attn_fwd_static_scratch(ctypes.byref(binding.make_params(0, 0, 2, 2, 64, False, 0.1)),
                                              None, None, None, None, None, None, None) == 0
