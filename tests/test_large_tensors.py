"""GPU parity on packed batches whose Q / O / dO / dQ exceed 2^31 elements (and 4 GiB): every offset
that is computed from a token index has to be 64-bit.

The batches are drawn on the device (torch's seeded generator: 2.3e9 normals on the host would take
minutes); the oracle gets the very same bf16 values, copied back for the samples it evaluates.  Those
are the first sample, the sample that holds the first element past 2^31, and the last one; the
gradient identities of tests/test_full_configs.py cover all the others.
"""
import numpy as np
import pytest
import torch

from tests._util import LSE_ABS, assert_close, assert_gradients_close, to_f64

pytestmark = pytest.mark.gpu


def _lengths(rng, total, lo, hi):
    out = []
    left = total
    while left > 0:
        n = int(min(left, rng.integers(lo, hi + 1)))
        out.append(n)
        left -= n
    return np.asarray(out, dtype=np.int64)


def _normal_bf16(shape, gen):
    return torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(torch.bfloat16)


@pytest.mark.parametrize("name,T,Hq,Hkv,D,causal,lo,hi", [
    ("llm_d128", 540_000, 32, 8, 128, True, 300, 1800),     # 2.21e9 elements of Q, 4.4 GB
    ("vit_d64", 2_150_000, 16, 16, 64, False, 500, 3000),   # 2.20e9 elements of Q, K and V each
])
def test_tensors_beyond_two_to_the_31_elements(name, T, Hq, Hkv, D, causal, lo, hi):
    import oracle
    from paper_2605_08962_amd import binding
    from tests.test_full_configs import _gradient_identities

    assert T * Hq * D > 2 ** 31
    rng = np.random.default_rng(31)
    lengths = _lengths(rng, T, lo, hi)
    cu = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(lengths, out=cu[1:])
    scale = 1.0 / np.sqrt(D)
    print(f"case {name} B={len(lengths)} T={T} Hq={Hq} Hkv={Hkv} D={D} causal={causal}", flush=True)

    gen = torch.Generator(device="cuda").manual_seed(2 ** 31 + D)
    d = {"q": _normal_bf16((T, Hq, D), gen), "k": _normal_bf16((T, Hkv, D), gen),
         "v": _normal_bf16((T, Hkv, D), gen), "dout": _normal_bf16((T, Hq, D), gen),
         "cu": torch.from_numpy(cu.astype(np.int32)).cuda()}
    o, lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], causal, scale)
    dq, dk, dv = binding.varlen_attn_bwd(d["dout"], d["q"], d["k"], d["v"], o, lse, d["cu"], causal, scale)
    torch.cuda.synchronize()
    for t in (o, lse, dq, dk, dv):
        assert bool(torch.isfinite(t).all())

    class Shape:  # what _gradient_identities reads of a workload
        num_q_heads, num_kv_heads, total_tokens, num_seqs = Hq, Hkv, T, len(lengths)
    Shape.lengths = lengths
    _gradient_identities(Shape, d, o, dq, dk, dv)

    g = Hq // Hkv
    first_past = (2 ** 31) // (Hq * D)                       # token that holds element 2^31 of Q
    picks = [0, int(np.searchsorted(cu, first_past, side="right") - 1), len(lengths) - 1]
    f32 = lambda t: t.float().cpu().numpy()
    for s, c in zip(picks, (0, Hkv // 2, Hkv - 1)):
        a, b = int(cu[s]), int(cu[s + 1])
        one = np.array([0, b - a], np.int32)
        hs = slice(c * g, (c + 1) * g)
        q, k, v, do = f32(d["q"][a:b, hs]), f32(d["k"][a:b, c:c + 1]), f32(d["v"][a:b, c:c + 1]), f32(d["dout"][a:b, hs])
        ro, rlse = oracle.fwd(q, k, v, one, causal, scale)
        res = [assert_close(f"O[sample {s}]", to_f64(o[a:b, hs]), ro)]
        e = float(np.abs(to_f64(lse[hs, a:b]) - rlse).max())
        assert e <= LSE_ABS, f"LSE[sample {s}]: {e:.3e}"
        # causal and grouped gradients reach |x| >= 2: bound before the final bf16 rounding (tests/_util.py)
        res += assert_gradients_close(f"sample {s} kv head {c}", (to_f64(dq[a:b, hs]), to_f64(dk[a:b, c:c + 1]),
                                                                    to_f64(dv[a:b, c:c + 1])),
                                      q, k, v, do, one, causal, scale, to_f64(o[a:b, hs]), allow_output_rounding=causal)
        print(f"   sample {s} (tokens {a}..{b}) kv head {c}: LSE {e:.2e} " +
              " ".join(f"{n} {x[0]:.2e}/{x[1]:.2e}" for n, x in zip(("O", "dQ", "dK", "dV"), res)), flush=True)
