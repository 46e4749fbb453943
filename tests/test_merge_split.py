"""GPU parity of the merge primitive (varlen_attn_merge) and of the forward with the keys of each
query tile split over several workgroups (kv_splits), both against the fp64 oracle."""
import numpy as np
import pytest
import torch

from paper_2605_08962_amd import workloads as W
from tests._util import LSE_ABS, assert_close, to_f64, to_gpu_bf16, upload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("P,T,H,D", [(1, 50, 2, 64), (2, 777, 3, 80), (3, 1030, 2, 128), (5, 129, 4, 96), (64, 33, 1, 64)])
def test_merge_matches_oracle(P, T, H, D):
    import oracle
    from paper_2605_08962_amd import binding
    print(f"case merge P={P} T={T} H={H} D={D}", flush=True)
    rng = np.random.default_rng(1000 + P + T)
    o_bits = W.f32_to_bf16_bits(rng.standard_normal((P, T, H, D)).astype(np.float32))
    lse = (rng.standard_normal((P, H, T)) * 3.0).astype(np.float32)
    if P > 1:
        # empty parts: some (part, head, row) entries hold no key; their O is NaN garbage that must
        # never be read, and a few rows are empty in every part
        empty = rng.random((P, H, T)) < 0.2
        empty[:, :, :3] = True
        lse[empty] = -np.inf
        nan_bits = np.uint16(0x7FC0)
        o_bits[np.broadcast_to(empty.transpose(0, 2, 1)[..., None], o_bits.shape)] = nan_bits
    ref_o, ref_lse = oracle.merge(W.bf16_bits_to_f32(o_bits), lse.astype(np.float64))
    got_o, got_lse = binding.varlen_attn_merge(to_gpu_bf16(o_bits), torch.from_numpy(lse).cuda())
    torch.cuda.synchronize()
    got_o, got_lse = to_f64(got_o), to_f64(got_lse)
    # single parts pass through, so |O| reaches 4 and more, where half a bf16 ulp alone exceeds 1e-2:
    # the bound is on the value before the one final rounding
    assert_close("O", got_o, ref_o, allow_output_rounding=True)
    fin = np.isfinite(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), ~fin)
    assert np.abs(got_lse[fin] - ref_lse[fin]).max() <= LSE_ABS
    if P > 1:
        assert np.all(got_o[:3] == 0)


def _fwd(w, d, splits):
    from paper_2605_08962_amd import binding
    o, lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], w.causal, w.scale, kv_splits=splits)
    torch.cuda.synchronize()
    return o, lse


@pytest.mark.parametrize("D,causal,Hq,Hkv", [(64, False, 2, 2), (128, True, 4, 2), (80, False, 2, 1), (96, True, 2, 2)])
@pytest.mark.parametrize("splits", [2, 3, 8])
def test_split_forward_matches_oracle(D, causal, Hq, Hkv, splits):
    import oracle
    # lengths: several tiles with a ragged tail, exactly one tile, fewer tiles than chunks, one row
    w = W.make_custom([700, 64, 40, 1, 333], Hq, Hkv, D, causal, seed=300 + D + splits)
    print(f"case split fwd D={D} causal={causal} Hq={Hq} Hkv={Hkv} splits={splits}", flush=True)
    d = upload(w)
    o, lse = _fwd(w, d, splits)
    ro, rlse = oracle.fwd(w.f32("q"), w.f32("k"), w.f32("v"), w.cu_seqlens, w.causal, w.scale)
    assert_close("O", to_f64(o), ro, allow_output_rounding=True)
    assert float(np.abs(to_f64(lse) - rlse).max()) <= LSE_ABS
    # and it is a tuning hint: the unsplit launch gives the same to within one bf16 rounding
    o1, lse1 = _fwd(w, d, 1)
    assert float((o.float() - o1.float()).abs().max()) <= 2.0 ** -6
    assert float((lse - lse1).abs().max()) <= 1e-4


def test_small_launch_is_split_automatically():
    import oracle
    from paper_2605_08962_amd import binding
    # one sample of 4096 tokens, 2 heads of 128: 64 workgroups for 512 slots
    w = W.make_custom([4096], 2, 2, 128, True, seed=99)
    p_auto = binding.make_params(4096, 1, 2, 2, 128, True, w.scale)
    p_off = binding.make_params(4096, 1, 2, 2, 128, True, w.scale, kv_splits=1)
    assert binding.fwd_workspace_bytes(p_auto) > binding.fwd_workspace_bytes(p_off)   # room for the parts
    big = binding.make_params(178572, 64, 16, 16, 64, False, 0.125)
    big_off = binding.make_params(178572, 64, 16, 16, 64, False, 0.125, kv_splits=1)
    assert binding.fwd_workspace_bytes(big) == binding.fwd_workspace_bytes(big_off)  # large launches are not
    d = upload(w)
    o, lse = _fwd(w, d, 0)
    rows = np.unique(np.concatenate([np.arange(0, 130), np.arange(2040, 2060), np.arange(4000, 4096)])).astype(np.int64)
    ro, rlse = oracle.fwd_rows(w.f32("q"), w.f32("k"), w.f32("v"), w.cu_seqlens, True, w.scale, rows)
    rt = torch.from_numpy(rows).cuda()
    assert_close("O", to_f64(o[rt]), ro, allow_output_rounding=True)
    assert float(np.abs(to_f64(lse[:, rt]) - rlse.T).max()) <= LSE_ABS
