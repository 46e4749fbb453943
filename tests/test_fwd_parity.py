"""GPU forward parity: the HIP path through the C ABI against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2605_08962_amd import workloads as W
from tests._util import LSE_ABS, assert_close, to_f64, upload

pytestmark = pytest.mark.gpu


def _run_fwd(w):
    from paper_2605_08962_amd import binding
    d = upload(w)
    o, lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], w.causal, w.scale)
    torch.cuda.synchronize()
    return to_f64(o), to_f64(lse)


def _check_full(w, allow_output_rounding=False):
    import oracle
    print(f"case {w.name} seed={w.seed} B={w.num_seqs} T={w.total_tokens} Hq={w.num_q_heads} "
          f"Hkv={w.num_kv_heads} D={w.head_dim} causal={w.causal}", flush=True)
    o, lse = _run_fwd(w)
    ro, rlse = oracle.fwd(w.f32("q"), w.f32("k"), w.f32("v"), w.cu_seqlens, w.causal, w.scale)
    assert_close("O", o, ro, allow_output_rounding=allow_output_rounding)
    if lse.size:
        assert float(np.abs(lse - rlse).max()) <= LSE_ABS


def test_config1_tiny_noncausal():
    _check_full(W.make(1))


@pytest.mark.parametrize("D", [64, 80, 96, 128])
@pytest.mark.parametrize("causal", [False, True])
def test_ragged_multi_tile(D, causal):
    # spans several 128-row query tiles and 64-row key tiles, with ragged tails and tiny samples
    w = W.make_custom([300, 1, 129, 64, 0, 513, 7, 128, 65], 4, 4, D, causal, seed=11 + D + causal)
    _check_full(w)


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 2, 128), (6, 1, 64), (32, 8, 128), (4, 4, 80)])
@pytest.mark.parametrize("causal", [False, True])
def test_gqa(Hq, Hkv, D, causal):
    w = W.make_custom([257, 33, 190], Hq, Hkv, D, causal, seed=5 + Hq + D)
    _check_full(w)


@pytest.mark.parametrize("D", [64, 80, 128])
def test_peaky_softmax(D):
    # Q scaled by 8 makes rows nearly one-hot and moves the running max often.  Outputs are then
    # close to single V rows, |O| reaches 4 and more, where bf16 cannot hold a value to 1e-2.
    w = W.make_custom([400, 90], 2, 2, D, False, seed=21 + D, q_gain=8.0)
    _check_full(w, allow_output_rounding=True)
    w = W.make_custom([400, 90], 2, 1, D, True, seed=22 + D, q_gain=8.0)
    _check_full(w, allow_output_rounding=True)


@pytest.mark.parametrize("D,causal", [(64, False), (128, True), (80, False)])
def test_scores_that_outgrow_the_first_tile(D, causal):
    # The keys of each sample's first tile are tiny and the later ones large, so the reference
    # maximum fixed by the first tile is exceeded by far more than 2^30 afterwards (scores reach
    # several hundred): the mask-free tiles taken on trust must notice and repeat with a new maximum.
    w = W.make_custom([500, 321, 64], 2, 2, D, causal, seed=77 + D)
    k = W.bf16_bits_to_f32(w.k)
    cu = w.cu_seqlens
    for s in range(w.num_seqs):
        k[cu[s]:cu[s] + 64] *= 0.01
        k[cu[s] + 64:cu[s + 1]] *= 12.0
    w.k = W.f32_to_bf16_bits(k)
    _check_full(w, allow_output_rounding=True)


def test_scale_zero_gives_prefix_means():
    from paper_2605_08962_amd import binding
    w = W.make_custom([70, 130], 2, 2, 64, True, seed=3)
    d = upload(w)
    o, lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], True, 0.0)
    torch.cuda.synchronize()
    v = w.f32("v").astype(np.float64)
    cu = w.cu_seqlens
    for s in range(2):
        seg = v[cu[s]:cu[s + 1]]
        n = np.arange(1, len(seg) + 1)[:, None, None]
        ref = np.cumsum(seg, 0) / n
        assert_close("O", to_f64(o)[cu[s]:cu[s + 1]], ref)
        assert np.abs(to_f64(lse)[:, cu[s]:cu[s + 1]] - np.log(n[:, 0, 0])[None]).max() <= LSE_ABS


def test_length_one_returns_v_bit_exact():
    w = W.make_custom([1] * 9, 4, 2, 128, True, seed=9)
    o, _ = _run_fwd(w)
    assert np.array_equal(o, np.repeat(w.f32("v").astype(np.float64), 2, axis=1))


def test_packed_equals_alone_and_order_free():
    from paper_2605_08962_amd import binding
    w = W.make_custom([200, 64, 333], 4, 2, 64, False, seed=17)
    d = upload(w)
    # (kv_splits=1: how many workgroups share a query tile's keys is chosen from the size of the
    # launch and changes the rounding; with that fixed, a sample's results are bit-identical whatever
    # it is packed with)
    o, lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], False, w.scale, kv_splits=1)
    cu = w.cu_seqlens
    for s in range(3):
        a, b = int(cu[s]), int(cu[s + 1])
        one = torch.tensor([0, b - a], dtype=torch.int32, device="cuda")
        o1, lse1 = binding.varlen_attn_fwd(d["q"][a:b].contiguous(), d["k"][a:b].contiguous(),
                                           d["v"][a:b].contiguous(), one, False, w.scale, kv_splits=1)
        assert torch.equal(o1, o[a:b]) and torch.equal(lse1, lse[:, a:b])
        o2, lse2 = binding.varlen_attn_fwd(d["q"][a:b].contiguous(), d["k"][a:b].contiguous(),
                                           d["v"][a:b].contiguous(), one, False, w.scale)
        assert float((o2.float() - o[a:b].float()).abs().max()) <= 2.0 ** -6
        assert float((lse2 - lse[:, a:b]).abs().max()) <= 1e-4


def test_empty_inputs_and_errors():
    from paper_2605_08962_amd import binding
    q = torch.empty((0, 2, 64), dtype=torch.bfloat16, device="cuda")
    cu = torch.zeros(1, dtype=torch.int32, device="cuda")
    o, lse = binding.varlen_attn_fwd(q, q, q, cu, False, 0.125)
    assert o.shape == (0, 2, 64) and lse.shape == (2, 0)
    q = torch.zeros((8, 2, 48), dtype=torch.bfloat16, device="cuda")
    cu = torch.tensor([0, 8], dtype=torch.int32, device="cuda")
    with pytest.raises(binding.VarlenAttnError) as e:
        binding.varlen_attn_fwd(q, q, q, cu, False, 0.125)
    assert e.value.status == 3
    q = torch.zeros((8, 2, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.VarlenAttnError) as e:
        binding.varlen_attn_fwd(q, q, q, cu, False, -1.0)
    assert e.value.status == 5
    with pytest.raises(binding.VarlenAttnError) as e:
        binding.varlen_attn_fwd(q, q, q, cu, False, 0.125, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 4


def test_cu_seqlens_contents_check():
    """varlen_attn_check_cu_seqlens against the precondition it states, on arrays a packing bug would produce."""
    from paper_2605_08962_amd import binding
    rng = np.random.default_rng(8)
    lengths = rng.integers(0, 300, size=5000)            # several passes of the checking workgroup, empty samples
    cu = np.zeros(lengths.size + 1, dtype=np.int32)
    np.cumsum(lengths, out=cu[1:])
    T = int(cu[-1])
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    assert binding.check_cu_seqlens(dev(cu), T)
    assert binding.check_cu_seqlens(dev([0]), 0) and binding.check_cu_seqlens(dev([0, 7]), 7)
    assert not binding.check_cu_seqlens(dev(cu), T + 1)          # does not end at total_tokens
    assert not binding.check_cu_seqlens(dev(cu + 1), T + 1)      # does not start at 0
    for at in (1, 2500, 4999):                                   # one sample of negative length
        bad = cu.copy()
        bad[at] = bad[at + 1] + 1
        assert not binding.check_cu_seqlens(dev(bad), T)
    assert not binding.check_cu_seqlens(dev([0, -3, 4]), 4)
    assert not binding.check_cu_seqlens(dev([0]), 4)



@pytest.mark.parametrize("D,causal", [(64, False), (80, False), (128, True)])
def test_self_similar_and_shifted_keys(D, causal):
    # Structure that i.i.d. inputs never show: K = Q (every row's own key scores |q|^2 / sqrt(D), about
    # sqrt(D), far above the N(0, 1) rest: a sharp diagonal across every tile), then the same keys moved by
    # a common offset of 3 per channel (softmax does not change, every score does: the running maximum
    # works against a large per-row constant).
    w = W.make_custom([700, 129, 64], 2, 2, D, causal, seed=300 + D)
    w.k = w.q.copy()
    _check_full(w, allow_output_rounding=True)
    w.k = W.f32_to_bf16_bits(W.bf16_bits_to_f32(w.q) + 3.0)
    _check_full(w, allow_output_rounding=True)


@pytest.mark.parametrize("D", [64, 80, 96, 128])
@pytest.mark.parametrize("causal", [False, True])
def test_max_seqlen_hint_selects_the_lean_kernel_and_changes_nothing(D, causal):
    """0 < max_seqlen <= 1024 makes the forward take its lean form (no loads past a tile list's end).  Same
    arithmetic in the same order: the results are bit-identical to the call without the hint, whether the hint
    is right, generous, or WRONG (a sample longer than promised); and they match the oracle."""
    import oracle
    from paper_2605_08962_amd import binding
    lengths = [64, 1, 300, 0, 129, 128, 63, 65, 700, 2, 256, 1000]
    w = W.make_custom(lengths, 4, 2, D, causal, seed=640 + D + causal)
    d = upload(w)
    ref_o, ref_lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], causal, w.scale, kv_splits=1)
    for hint in (1000, 1024, 100, 1):                       # exact, generous, wrong, absurdly wrong
        o, lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], causal, w.scale, kv_splits=1, max_seqlen=hint)
        torch.cuda.synchronize()
        assert torch.equal(o, ref_o) and torch.equal(lse, ref_lse), f"hint {hint}"
    ro, rlse = oracle.fwd(w.f32("q"), w.f32("k"), w.f32("v"), w.cu_seqlens, causal, w.scale)
    assert_close("O", to_f64(o), ro, allow_output_rounding=True)
    assert float(np.abs(to_f64(lse) - rlse).max()) <= LSE_ABS
