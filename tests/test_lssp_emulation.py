"""Long-short sequence parallelism (Section 4.1.1) as the ranks of one node execute it, emulated on one GPU
with no communication: the samples of a mixed batch are split at a length threshold eta; the long ones run in
the sequence-parallel (Ulysses) state, where every rank holds ALL tokens of the long samples for H / SP of the
heads; the short ones run in the data-parallel state, where every rank holds whole samples (its share of a
length-balanced partition, varlen_attn_balance_partition) for all heads.  The pieces are put back together and
must be what one call on the unsplit batch gives: bit for bit against the GPU's own unsplit call (a (sample,
head) result depends on nothing it is packed or launched with), and within the stated bounds against the
oracle on the unsplit batch."""
import numpy as np
import pytest
import torch

from paper_2605_08962_amd import workloads as W
from tests._util import LSE_ABS, assert_close, assert_gradients_close, to_f64, upload

pytestmark = pytest.mark.gpu


def _run(binding, d, rows, heads_q, heads_kv, lengths, causal, scale):
    """Forward + backward on the listed packed rows and head slices, as one rank would: its own packed buffers."""
    idx = torch.from_numpy(rows).cuda()
    q, do = (d[n][idx][:, heads_q].contiguous() for n in ("q", "dout"))
    k, v = (d[n][idx][:, heads_kv].contiguous() for n in ("k", "v"))
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)).cuda()
    o, lse = binding.varlen_attn_fwd(q, k, v, cu, causal, scale, kv_splits=1)
    dq, dk, dv = binding.varlen_attn_bwd(do, q, k, v, o, lse, cu, causal, scale)
    return idx, o, lse, dq, dk, dv


@pytest.mark.parametrize("Hq,Hkv,D,causal,SP,eta", [(8, 8, 80, False, 4, 1024), (8, 8, 64, False, 8, 512),
                                                     (16, 4, 128, True, 2, 700)])
def test_lssp_split_reassembles_to_the_unsplit_result(Hq, Hkv, D, causal, SP, eta):
    from paper_2605_08962_amd import binding
    lengths = np.array([3000, 200, 64, 700, 5000, 129, 1024, 333, 90, 2048, 1, 513, 77, 1500, 260], dtype=np.int64)
    w = W.make_custom(lengths, Hq, Hkv, D, causal, seed=1500 + D + SP, with_dout=True)
    print(f"lengths={list(lengths)} Hq={Hq} Hkv={Hkv} D={D} causal={causal} SP={SP} eta={eta}", flush=True)
    d = upload(w)
    cu = w.cu_seqlens.astype(np.int64)
    g = Hq // Hkv
    # the unsplit call
    o0, lse0 = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], causal, w.scale, kv_splits=1)
    dq0, dk0, dv0 = binding.varlen_attn_bwd(d["dout"], d["q"], d["k"], d["v"], o0, lse0, d["cu"], causal, w.scale)

    o, dq = torch.full_like(o0, float("nan")), torch.full_like(dq0, float("nan"))
    lse = torch.full_like(lse0, float("nan"))
    dk, dv = torch.full_like(dk0, float("nan")), torch.full_like(dv0, float("nan"))
    rows_of = lambda samples: np.concatenate([np.arange(cu[s], cu[s + 1]) for s in samples]) if len(samples) else np.zeros(0, np.int64)

    def put(idx, hq, hkv, res):
        ro, rlse, rdq, rdk, rdv = res
        hq_i, hkv_i = torch.arange(Hq, device="cuda")[hq], torch.arange(Hkv, device="cuda")[hkv]
        o[idx[:, None], hq_i[None, :]] = ro
        dq[idx[:, None], hq_i[None, :]] = rdq
        lse[hq_i[:, None], idx[None, :]] = rlse
        dk[idx[:, None], hkv_i[None, :]] = rdk
        dv[idx[:, None], hkv_i[None, :]] = rdv

    long_s = [s for s in range(len(lengths)) if lengths[s] > eta]
    short_s = [s for s in range(len(lengths)) if lengths[s] <= eta]
    assert long_s and short_s
    # sequence-parallel state: rank r holds every token of the long samples for its slice of the heads
    for r in range(SP):
        hkv = slice(r * Hkv // SP, (r + 1) * Hkv // SP)
        hq = slice(hkv.start * g, hkv.stop * g)
        idx, *res = _run(binding, d, rows_of(long_s), hq, hkv, lengths[long_s], causal, w.scale)
        put(idx, hq, hkv, res)
    # data-parallel state: whole short samples, balanced over the ranks by the library's partitioner
    bin_of, _ = binding.balance_partition(lengths[short_s], SP, binding.PARTITION_KARMARKAR_KARP)
    for r in range(SP):
        mine = [short_s[i] for i in range(len(short_s)) if bin_of[i] == r]
        if not mine:
            continue
        idx, *res = _run(binding, d, rows_of(mine), slice(0, Hq), slice(0, Hkv), lengths[mine], causal, w.scale)
        put(idx, slice(0, Hq), slice(0, Hkv), res)
    torch.cuda.synchronize()

    for name, a, b in (("O", o, o0), ("LSE", lse, lse0), ("dQ", dq, dq0), ("dK", dk, dk0), ("dV", dv, dv0)):
        assert torch.equal(a, b), f"{name}: the reassembled pieces differ from the unsplit call"
    # and against the oracle on the unsplit batch
    import oracle
    q, k, v, do = w.f32("q"), w.f32("k"), w.f32("v"), w.f32("dout")
    ro, rlse = oracle.fwd(q, k, v, w.cu_seqlens, causal, w.scale)
    assert_close("O", to_f64(o), ro, allow_output_rounding=True)
    assert float(np.abs(to_f64(lse) - rlse).max()) <= LSE_ABS
    assert_gradients_close("reassembled", (to_f64(dq), to_f64(dk), to_f64(dv)), q, k, v, do, w.cu_seqlens, causal,
                           w.scale, to_f64(o), allow_output_rounding=True)
