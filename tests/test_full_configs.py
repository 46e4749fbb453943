"""GPU parity at the five benchmark configurations' full sizes, in the launch configuration bench.py
times (same binding calls, same tile sizes), on sampled outputs.

The oracle cannot finish these sizes whole in seconds, so it is evaluated exactly on samples:
forward rows are independent given K and V (oracle.fwd_rows on a head slice); gradients need whole
samples, and heads are independent, so the oracle runs on (sample, head-group) slices cut out of the
packed batch (a sample's results do not depend on what it is packed with).  Tolerances are the
strict ones: max abs 1e-2, relative RMS 5e-3, LSE abs 1e-3.
"""
import numpy as np
import pytest
import torch

from paper_2605_08962_amd import workloads as W
from tests._util import LSE_ABS, assert_close, assert_gradients_close, to_f64, upload

pytestmark = pytest.mark.gpu


def _sample_rows(w, rng, per_long=192, per_short=6):
    """First/last rows of every sample, rows at tile edges, and random rows."""
    cu = w.cu_seqlens.astype(np.int64)
    rows = []
    for s in range(w.num_seqs):
        a, b = cu[s], cu[s + 1]
        if a == b:
            continue
        L = b - a
        fixed = [0, 1, 2, 3, L - 1, 63, 64, 127, 128, L // 2]
        n = per_long if L > 4096 else per_short
        extra = rng.integers(0, L, size=n)
        for r in list(fixed) + list(extra):
            if 0 <= r < L:
                rows.append(a + r)
    return np.unique(np.asarray(rows, dtype=np.int64))


def _fwd_gpu(w, d):
    from paper_2605_08962_amd import binding
    o, lse = binding.varlen_attn_fwd(d["q"], d["k"], d["v"], d["cu"], w.causal, w.scale)
    torch.cuda.synchronize()
    return o, lse


def _long_sample_rows(w, rng, per_tile=4, tile=128):
    """Rows of the longest sample: per_tile random rows in EVERY query tile, plus the rows around tile and
    key-tile edges and the sample's ends."""
    cu = w.cu_seqlens.astype(np.int64)
    s = int(np.argmax(w.lengths))
    a, L = int(cu[s]), int(w.lengths[s])
    rows = [rng.integers(t * tile, min(L, (t + 1) * tile), size=per_tile) for t in range(-(-L // tile))]
    edges = [0, 1, 31, 32, 63, 64, 65, 127, 128, 129, L // 2 - 1, L // 2, L - 129, L - 128, L - 65, L - 64, L - 1]
    rows.append(np.array([r for r in edges if 0 <= r < L]))
    return a + np.unique(np.concatenate(rows))


def _check_fwd_sampled(w, heads, seed, long_rows_per_tile=0):
    import oracle
    print(f"case {w.name} seed={w.seed} B={w.num_seqs} T={w.total_tokens} Hq={w.num_q_heads} "
          f"Hkv={w.num_kv_heads} D={w.head_dim} causal={w.causal} heads={heads}", flush=True)
    d = upload(w)
    o, lse = _fwd_gpu(w, d)
    rng = np.random.default_rng(seed)
    rows = _sample_rows(w, rng)
    if long_rows_per_tile:
        rows = np.unique(np.concatenate([rows, _long_sample_rows(w, rng, long_rows_per_tile)]))
    rows_t = torch.from_numpy(rows).cuda()
    g = w.num_q_heads // w.num_kv_heads
    q, k, v = w.f32("q"), w.f32("k"), w.f32("v")
    for h in heads:
        c = h // g
        ro, rlse = oracle.fwd_rows(q[:, h:h + 1], k[:, c:c + 1], v[:, c:c + 1], w.cu_seqlens, w.causal,
                                   w.scale, rows)
        got_o = to_f64(o[rows_t, h])
        got_lse = to_f64(lse[h, rows_t])
        a, r = assert_close(f"O[head {h}]", got_o, ro[:, 0])
        e = float(np.abs(got_lse - rlse[:, 0]).max())
        print(f"   head {h}: {rows.size} rows, O max_abs={a:.2e} rel_rms={r:.2e}, LSE max_abs={e:.2e}", flush=True)
        assert e <= LSE_ABS
    # every output element must have been written with something finite
    assert bool(torch.isfinite(o).all()) and bool(torch.isfinite(lse).all())
    return d, o, lse


def test_config2_vit_forward():
    _check_fwd_sampled(W.make(2), heads=(0, 7, 15), seed=2)


@pytest.mark.parametrize("long_pos", ["first", "middle", "last"])
def test_config3_long_short_forward(long_pos):
    # long sample first: ALL 16 heads, and of the 65536-token sample four rows in every one of its 512 query
    # tiles plus the tile-edge rows (2048+ rows; each row is exact on its own); the other two positions
    # re-check one head with the lighter sampling (the results are bit-identical across positions, next test)
    w = W.make(3, long_pos=long_pos)
    if long_pos == "first":
        _check_fwd_sampled(w, heads=tuple(range(16)), seed=3, long_rows_per_tile=4)
    else:
        _check_fwd_sampled(w, heads=(5,), seed=3)


def test_config3_results_do_not_depend_on_long_position():
    # the long sample's output rows are bit-identical wherever the scheduler finds it in the batch
    from paper_2605_08962_amd import binding
    w = W.make(3, long_pos="first")
    d = upload(w)
    o1, lse1 = _fwd_gpu(w, d)
    cu = w.cu_seqlens.astype(np.int64)
    order = list(range(1, 129)) + [0] + list(range(129, 257))       # move the long sample to the middle
    idx = torch.from_numpy(np.concatenate([np.arange(cu[s], cu[s + 1]) for s in order])).cuda()
    lens = w.lengths[order]
    cu2 = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
    o2, lse2 = binding.varlen_attn_fwd(d["q"][idx].contiguous(), d["k"][idx].contiguous(),
                                       d["v"][idx].contiguous(), cu2, False, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(o2, o1[idx]) and torch.equal(lse2, lse1[:, idx])


def test_config4_llm_causal_gqa_forward():
    _check_fwd_sampled(W.make(4), heads=(0, 13, 31), seed=4)


def test_config5_vit_forward_backward():
    import oracle
    from paper_2605_08962_amd import binding
    w = W.make(5)
    d, o, lse = _check_fwd_sampled(w, heads=(3,), seed=5)
    dq, dk, dv = binding.varlen_attn_bwd(d["dout"], d["q"], d["k"], d["v"], o, lse, d["cu"], w.causal, w.scale)
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(t).all()) for t in (dq, dk, dv))
    cu = w.cu_seqlens.astype(np.int64)
    order = np.argsort(w.lengths, kind="stable")
    picks = [(int(order[0]), (0, 15)), (int(order[len(order) // 2]), (6,)), (int(order[-1]), (11,))]
    q, k, v, do = w.f32("q"), w.f32("k"), w.f32("v"), w.f32("dout")
    for s, heads in picks:
        a, b = int(cu[s]), int(cu[s + 1])
        one = np.array([0, b - a], np.int32)
        for h in heads:
            rdq, rdk, rdv = oracle.bwd(q[a:b, h:h + 1], k[a:b, h:h + 1], v[a:b, h:h + 1], do[a:b, h:h + 1],
                                       one, w.causal, w.scale)
            res = []
            for name, got, ref in (("dQ", dq, rdq), ("dK", dk, rdk), ("dV", dv, rdv)):
                res.append(assert_close(f"{name}[sample {s} head {h}]", to_f64(got[a:b, h:h + 1]), ref))
            print(f"   sample {s} (L={b - a}) head {h}: " +
                  " ".join(f"{n} {x[0]:.2e}/{x[1]:.2e}" for n, x in zip(("dQ", "dK", "dV"), res)), flush=True)


# --- backward at the other benchmark shapes (causal + GQA at D = 128, the long/short mix at D = 80) ---

def _gradient_identities(w, d, o, dq, dk, dv):
    """Properties of the exact gradients that hold for every sample at any size.

    With S = scale Q K^T:  dQ = scale dS K and dK = scale dS^T Q give
    sum_i <dQ_i, Q_i> = sum_j <dK_j, K_j> per (sample, kv head) once the query heads of the group are
    added up; dV = P^T dO and O = P V give sum_j <dV_j, V_j> = sum_i <dO_i, O_i>.  The comparison is
    relative to the sum of absolute values of the terms, which bounds what bf16 rounding of the
    outputs (2^-9 per term) can contribute.
    """
    g = w.num_q_heads // w.num_kv_heads
    T = w.total_tokens
    seg = torch.repeat_interleave(torch.arange(w.num_seqs, device="cuda"),
                                  torch.from_numpy(w.lengths).cuda())

    def per_sample(x, heads):       # x: [T, heads] -> [B, heads]
        out = torch.zeros((w.num_seqs, heads), dtype=torch.float64, device="cuda")
        return out.index_add_(0, seg, x)

    f = lambda t: t.double()
    qq = (f(dq) * f(d["q"])).sum(-1).view(T, w.num_kv_heads, g)
    kk = (f(dk) * f(d["k"])).sum(-1)
    vv = (f(dv) * f(d["v"])).sum(-1)
    oo = (f(d["dout"]) * f(o)).sum(-1).view(T, w.num_kv_heads, g)
    pairs = (("<dQ,Q> = <dK,K>", qq.sum(-1), kk, qq.abs().sum(-1) + kk.abs()),
             ("<dV,V> = <dO,O>", vv, oo.sum(-1), vv.abs() + oo.abs().sum(-1)))
    for name, a, b, mag in pairs:
        a, b, mag = per_sample(a, w.num_kv_heads), per_sample(b, w.num_kv_heads), per_sample(mag, w.num_kv_heads)
        rel = ((a - b).abs() / mag.clamp_min(1e-30)).max().item()
        print(f"   identity {name}: worst |lhs - rhs| / sum|terms| = {rel:.2e}", flush=True)
        assert rel <= 2e-3, name


def _bwd_gpu(w):
    from paper_2605_08962_amd import binding
    d = upload(w)
    o, lse = _fwd_gpu(w, d)
    dq, dk, dv = binding.varlen_attn_bwd(d["dout"], d["q"], d["k"], d["v"], o, lse, d["cu"], w.causal, w.scale)
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(t).all()) for t in (dq, dk, dv))
    return d, o, dq, dk, dv


def _check_bwd_sampled(w, picks, allow_output_rounding=False):
    """Full-size backward on the GPU; the oracle on whole (sample, kv-head group) slices, at the strict
    bounds against the exact gradients of what the backward was given (tests/_util.py)."""
    print(f"case {w.name} seed={w.seed} B={w.num_seqs} T={w.total_tokens} Hq={w.num_q_heads} "
          f"Hkv={w.num_kv_heads} D={w.head_dim} causal={w.causal} picks={picks}", flush=True)
    d, o, dq, dk, dv = _bwd_gpu(w)
    _gradient_identities(w, d, o, dq, dk, dv)
    g = w.num_q_heads // w.num_kv_heads
    cu = w.cu_seqlens.astype(np.int64)
    q, k, v, do = w.f32("q"), w.f32("k"), w.f32("v"), w.f32("dout")
    for s, c in picks:
        a, b = int(cu[s]), int(cu[s + 1])
        one = np.array([0, b - a], np.int32)
        hs = slice(c * g, (c + 1) * g)
        assert_gradients_close(f"sample {s} (L={b - a}) kv head {c}",
                               (to_f64(dq[a:b, hs]), to_f64(dk[a:b, c:c + 1]), to_f64(dv[a:b, c:c + 1])),
                               q[a:b, hs], k[a:b, c:c + 1], v[a:b, c:c + 1], do[a:b, hs], one, w.causal, w.scale,
                               to_f64(o[a:b, hs]), allow_output_rounding=allow_output_rounding)
    return d, o, dq, dk, dv


def test_config4_llm_causal_gqa_backward():
    # gradients under the causal mask summed over a GQA group of 4 reach |x| >= 2: the bound is 1e-2 before
    # the final bf16 rounding
    w = W.make(4, with_dout=True)
    order = np.argsort(w.lengths, kind="stable")
    mid = [int(s) for s in order if w.lengths[s] <= 4096]
    picks = [(int(order[0]), 0), (mid[-1], 5), (int(order[-2]), 7)]
    _check_bwd_sampled(w, picks, allow_output_rounding=True)


def test_config3_long_short_backward():
    """D = 80, full attention.  Short samples: the oracle on whole (sample, head) slices.  The 65536-token
    sample (98.9 % of the flops): element by element on sampled rows.  dQ rows are independent given K and
    V (oracle.bwd_q_rows: rows in every fourth query tile, the tile-edge rows, all 16 heads); dK/dV rows of
    one head need LSE and Delta of all 65536 query rows of that head first (oracle.bwd_kv_rows, about
    1.4e12 flop), then the listed key rows.  Strict bounds, stored-O reference (tests/_util.py)."""
    import oracle
    w = W.make(3, with_dout=True)
    order = np.argsort(w.lengths, kind="stable")
    picks = [(int(order[0]), 2), (int(order[128]), 9), (int(order[-2]), 15)]
    d, o, dq, dk, dv = _check_bwd_sampled(w, picks)
    cu = w.cu_seqlens.astype(np.int64)
    s = int(np.argmax(w.lengths))
    a, b = int(cu[s]), int(cu[s + 1])
    L = b - a
    one = np.array([0, L], np.int32)
    rng = np.random.default_rng(33)
    edges = np.array([0, 1, 63, 64, 127, 128, 129, 191, 192, L // 2, L - 129, L - 128, L - 64, L - 1])
    q, k, v, do = (w.f32(n)[a:b] for n in ("q", "k", "v", "dout"))
    o_l = to_f64(o[a:b])

    # dQ: one random row in every fourth query tile (128 tiles of the 512) + the edges, all heads
    rows = np.unique(np.concatenate([edges, np.arange(0, L, 512) + rng.integers(0, 128, size=L // 512)]))
    ref = oracle.bwd_q_rows(q, k, v, do, one, False, w.scale, rows, o_saved=o_l)
    own = oracle.bwd_q_rows(q, k, v, do, one, False, w.scale, rows)
    got = to_f64(dq[a:b][torch.from_numpy(rows).cuda()])
    am, rm = assert_close("dQ[long sample rows]", got, ref)
    print(f"   long sample dQ: {rows.size} rows x 16 heads, max_abs={am:.2e} rel_rms={rm:.2e} | stored-O vs own-O "
          f"oracle {np.abs(ref - own).max():.2e}, GPU vs own-O oracle {np.abs(got - own).max():.2e}", flush=True)

    # dK, dV: head 9 (kv head = query head here), key rows in every fourth key tile + the edges
    c = 9
    rows = np.unique(np.concatenate([edges, np.arange(0, L, 512) + rng.integers(0, 128, size=L // 512)]))
    rdk, rdv = oracle.bwd_kv_rows(q[:, c:c + 1], k[:, c:c + 1], v[:, c:c + 1], do[:, c:c + 1], one, False, w.scale,
                                  0, rows, o_saved=o_l[:, c:c + 1])
    rows_t = torch.from_numpy(rows).cuda()
    for name, got, ref in (("dK", dk[a:b][rows_t, c], rdk), ("dV", dv[a:b][rows_t, c], rdv)):
        am, rm = assert_close(f"{name}[long sample rows, head {c}]", to_f64(got), ref)
        print(f"   long sample {name}: {rows.size} rows of head {c}, max_abs={am:.2e} rel_rms={rm:.2e}", flush=True)
