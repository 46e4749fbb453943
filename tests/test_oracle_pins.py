"""Pins for the fp64 CPU oracle (CPU only).

The paper prints no attention formula or worked number (Section 6, "Efficient Operators",
only names the exact tiled algorithm it adopts), so the oracle is pinned to what the
mathematics fixes: brute force in a different evaluation order, closed forms, invariances,
reductions to simpler calls, finite differences and a library autograd.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2605_08962_amd import workloads as W


def _tiny(lengths=(5, 1, 9, 3), Hq=2, Hkv=2, D=8, causal=False, seed=7, with_dout=False, q_gain=1.0, scale=None):
    w = W.make_custom(lengths, Hq, Hkv, D, causal, seed, with_dout=with_dout, q_gain=q_gain, scale=scale)
    return w, w.f32("q"), w.f32("k"), w.f32("v")


def _brute(q, k, v, cu, causal, scale):
    """Dense T x T masked scores per head, plain exp / sum with no max subtraction."""
    q, k, v = (np.asarray(a, np.float64) for a in (q, k, v))
    T, Hq, D = q.shape
    g = Hq // k.shape[1]
    sid = np.zeros(T, np.int64)
    for s in range(len(cu) - 1):
        sid[cu[s]:cu[s + 1]] = s
    idx = np.arange(T)
    allowed = sid[:, None] == sid[None, :]
    if causal:
        allowed &= idx[None, :] <= idx[:, None]
    o = np.zeros((T, Hq, D))
    lse = np.zeros((Hq, T))
    for h in range(Hq):
        e = np.where(allowed, np.exp(scale * (q[:, h] @ k[:, h // g].T)), 0.0)
        z = e.sum(1)
        o[:, h] = (e / z[:, None]) @ v[:, h // g]
        lse[h] = np.log(z)
    return o, lse


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (6, 1)])
def test_p1_brute_force(causal, Hq, Hkv):
    w, q, k, v = _tiny(Hq=Hq, Hkv=Hkv, causal=causal)
    o, lse = oracle.fwd(q, k, v, w.cu_seqlens, causal, w.scale)
    o2, lse2 = _brute(q, k, v, w.cu_seqlens, causal, w.scale)
    assert np.abs(o - o2).max() < 1e-12
    assert np.abs(lse - lse2).max() < 1e-12


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("zero", ["q", "scale"])
def test_p2_zero_scores_give_means(causal, zero):
    w, q, k, v = _tiny(lengths=(7, 4, 1), causal=causal)
    scale = w.scale
    if zero == "q":
        q = np.zeros_like(q)
    else:
        scale = 0.0
    o, lse = oracle.fwd(q, k, v, w.cu_seqlens, causal, scale)
    cu = w.cu_seqlens
    v64 = v.astype(np.float64)
    for s in range(w.num_seqs):
        for i in range(cu[s], cu[s + 1]):
            hi = i + 1 if causal else cu[s + 1]
            n = hi - cu[s]
            for h in range(w.num_q_heads):
                assert np.allclose(o[i, h], v64[cu[s]:hi, h].mean(0), rtol=0, atol=1e-14)
                assert abs(lse[h, i] - math.log(n)) < 1e-14


@pytest.mark.parametrize("causal", [False, True])
def test_p3_length_one_returns_v(causal):
    w, q, k, v = _tiny(lengths=(1, 1, 1, 1, 1), Hq=4, Hkv=2, causal=causal)
    o, lse = oracle.fwd(q, k, v, w.cu_seqlens, causal, w.scale)
    for h in range(4):
        assert np.array_equal(o[:, h], v[:, h // 2].astype(np.float64))
        ref = w.scale * np.einsum("td,td->t", q[:, h].astype(np.float64), k[:, h // 2].astype(np.float64))
        assert np.abs(lse[h] - ref).max() < 1e-14


@pytest.mark.parametrize("causal", [False, True])
def test_p4_packed_equals_each_alone(causal):
    w, q, k, v = _tiny(lengths=(6, 11, 2, 0, 4), Hq=4, Hkv=2, causal=causal, with_dout=True)
    do = w.f32("dout")
    cu = w.cu_seqlens
    o, lse = oracle.fwd(q, k, v, cu, causal, w.scale)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, causal, w.scale)
    for s in range(w.num_seqs):
        a, b = cu[s], cu[s + 1]
        if a == b:
            continue
        one = np.array([0, b - a], np.int32)
        o1, lse1 = oracle.fwd(q[a:b], k[a:b], v[a:b], one, causal, w.scale)
        assert np.array_equal(o1, o[a:b]) and np.array_equal(lse1, lse[:, a:b])
        dq1, dk1, dv1 = oracle.bwd(q[a:b], k[a:b], v[a:b], do[a:b], one, causal, w.scale)
        assert np.array_equal(dq1, dq[a:b]) and np.array_equal(dk1, dk[a:b]) and np.array_equal(dv1, dv[a:b])


def test_p5_permutations():
    w, q, k, v = _tiny(lengths=(9, 5), causal=False)
    cu = w.cu_seqlens
    o, lse = oracle.fwd(q, k, v, cu, False, w.scale)
    rng = np.random.default_rng(0)
    perm = np.concatenate([cu[s] + rng.permutation(cu[s + 1] - cu[s]) for s in range(2)])
    # permuting keys and values together leaves every row unchanged (up to summation order)
    o2, lse2 = oracle.fwd(q, k[perm], v[perm], cu, False, w.scale)
    assert np.abs(o2 - o).max() < 1e-14 and np.abs(lse2 - lse).max() < 1e-14
    # permuting queries permutes output rows
    o3, lse3 = oracle.fwd(q[perm], k, v, cu, False, w.scale)
    assert np.array_equal(o3, o[perm]) and np.array_equal(lse3, lse[:, perm])
    # swapping whole sequences swaps their outputs
    sw = np.concatenate([np.arange(9, 14), np.arange(0, 9)])
    o4, lse4 = oracle.fwd(q[sw], k[sw], v[sw], np.array([0, 5, 14], np.int32), False, w.scale)
    assert np.array_equal(o4, o[sw]) and np.array_equal(lse4, lse[:, sw])


@pytest.mark.parametrize("causal", [False, True])
def test_p6_key_shift_invariance(causal):
    w, q, k, v = _tiny(lengths=(8,), Hq=2, Hkv=1, causal=causal)
    c = np.array([0.5, -1.0, 0.25, 2.0, -0.5, 1.0, 0.0, -2.0], np.float32)
    o, lse = oracle.fwd(q, k, v, w.cu_seqlens, causal, w.scale)
    o2, lse2 = oracle.fwd(q, k + c, v, w.cu_seqlens, causal, w.scale)
    assert np.abs(o2 - o).max() < 1e-13
    shift = w.scale * np.einsum("thd,d->ht", q.astype(np.float64), c.astype(np.float64))
    assert np.abs(lse2 - (lse + shift)).max() < 1e-13


def test_p7_causal_row_is_noncausal_prefix():
    w, q, k, v = _tiny(lengths=(10, 3), Hq=2, Hkv=1, causal=True)
    cu = w.cu_seqlens
    o, lse = oracle.fwd(q, k, v, cu, True, w.scale)
    for s in range(2):
        for i in range(cu[s], cu[s + 1]):
            a, b = cu[s], i + 1
            o1, lse1 = oracle.fwd(q[a:b], k[a:b], v[a:b], np.array([0, b - a], np.int32), False, w.scale)
            assert np.array_equal(o1[-1], o[i]) and np.array_equal(lse1[:, -1], lse[:, i])
    # first row of every sequence sees only itself
    assert np.array_equal(o[0, 0], v[0, 0].astype(np.float64))


@pytest.mark.parametrize("causal", [False, True])
def test_p8_gqa_equals_repeated_heads(causal):
    w, q, k, v = _tiny(lengths=(7, 5), Hq=6, Hkv=2, causal=causal, with_dout=True)
    do, cu, g = w.f32("dout"), w.cu_seqlens, 3
    kr, vr = np.repeat(k, g, axis=1), np.repeat(v, g, axis=1)
    o, lse = oracle.fwd(q, k, v, cu, causal, w.scale)
    o2, lse2 = oracle.fwd(q, kr, vr, cu, causal, w.scale)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, causal, w.scale)
    dq2, dk2, dv2 = oracle.bwd(q, kr, vr, do, cu, causal, w.scale)
    assert np.abs(dq - dq2).max() < 1e-14
    T = w.total_tokens
    assert np.abs(dk - dk2.reshape(T, 2, g, -1).sum(2)).max() < 1e-13
    assert np.abs(dv - dv2.reshape(T, 2, g, -1).sum(2)).max() < 1e-13
    # a different (wrong) mapping, h -> h % Hkv, must not give the same answer
    kw = np.tile(k, (1, g, 1))
    o3, _ = oracle.fwd(q, kw, np.tile(v, (1, g, 1)), cu, causal, w.scale)
    assert np.abs(o3 - o).max() > 1e-3


@pytest.mark.parametrize("causal", [False, True])
def test_p9_finite_differences(causal):
    w, q, k, v = _tiny(lengths=(4, 3), Hq=2, Hkv=1, D=4, causal=causal, with_dout=True)
    do, cu = w.f32("dout").astype(np.float64), w.cu_seqlens
    dq, dk, dv = oracle.bwd(q, k, v, do.astype(np.float32), cu, causal, w.scale)

    # the oracle takes float inputs, so differentiate a float64 re-evaluation by brute force
    def loss(q_, k_, v_):
        o_, _ = _brute(q_, k_, v_, cu, causal, w.scale)
        return float((o_ * do).sum())

    eps = 1e-6
    base = [a.astype(np.float64) for a in (q, k, v)]
    for which, grad in enumerate((dq, dk, dv)):
        num = np.zeros_like(grad)
        it = np.nditer(base[which], flags=["multi_index"])
        for _ in it:
            ix = it.multi_index
            args_p = [a.copy() for a in base]
            args_m = [a.copy() for a in base]
            args_p[which][ix] += eps
            args_m[which][ix] -= eps
            num[ix] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        assert np.abs(num - grad).max() < 1e-7 * max(1.0, np.abs(grad).max())


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2)])
def test_p9b_library_autograd(causal, Hq, Hkv):
    """Gradients of a dense masked torch.softmax attention (fp64 autograd) agree with the oracle."""
    w, q, k, v = _tiny(lengths=(6, 1, 9), Hq=Hq, Hkv=Hkv, D=8, causal=causal, with_dout=True)
    do, cu = w.f32("dout"), w.cu_seqlens
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, causal, w.scale)
    o, _ = oracle.fwd(q, k, v, cu, causal, w.scale)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    T = w.total_tokens
    sid = torch.zeros(T, dtype=torch.long)
    for s in range(w.num_seqs):
        sid[cu[s]:cu[s + 1]] = s
    mask = sid[:, None] == sid[None, :]
    if causal:
        mask &= torch.tril(torch.ones(T, T, dtype=torch.bool))
    g = Hq // Hkv
    outs = []
    for h in range(Hq):
        s_ = (tq[:, h] @ tk[:, h // g].T) * w.scale
        p_ = torch.softmax(s_.masked_fill(~mask, float("-inf")), dim=-1)
        outs.append(p_ @ tv[:, h // g])
    to = torch.stack(outs, 1)
    assert np.abs(to.detach().numpy() - o).max() < 1e-13
    to.backward(torch.tensor(do, dtype=torch.float64))
    assert np.abs(tq.grad.numpy() - dq).max() < 1e-12
    assert np.abs(tk.grad.numpy() - dk).max() < 1e-12
    assert np.abs(tv.grad.numpy() - dv).max() < 1e-12


def test_p10_row_identities():
    """dQ is orthogonal to shifts of the scores: sum_j dS_ij = 0 means adding one vector c to every
    key of a sequence changes nothing, so sum_j dK_j-contributions cancel: K-shift directional
    derivative of the loss is 0, i.e. sum over rows of dK (weighted by nothing) has zero q-part."""
    w, q, k, v = _tiny(lengths=(9,), Hq=1, Hkv=1, D=8, causal=False, with_dout=True)
    do = w.f32("dout")
    dq, dk, dv = oracle.bwd(q, k, v, do, w.cu_seqlens, False, w.scale)
    # d loss / d c for K -> K + c (all rows) equals sum_j dK_j and must vanish (shift invariance, P6)
    assert np.abs(dk.sum(0)).max() < 1e-13
    # sum_j dV_j = sum_i dO_i because every row of P sums to one
    assert np.abs(dv.sum(0) - do.astype(np.float64).sum(0)).max() < 1e-13


@pytest.mark.parametrize("causal", [False, True])
def test_p10b_every_row_of_dS_sums_to_zero(causal):
    """Per row: sum_j dS_ij = 0 (because Delta_i = sum_j P_ij dP_ij and sum_j P_ij = 1).  Adding one
    vector c to every key of a sample shifts row i of the scores by the constant q_i.c, which leaves P,
    dP and Delta alone, so dQ_i = scale sum_j dS_ij k_j moves by scale (sum_j dS_ij) c: it must not move,
    for every row and head separately.  dV does not move either; dK_j = scale sum_i dS_ij q_i has no k in it."""
    w, q, k, v = _tiny(lengths=(9, 4, 1), Hq=4, Hkv=2, D=8, causal=causal, with_dout=True)
    do = w.f32("dout")
    # (multiples of 1/2: k + c is then exact in the float32 the oracle takes its inputs in)
    c = (np.random.default_rng(3).integers(-4, 5, size=(1, 2, 8)) / 2.0).astype(np.float32)
    dq, dk, dv = oracle.bwd(q, k, v, do, w.cu_seqlens, causal, w.scale)
    dq2, dk2, dv2 = oracle.bwd(q, k + c, v, do, w.cu_seqlens, causal, w.scale)
    assert np.abs(dq2 - dq).max() < 1e-12 and np.abs(dk2 - dk).max() < 1e-12 and np.abs(dv2 - dv).max() < 1e-12
    assert np.abs(dq).max() > 1e-2      # (the gradients themselves are not small)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2)])
def test_stored_o_variant(causal, Hq, Hkv):
    """Backward with Delta formed from a forward output the caller stored.  Fed the oracle's own fp64 O
    it is the plain backward, bit for bit.  Fed O + E it differs by exactly what the formulas say:
    Delta_i moves by e_i = <dO_i, E_i>, dS_ij by -P_ij e_i, hence
        dQ_i moves by -scale e_i (P K)_i       (P K is the forward's output with V := K),
        dK_j moves by -scale sum_i P_ij e_i q_i (the dV formula with dO := -scale e_i q_i),
        dV does not move."""
    w, q, k, v = _tiny(lengths=(7, 1, 12), Hq=Hq, Hkv=Hkv, D=8, causal=causal, with_dout=True)
    do, cu = w.f32("dout"), w.cu_seqlens
    o, _ = oracle.fwd(q, k, v, cu, causal, w.scale)
    ref = oracle.bwd(q, k, v, do, cu, causal, w.scale)
    same = oracle.bwd(q, k, v, do, cu, causal, w.scale, o_saved=o)
    assert all(np.array_equal(a, b) for a, b in zip(ref, same))
    E = 0.05 * np.random.default_rng(11).standard_normal(o.shape)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, causal, w.scale, o_saved=o + E)
    e = (do.astype(np.float64) * E).sum(-1)                              # [T, Hq]
    pk, _ = oracle.fwd(q, k, k, cu, causal, w.scale)                      # (P K)_i per query head
    assert np.abs(dq - (ref[0] - w.scale * e[..., None] * pk)).max() < 1e-13
    fake_do = (-w.scale * e[..., None] * q.astype(np.float64))
    # the dV formula is linear in dO and only needs P: evaluate it in numpy from the brute-force P
    T = q.shape[0]
    sid = np.repeat(np.arange(len(cu) - 1), np.diff(cu))
    allowed = sid[:, None] == sid[None, :]
    if causal:
        allowed &= np.arange(T)[None, :] <= np.arange(T)[:, None]
    g = Hq // Hkv
    shift = np.zeros_like(ref[1])
    for h in range(Hq):
        sc = np.where(allowed, np.exp(w.scale * (q[:, h].astype(np.float64) @ k[:, h // g].astype(np.float64).T)), 0.0)
        p = sc / sc.sum(1, keepdims=True)
        shift[:, h // g] += p.T @ fake_do[:, h]
    assert np.abs(dk - (ref[1] + shift)).max() < 1e-13
    assert np.array_equal(dv, ref[2])
    assert np.abs(dq - ref[0]).max() > 1e-3 and np.abs(dk - ref[1]).max() > 1e-3   # (E was not negligible)


@pytest.mark.parametrize("causal", [False, True])
def test_backward_row_subsets_match_the_full_backward(causal):
    """dQ of listed query rows, and dK/dV of listed key rows of one kv head, are the full backward's rows
    (same arithmetic, same order: bit for bit), with and without a stored O."""
    w, q, k, v = _tiny(lengths=(6, 0, 11, 1, 3), Hq=4, Hkv=2, D=8, causal=causal, with_dout=True)
    do, cu = w.f32("dout"), w.cu_seqlens
    o, _ = oracle.fwd(q, k, v, cu, causal, w.scale)
    o_st = o + 0.01 * np.random.default_rng(5).standard_normal(o.shape)
    rows = np.array([0, 20, 5, 6, 16, 17, 18], np.int64)
    for saved in (None, o_st):
        dq, dk, dv = oracle.bwd(q, k, v, do, cu, causal, w.scale, o_saved=saved)
        assert np.array_equal(oracle.bwd_q_rows(q, k, v, do, cu, causal, w.scale, rows, o_saved=saved), dq[rows])
        for c in (0, 1):
            dk_r, dv_r = oracle.bwd_kv_rows(q, k, v, do, cu, causal, w.scale, c, rows, o_saved=saved)
            assert np.array_equal(dk_r, dk[rows, c]) and np.array_equal(dv_r, dv[rows, c])
    assert oracle.bwd_q_rows(q, k, v, do, cu, causal, w.scale, np.zeros(0, np.int64)).shape == (0, 4, 8)
    with pytest.raises(RuntimeError):
        oracle.bwd_kv_rows(q, k, v, do, cu, causal, w.scale, 2, rows)
    with pytest.raises(RuntimeError):
        oracle.bwd_q_rows(q, k, v, do, cu, causal, w.scale, np.array([21], np.int64))


def test_p11_zero_q_backward_closed_forms():
    w, q, k, v = _tiny(lengths=(6, 3), Hq=1, Hkv=1, D=8, causal=False, with_dout=True)
    q = np.zeros_like(q)
    do, cu = w.f32("dout").astype(np.float64), w.cu_seqlens
    dq, dk, dv = oracle.bwd(q, k, v, do.astype(np.float32), cu, False, w.scale)
    assert np.abs(dk).max() == 0.0
    for s in range(2):
        a, b = cu[s], cu[s + 1]
        L = b - a
        assert np.abs(dv[a:b, 0] - do[a:b, 0].mean(0)).max() < 1e-14
        dp = do[a:b, 0] @ v[a:b, 0].astype(np.float64).T
        ds = (dp - dp.mean(1, keepdims=True)) / L
        assert np.abs(dq[a:b, 0] - w.scale * ds @ k[a:b, 0].astype(np.float64)).max() < 1e-13


@pytest.mark.parametrize("causal", [False, True])
def test_p12_constant_v(causal):
    w, q, k, v = _tiny(lengths=(7, 2), Hq=2, Hkv=2, causal=causal, q_gain=3.0)
    u = v[0:1].copy()
    vc = np.broadcast_to(u, v.shape).copy()
    o, _ = oracle.fwd(q, k, vc, w.cu_seqlens, causal, w.scale)
    assert np.abs(o - u.astype(np.float64)).max() < 1e-14


def test_p13_large_logits_stay_finite():
    w, q, k, v = _tiny(lengths=(12,), Hq=1, Hkv=1, D=8, causal=False, q_gain=64.0, scale=1.0)
    o, lse = oracle.fwd(q, k, v, w.cu_seqlens, False, 1.0)
    s = (q[:, 0].astype(np.longdouble) @ k[:, 0].astype(np.longdouble).T)
    assert float(np.abs(s).max()) > 400.0
    m = s.max(1, keepdims=True)
    e = np.exp(s - m)
    lse_ld = (m[:, 0] + np.log(e.sum(1))).astype(np.float64)
    o_ld = ((e / e.sum(1, keepdims=True)) @ v[:, 0].astype(np.longdouble)).astype(np.float64)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    assert np.abs(lse[0] - lse_ld).max() < 1e-9 * np.abs(lse_ld).max()
    assert np.abs(o[:, 0] - o_ld).max() < 1e-9


def test_fwd_rows_matches_full():
    w, q, k, v = _tiny(lengths=(6, 0, 11, 1), Hq=4, Hkv=2, causal=True)
    o, lse = oracle.fwd(q, k, v, w.cu_seqlens, True, w.scale)
    rows = np.array([0, 17, 5, 6, 16], np.int64)
    o_r, lse_r = oracle.fwd_rows(q, k, v, w.cu_seqlens, True, w.scale, rows)
    assert np.array_equal(o_r, o[rows]) and np.array_equal(lse_r, lse[:, rows].T)


def test_empty_and_bad_args():
    w, q, k, v = _tiny(lengths=(0, 0), Hq=2, Hkv=2)
    o, lse = oracle.fwd(q, k, v, w.cu_seqlens, False, w.scale)
    assert o.shape == (0, 2, 8) and lse.shape == (2, 0)
    w, q, k, v = _tiny()
    bad = w.cu_seqlens.copy()
    bad[1], bad[2] = bad[2], bad[1]
    with pytest.raises(RuntimeError):
        oracle.fwd(q, k, v, bad, False, w.scale)


def test_config1_matches_brute_force_and_golden():
    """BASELINE config 1 (4 sequences {16,37,64,129}, 2 heads, D=64) against brute force, and the
    stored oracle values (written by tests/golden/make_golden.py from oracle/ alone)."""
    w = W.make(1)
    assert list(w.cu_seqlens) == [0, 16, 53, 117, 246]
    q, k, v = w.f32("q"), w.f32("k"), w.f32("v")
    o, lse = oracle.fwd(q, k, v, w.cu_seqlens, False, w.scale)
    o2, lse2 = _brute(q, k, v, w.cu_seqlens, False, w.scale)
    assert np.abs(o - o2).max() < 1e-12 and np.abs(lse - lse2).max() < 1e-12
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "config1_fwd_samples.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    for kind, a, b, c, val in rows:
        a, b, c = int(a), int(b), int(c)
        got = o[a, b, c] if kind == "O" else lse[b, a]
        assert abs(got - float(val)) < 1e-12


# --- merge of partial results over key shards (oracle.merge) ---

def _partial_attention_numpy(q, k, v, keys, scale):
    """Brute force for ONE sample and head: attention of every query over the key subset `keys`
    (written independently of the C oracle: dense scores, no max subtraction; tiny inputs only)."""
    if len(keys) == 0:
        return np.zeros((q.shape[0], v.shape[1])), np.full(q.shape[0], -np.inf)
    s = scale * (q.astype(np.float64) @ k[keys].astype(np.float64).T)
    e = np.exp(s)
    den = e.sum(1)
    return (e @ v[keys].astype(np.float64)) / den[:, None], np.log(den)


def test_merge_of_shard_results_is_full_attention():
    import oracle
    rng = np.random.default_rng(17)
    L, D = 37, 16
    q, k, v = (rng.standard_normal((L, 1, D)).astype(np.float32) for _ in range(3))
    full_o, full_lse = oracle.fwd(q, k, v, np.array([0, L], np.int32), False, 0.3)
    for shards in ([range(0, 20), range(20, 37)], [range(0, 1), range(1, 36), range(36, 37)],
                   [list(range(0, 37, 2)), list(range(1, 37, 2))], [range(0, 37), []]):
        parts = [_partial_attention_numpy(q[:, 0], k[:, 0], v[:, 0], list(sh), 0.3) for sh in shards]
        o_parts = np.stack([p[0] for p in parts])[:, :, None, :]
        lse_parts = np.stack([p[1] for p in parts])[:, None, :]
        o, lse = oracle.merge(o_parts, lse_parts)
        # o_parts pass through float32 on their way in: 1e-6 is that rounding, not the merge
        assert np.abs(o - full_o).max() < 1e-6 and np.abs(lse - full_lse).max() < 1e-12


def test_merge_special_cases():
    import oracle
    rng = np.random.default_rng(18)
    o = rng.standard_normal((3, 5, 2, 4)).astype(np.float32)
    lse = rng.standard_normal((3, 2, 5))
    # one part: identity
    m_o, m_lse = oracle.merge(o[:1], lse[:1])
    assert np.array_equal(m_o, o[0].astype(np.float64)) and np.allclose(m_lse, lse[0], rtol=0, atol=1e-15)
    # an empty part (-inf) changes nothing, wherever it stands and whatever garbage its O holds
    empty_lse = np.full((1, 2, 5), -np.inf)
    garbage = np.full((1, 5, 2, 4), np.nan, np.float32)
    a_o, a_lse = oracle.merge(o[:2], lse[:2])
    b_o, b_lse = oracle.merge(np.concatenate([o[:1], garbage, o[1:2]]), np.concatenate([lse[:1], empty_lse, lse[1:2]]))
    assert np.array_equal(a_o, b_o) and np.array_equal(a_lse, b_lse)
    # all parts empty: zero output, -inf
    z_o, z_lse = oracle.merge(garbage, empty_lse)
    assert np.all(z_o == 0) and np.all(np.isneginf(z_lse))
    # equal LSEs: plain average and + ln P
    same = np.repeat(lse[:1], 3, axis=0)
    e_o, e_lse = oracle.merge(o, same)
    assert np.allclose(e_o, o.astype(np.float64).mean(0), atol=1e-15) and np.allclose(e_lse, lse[0] + np.log(3.0), atol=1e-14)
    # order of the parts does not matter; merging in two stages gives the same as in one
    p_o, p_lse = oracle.merge(o[::-1], lse[::-1])
    f_o, f_lse = oracle.merge(o, lse)
    assert np.allclose(p_o, f_o, atol=1e-14) and np.allclose(p_lse, f_lse, atol=1e-14)
    ab_o, ab_lse = oracle.merge(o[:2], lse[:2])
    s_o, s_lse = oracle.merge(np.stack([ab_o.astype(np.float32), o[2]]), np.stack([ab_lse, lse[2]]))
    assert np.abs(s_o - f_o).max() < 1e-6 and np.abs(s_lse - f_lse).max() < 1e-14


# --- the scheduler's work list (oracle/schedule.py) ---

def test_schedule_costs_match_the_mask_counted_pair_by_pair():
    from oracle import schedule
    # partner tiles with at least one allowed (query, key) pair, for every tile of samples around the
    # tile sizes the kernels use (row tiles of 128, partner tiles of 64) and a smaller pair of sizes
    for R, U in ((128, 64), (8, 4)):
        for L in [1, U - 1, U, U + 1, R - 1, R, R + 1, 2 * R, 2 * R + U + 3, 3 * R - 1]:
            for mode in schedule.MODES:
                items = schedule.work_items([0, L], R, U, mode)
                assert [it[3] for it in items] == list(range(-(-L // R)))
                for first, begin, end, t, cost in items:
                    assert (first, begin, end) == (t * R, 0, L)
                    assert cost == schedule.cost_by_brute_force(L, t, R, U, mode), (R, U, L, t, mode)


def test_schedule_of_config_1_by_hand():
    from oracle import schedule
    cu = [0, 16, 53, 117, 246]          # lengths 16, 37, 64, 129
    full = schedule.work_items(cu, 128, 64, "full")
    assert full == [(0, 0, 16, 0, 1), (16, 16, 53, 0, 1), (53, 53, 117, 0, 1), (117, 117, 246, 0, 3), (245, 117, 246, 1, 3)]
    cq = schedule.work_items(cu, 128, 64, "causal_query")
    assert [it[4] for it in cq] == [1, 1, 1, 2, 3]      # rows 0..127 of the last sample see keys 0..127 only
    ck = schedule.work_items(cu, 128, 64, "causal_key")
    assert [it[4] for it in ck] == [1, 1, 1, 3, 1]      # its last key is seen by one query
    # empty samples produce no tiles
    assert schedule.work_items([0, 0, 5, 5], 128, 64, "full") == [(0, 0, 5, 0, 1)]
