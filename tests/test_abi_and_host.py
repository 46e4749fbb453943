"""CPU-only checks of the C-ABI library: it loads, exports what include/varlen_attn.h declares,
validates host-visible arguments before touching a device, and sizes its work lists safely.
No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_08962_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2605_08962_amd import binding
    return binding.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "varlen_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(varlen_attn_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"varlen_attn_fwd", "varlen_attn_bwd", "varlen_attn_fwd_workspace_bytes",
            "varlen_attn_bwd_workspace_bytes", "varlen_attn_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def test_params_struct_matches_header():
    from paper_2605_08962_amd import binding
    assert ctypes.sizeof(binding.Params) == 36
    assert [f[0] for f in binding.Params._fields_] == [
        "total_tokens", "num_seqs", "num_q_heads", "num_kv_heads", "head_dim", "causal", "softmax_scale", "max_seqlen",
        "kv_splits"]
    # the header's struct, member by member, in the same order
    text = open(os.path.join(ROOT, "include", "varlen_attn.h")).read()
    body = re.sub(r"/\*.*?\*/", "", text[text.index("typedef struct {"):text.index("} varlen_attn_params;")], flags=re.S)
    assert re.findall(r"(?:int32_t|float)\s+(\w+);", body) == [f[0] for f in binding.Params._fields_]


def test_status_strings(lib):
    from paper_2605_08962_amd import binding
    seen = {binding.status_string(i) for i in range(10)}
    assert len(seen) == 10 and binding.status_string(0) == "ok"
    assert binding.status_string(99) == "unknown status"


def _call_fwd(lib, p, q=16, k=16, v=16, cu=16, o=16, lse=16, ws=16, ws_bytes=1 << 30):
    # fake, never dereferenced pointers: every case below must be rejected on the host
    return lib.varlen_attn_fwd(ctypes.byref(p), q, k, v, cu, o, lse, ws, ws_bytes, None)


def test_host_side_validation_needs_no_gpu(lib):
    from paper_2605_08962_amd import binding
    mk = binding.make_params
    assert _call_fwd(lib, mk(0, 0, 2, 2, 64, 0, 0.125)) == 0            # empty: OK, nothing launched
    assert _call_fwd(lib, mk(0, 3, 2, 2, 64, 0, 0.125)) == 0
    assert _call_fwd(lib, mk(-1, 1, 2, 2, 64, 0, 0.125)) == 2
    assert _call_fwd(lib, mk(8, 1, 3, 2, 64, 0, 0.125)) == 2            # Hq % Hkv
    assert _call_fwd(lib, mk(8, 1, 2, 0, 64, 0, 0.125)) == 2
    p = mk(8, 1, 2, 2, 64, 0, 0.125); p.causal = 2
    assert _call_fwd(lib, p) == 2
    for bad in (-1, 9):
        p = mk(8, 1, 2, 2, 64, 0, 0.125); p.kv_splits = bad
        assert _call_fwd(lib, p) == 2
    p = mk(8, 1, 2, 2, 64, 0, 0.125); p.max_seqlen = -1
    assert _call_fwd(lib, p) == 2
    for d in (0, 32, 48, 72, 256):
        assert _call_fwd(lib, mk(8, 1, 2, 2, d, 0, 0.125)) == 3
    for s in (float("nan"), float("inf"), -0.5):
        assert _call_fwd(lib, mk(8, 1, 2, 2, 64, 0, s)) == 5
    ok = mk(8, 1, 2, 2, 64, 0, 0.125)
    assert _call_fwd(lib, ok, q=None) == 1
    assert _call_fwd(lib, ok, lse=None) == 1
    assert _call_fwd(lib, ok, k=24) == 7                                 # not 16-byte aligned
    assert _call_fwd(lib, ok, ws_bytes=8) == 4
    assert lib.varlen_attn_fwd(None, 16, 16, 16, 16, 16, 16, 16, 64, None) == 1
    # backward: same order of checks
    args = [16] * 11
    assert lib.varlen_attn_bwd(ctypes.byref(mk(8, 1, 2, 2, 64, 0, -1.0)), *args, 1 << 30, None) == 5
    assert lib.varlen_attn_bwd(ctypes.byref(ok), *args, 8, None) == 4
    args[9] = None
    assert lib.varlen_attn_bwd(ctypes.byref(ok), *args, 1 << 30, None) == 1
    assert lib.varlen_attn_bwd(ctypes.byref(mk(0, 0, 2, 2, 64, 0, 0.125)), *([None] * 11), 0, None) == 0


def test_cu_seqlens_check_validates_its_arguments_on_the_host(lib):
    from paper_2605_08962_amd import binding
    mk = binding.make_params
    call = lambda p, cu=16, ws=16, n=16: lib.varlen_attn_check_cu_seqlens(ctypes.byref(p), cu, ws, n, None)
    assert call(mk(0, 0, 1, 1, 64, 0, 1.0), None, None, 0) == 0          # no samples, no tokens: fine, no launch
    assert call(mk(5, 0, 1, 1, 64, 0, 1.0), None, None, 0) == 8          # tokens that belong to no sample
    ok = mk(8, 2, 1, 1, 64, 0, 1.0)
    assert call(ok, cu=None) == 1 and call(ok, ws=None) == 1
    assert call(ok, cu=18) == 7 and call(ok, ws=24) == 7
    assert call(ok, n=8) == 4
    assert call(mk(-1, 2, 1, 1, 64, 0, 1.0)) == 2


def test_workspace_and_work_list_bounds():
    from paper_2605_08962_amd import binding
    rng = np.random.default_rng(0)
    for trial in range(50):
        B = int(rng.integers(1, 300))
        L = rng.integers(0, 700, size=B)
        if trial % 5 == 0:
            L[rng.integers(0, B)] = 70000
        T = int(L.sum())
        p = binding.make_params(T, B, 8, 2, 128, trial % 2, 0.1)
        for which, rows in ((0, 128), (1, 128), (2, 128)):
            need = int(np.sum((L + rows - 1) // rows))
            cap = binding.max_work_items(p, which)
            assert need <= cap <= T // rows + B
        fw, bw = binding.fwd_workspace_bytes(p), binding.bwd_workspace_bytes(p)
        assert fw >= 64 + 4 * (B + 1) + 16 * binding.max_work_items(p, 0) and fw % 256 == 0
        assert bw >= 4 * T * 8 + fw
    assert binding.fwd_workspace_bytes(binding.make_params(8, 1, 2, 2, 72, 0, 0.1)) == 0


def _host_schedule(binding, lib, cu, T, causal, which):
    cu = np.ascontiguousarray(cu, dtype=np.int32)
    p = binding.make_params(T, cu.size - 1, 1, 1, 64, causal, 0.125)
    cap = binding.max_work_items(p, which)
    items = np.full((cap + 1, 4), -7, dtype=np.int32)          # one guard row behind the list
    lib.varlen_attn_schedule_host.restype = ctypes.c_int64
    lib.varlen_attn_schedule_host.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_int64]
    n = lib.varlen_attn_schedule_host(ctypes.byref(p), which, cu.ctypes.data, items.ctypes.data, cap)
    assert 0 <= n <= cap and (items[n:] == -7).all()
    return items[:n]


def test_host_schedule_matches_the_oracle(lib):
    """The work list arithmetic the device scheduler shares with the host (sample clamp, tile cost, counting
    sort by cost) against oracle/schedule.py: same tiles, each once, heaviest first."""
    from oracle import schedule
    from paper_2605_08962_amd import binding
    rng = np.random.default_rng(5)
    cases = [np.array([16, 37, 64, 129]), np.array([0, 300, 0, 0, 129, 1, 0, 128, 127, 0]), np.array([5000]),
             W.make(3, lengths_only=True).lengths, W.make(4, lengths_only=True).lengths, rng.integers(0, 200, size=700)]
    for lengths in cases:
        cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
        for causal in (0, 1):
            for which, mode in ((0, "causal_query" if causal else "full"), (1, "causal_key" if causal else "full"),
                                (2, "causal_query" if causal else "full")):
                got = _host_schedule(binding, lib, cu, int(cu[-1]), causal, which)
                want = schedule.work_items(cu, 128, 64, mode)
                cost_of = {it[:4]: it[4] for it in want}
                keys = [tuple(int(x) for x in row) for row in got]
                assert len(keys) == len(want) and set(keys) == set(cost_of)
                assert np.all(np.diff([cost_of[k_] for k_ in keys]) <= 0)


def test_schedule_of_a_malformed_batch_stays_inside_the_tensors(lib):
    """cu_seqlens lives on the device and is not validated.  The scheduler clamps each sample into
    [0, T) and the list to the room the workspace has, so that a malformed array cannot make the
    attention kernels address memory outside the tensors (checked here on the host-side twin of the
    device arithmetic; no GPU is given a malformed batch)."""
    from paper_2605_08962_amd import binding
    T = 1000
    bad = [[0, 400, 2000], [0, -5, 1000], [0, 700, 300, 1000], [0, 1000, 0, 1000, 0, 1000, 0, 1000], [5, 9, 1 << 30],
           [0, -(1 << 31), (1 << 31) - 1], [0, 1000, 1000, 1000]]
    for cu in bad:
        for causal in (0, 1):
            for which in (0, 1, 2):
                items = _host_schedule(binding, lib, np.array(cu, dtype=np.int64).astype(np.int32), T, causal, which)
                first, begin, end, tile = items.T
                assert (0 <= begin).all() and (begin <= first).all() and (first < end).all() and (end <= T).all()
                assert (first == begin + 128 * tile).all()
    # bad arguments: no list
    p = binding.make_params(T, 2, 1, 1, 64, 0, 0.125)
    buf = np.zeros((64, 4), dtype=np.int32)
    cu = np.array([0, 500, 1000], dtype=np.int32)
    assert lib.varlen_attn_schedule_host(ctypes.byref(p), 3, cu.ctypes.data, buf.ctypes.data, 64) == -1
    assert lib.varlen_attn_schedule_host(ctypes.byref(p), 0, cu.ctypes.data, buf.ctypes.data, 2) == -1
    assert lib.varlen_attn_schedule_host(ctypes.byref(p), 0, None, buf.ctypes.data, 64) == -1


def test_workload_recipes():
    w1 = W.make(1, lengths_only=True)
    assert list(w1.lengths) == [16, 37, 64, 129] and w1.fwd_flops() == 4 * 64 * 2 * 22362
    w2 = W.make(2, lengths_only=True)
    assert w2.num_seqs == 64 and w2.lengths.min() >= 256 and w2.lengths.max() <= 9216
    assert all(int(n) % 4 == 0 for n in w2.lengths)
    for pos in ("first", "middle", "last"):
        w3 = W.make(3, lengths_only=True, long_pos=pos)
        assert w3.num_seqs == 257 and sorted(w3.lengths)[-1] == 65536 and sorted(w3.lengths)[-2] <= 1024
        assert w3.lengths.min() >= 64
        assert int(np.argmax(w3.lengths)) == {"first": 0, "middle": 128, "last": 256}[pos]
    w4 = W.make(4, lengths_only=True)
    assert w4.total_tokens == 32768 and w4.lengths.min() >= 128 and w4.lengths.max() <= 16384 + 127
    assert (w4.num_q_heads, w4.num_kv_heads, w4.head_dim, w4.causal) == (32, 8, 128, True)
    w5 = W.make(5, lengths_only=True)
    assert np.array_equal(w5.lengths, w2.lengths)


def test_bf16_rounding_matches_torch():
    import torch
    x = np.random.default_rng(1).standard_normal(100000).astype(np.float32) * 3
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]   # ties: to even
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    assert np.array_equal(W.bf16_bits_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_clock_probe_rejects_a_misaligned_pointer(lib):
    assert lib.varlen_attn_profile_clock_probe(ctypes.c_void_p(12)) == 7
    assert lib.varlen_attn_profile_clock_probe(None) == 0


def test_lds_tile_layouts_are_consistent_and_bank_conflict_free(tmp_path):
    # compiles tests/lds_layout_check.hip (host code only runs) against csrc/va_device.h: every
    # head_dim's layout is a bijection whose row-wise and transposing reads cover the banks once
    import shutil
    import subprocess
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not on PATH")
    exe = tmp_path / "lds_layout_check"
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lds_layout_check.hip")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17", src, "-o", str(exe)], check=True,
                   capture_output=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and "lds layouts ok" in r.stdout, r.stdout[-2000:]
