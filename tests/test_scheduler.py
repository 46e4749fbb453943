"""GPU parity of the length-aware tile scheduler (the device-side work lists) with oracle/schedule.py.

Integer work: the lists must hold exactly the oracle's tiles, each once, heaviest first.  The order
of tiles of equal cost is open (the kernel scatters them with atomics), so the comparison is on the
set of tiles and on the sequence of costs.  The lists are read out of the workspace that a forward /
backward call leaves behind; the layout parsed here is the library's internal one (csrc/va_internal.h):
16 int32 of header ([0] number of tiles, [1] work order: 128 = chunked per XCD when a sample of 1024
tokens or more is present, else 1), tile offsets per sample (B + 1 int32), then, 16-byte aligned, one
int4 {first row, sample begin, sample end, tile index} per tile with room for T / tile_rows + B of
them, the whole rounded up to 256 bytes.  The backward holds two lists back to back (key tiles for
dK/dV, then query tiles for dQ).
"""
import numpy as np
import pytest
import torch

from paper_2605_08962_amd import workloads as W

pytestmark = pytest.mark.gpu

ROW_TILE, PARTNER_TILE = 128, 64      # all three kernels: tiles of 128 rows walking partner tiles of 64


def _list_bytes(T, B):
    items_ofs = (64 + 4 * (B + 1) + 15) // 16 * 16
    return items_ofs, (items_ofs + 16 * (T // ROW_TILE + B) + 255) // 256 * 256


def _check_list(ws, offset, cu, mode):
    from oracle import schedule
    B, T = len(cu) - 1, int(cu[-1])
    items_ofs, size = _list_bytes(T, B)
    words = ws[offset:offset + size].view(np.int32)
    want = schedule.work_items(cu, ROW_TILE, PARTNER_TILE, mode)
    n = int(words[0])
    assert n == len(want)
    lengths = np.diff(cu)
    assert int(words[1]) == (128 if lengths.max() >= 1024 else 1)
    tiles_per_sample = -(-lengths // ROW_TILE)
    assert np.array_equal(words[16:16 + B + 1], np.concatenate([[0], np.cumsum(tiles_per_sample)]))
    got = words[items_ofs // 4: items_ofs // 4 + 4 * n].reshape(n, 4)
    cost_of = {it[:4]: it[4] for it in want}
    got_keys = [tuple(int(x) for x in row) for row in got]
    assert len(set(got_keys)) == n and set(got_keys) == set(cost_of), "the list must hold every tile exactly once"
    costs = np.array([cost_of[key] for key in got_keys])
    assert np.all(np.diff(costs) <= 0), "heaviest tiles first"
    return offset + size


def _lengths_cases():
    rng = np.random.default_rng(77)
    yield "config 1", np.array([16, 37, 64, 129])
    yield "long/short mix", W.make(3, lengths_only=True).lengths
    yield "llm", W.make(4, lengths_only=True).lengths
    yield "empty samples between", np.array([0, 300, 0, 0, 129, 1, 0, 128, 127, 0])
    yield "3000 samples (several passes of the 1024-thread scan)", rng.integers(0, 200, size=3000)
    yield "one sample", np.array([5000])
    yield "9000 samples (tile offsets in LDS, sample bounds from cu_seqlens)", rng.integers(0, 150, size=9000)
    yield "25000 samples (searches through the workspace)", rng.integers(0, 60, size=25000)


@pytest.mark.parametrize("causal", [False, True])
def test_work_lists_match_the_oracle(causal):
    from paper_2605_08962_amd import binding
    for name, lengths in _lengths_cases():
        cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
        B, T = len(lengths), int(cu[-1])
        print(f"case {name}: B={B} T={T} causal={causal}", flush=True)
        gen = torch.Generator(device="cuda").manual_seed(B)
        q, k, v, do = (torch.randn((T, 1, 64), device="cuda", generator=gen).to(torch.bfloat16) for _ in range(4))
        cu_d = torch.from_numpy(cu).cuda()
        p = binding.make_params(T, B, 1, 1, 64, causal, 0.125, 1)
        wsf = torch.zeros(binding.fwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        wsb = torch.zeros(binding.bwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        o, lse = binding.varlen_attn_fwd(q, k, v, cu_d, causal, 0.125, workspace=wsf, kv_splits=1)
        binding.varlen_attn_bwd(do, q, k, v, o, lse, cu_d, causal, 0.125, workspace=wsb)
        torch.cuda.synchronize()
        _check_list(wsf.cpu().numpy(), 0, cu, "causal_query" if causal else "full")
        wsb_h = wsb.cpu().numpy()
        nxt = _check_list(wsb_h, 0, cu, "causal_key" if causal else "full")
        _check_list(wsb_h, nxt, cu, "causal_query" if causal else "full")
