"""The library under HIP graph capture (forward + backward recorded once, replayed on new data) and called
from two host threads at once.

The calls allocate nothing and never synchronise, and the scheduler runs on the device inside every
call, so a recorded graph stays valid when the contents of the buffers change, sample boundaries
included (the grids are sized from total_tokens and num_seqs alone).  Every replay is compared with
an eager call on the same inputs, bit for bit (same kernels, same launch shapes), with eager work
and synchronisations between the replays; the second replay, the first on new sample boundaries, is
also checked against the oracle.
"""
import numpy as np
import pytest
import torch

from tests._util import LSE_ABS, assert_close, assert_gradients_close, to_f64

pytestmark = pytest.mark.gpu


def _cu(rng, B, T):
    cuts = np.sort(rng.choice(np.arange(1, T), size=B - 1, replace=False))
    return np.concatenate([[0], cuts, [T]]).astype(np.int32)


@pytest.mark.parametrize("Hq,Hkv,D,causal", [(4, 4, 64, False), (8, 2, 128, True), (2, 2, 80, False)])
def test_recorded_forward_backward_replays_on_new_data(Hq, Hkv, D, causal):
    import oracle
    from paper_2605_08962_amd import binding
    B, T = 7, 1500
    scale = D ** -0.5
    rng = np.random.default_rng(D)
    gen = torch.Generator(device="cuda").manual_seed(D)
    draw = lambda h: torch.randn((T, h, D), device="cuda", generator=gen).to(torch.bfloat16)
    print(f"case Hq={Hq} Hkv={Hkv} D={D} causal={causal} B={B} T={T}", flush=True)

    # static buffers of the recorded graph (kv_splits = 1: the automatic choice is made on the host
    # from the sizes and would be the same on every replay anyway; 1 keeps eager and graph identical)
    q, k, v, do = draw(Hq), draw(Hkv), draw(Hkv), draw(Hq)
    cu = torch.from_numpy(_cu(rng, B, T)).cuda()
    p = binding.make_params(T, B, Hq, Hkv, D, causal, scale, 1)
    wsf = torch.empty(binding.fwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(binding.bwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

    def run(q, k, v, do, cu, o, lse, dq, dk, dv, wsf, wsb):
        binding.varlen_attn_fwd(q, k, v, cu, causal, scale, out=o, lse=lse, workspace=wsf, kv_splits=1)
        binding.varlen_attn_bwd(do, q, k, v, o, lse, cu, causal, scale, dq=dq, dk=dk, dv=dv, workspace=wsb)

    run(q, k, v, do, cu, o, lse, dq, dk, dv, wsf, wsb)   # warm up outside the capture (device check, module load)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(q, k, v, do, cu, o, lse, dq, dk, dv, wsf, wsb)
    torch.cuda.synchronize()

    for replay in range(4):
        # new values and, from the second replay on, new sample boundaries, written into the recorded buffers
        nq, nk, nv, ndo = draw(Hq), draw(Hkv), draw(Hkv), draw(Hq)
        ncu = torch.from_numpy(_cu(rng, B, T)).cuda() if replay else cu.clone()
        q.copy_(nq); k.copy_(nk); v.copy_(nv); do.copy_(ndo); cu.copy_(ncu)
        for t in (o, dq, dk, dv):
            t.fill_(float("nan"))
        lse.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (o, lse, dq, dk, dv)]
        # the same call eagerly, on buffers of its own
        eo, edq, edk, edv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        elsE = torch.empty_like(lse)
        run(nq, nk, nv, ndo, ncu, eo, elsE, edq, edk, edv, torch.empty_like(wsf), torch.empty_like(wsb))
        torch.cuda.synchronize()
        for name, a, b in zip(("O", "LSE", "dQ", "dK", "dV"), got, (eo, elsE, edq, edk, edv)):
            assert torch.equal(a, b), f"replay {replay}: {name} differs from the eager call"
        if replay == 1:
            f32 = lambda t: t.float().cpu().numpy()
            cu_np = ncu.cpu().numpy()
            ro, rlse = oracle.fwd(f32(nq), f32(nk), f32(nv), cu_np, causal, scale)
            assert_close("O", to_f64(got[0]), ro)
            assert float(np.abs(to_f64(got[1]) - rlse).max()) <= LSE_ABS
            assert_gradients_close("replay 1", [to_f64(t) for t in got[2:]], f32(nq), f32(nk), f32(nv), f32(ndo),
                                   cu_np, causal, scale, to_f64(got[0]), allow_output_rounding=True)
        print(f"   replay {replay}: identical to the eager call", flush=True)


def test_two_host_threads_on_two_streams():
    """The library keeps no mutable state between calls (the header says so): two host threads, each with a
    stream, buffers and workspace of its own, call forward + backward at the same time (ctypes drops the GIL
    around the calls) and get what serial calls give, bit for bit."""
    import threading
    from paper_2605_08962_amd import binding
    cases = [(4, 4, 64, False, 11), (8, 2, 128, True, 12)]
    B, T = 9, 2000
    jobs = []
    for Hq, Hkv, D, causal, seed in cases:
        rng = np.random.default_rng(seed)
        gen = torch.Generator(device="cuda").manual_seed(seed)
        draw = lambda h: torch.randn((T, h, D), device="cuda", generator=gen).to(torch.bfloat16)
        jobs.append(dict(q=draw(Hq), k=draw(Hkv), v=draw(Hkv), do=draw(Hq), cu=torch.from_numpy(_cu(rng, B, T)).cuda(),
                         causal=causal, scale=D ** -0.5))

    def run(job, stream, reps):
        out = None
        with torch.cuda.stream(stream):
            for _ in range(reps):
                o, lse = binding.varlen_attn_fwd(job["q"], job["k"], job["v"], job["cu"], job["causal"], job["scale"],
                                                 kv_splits=1)
                dq, dk, dv = binding.varlen_attn_bwd(job["do"], job["q"], job["k"], job["v"], o, lse, job["cu"],
                                                     job["causal"], job["scale"])
                out = (o, lse, dq, dk, dv)
            stream.synchronize()
        return out

    serial = [run(job, torch.cuda.current_stream(), 1) for job in jobs]
    torch.cuda.synchronize()
    results = [None, None]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]

    def worker(i):
        results[i] = run(jobs[i], streams[i], 20)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for i in range(2):
        for name, a, b in zip(("O", "LSE", "dQ", "dK", "dV"), results[i], serial[i]):
            assert torch.equal(a, b), f"thread {i}: {name} differs from the serial call"
