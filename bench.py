#!/usr/bin/env python3
"""Benchmark of the varlen packed attention hot path on one MI355X.

A step is one pass of the whole path on one synthetic batch: forward (scheduler + attention kernel)
followed by backward (two schedulers, dQ with the row statistics, dK/dV).  The default workload is the ViT encoder
layer with dynamic resolution: 64 images of 256..9216 tokens packed non-causally, 16 heads, head_dim
64, bf16, forward + backward.  Inputs are resident in HBM before the timed region starts.

    python bench.py --gpus 1 --steps 20 --warmup 5

prints one JSON line: useful TFLOP/s of the step (forward 4*D*Hq*sum L^2, backward 2.5x that), the
roofline record of the kernel that takes the most time, and the CPU oracle timed on a bounded
sample of the same batch.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "varlen attention useful TFLOP/s fwd/bwd on 1 MI355X; % of bf16 MFMA peak"
PEAK_BF16_TFLOPS = 2500.0  # dense bf16 MFMA, MI355X
CSRC = os.path.join(ROOT, "paper_2605_08962_amd", "csrc")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_kernel.json")
KERNEL_SYMBOL = {"fwd": "fwd_kernel", "dkdv": "dkdv_kernel", "dq": "dq_kernel"}
KERNEL_SYMBOLS_ALL = ("fwd_kernel_lean", "fwd_kernel", "dkdv_kernel", "dq_kernel_direct", "dq_kernel")


def kernel_source_hash():
    """sha256 over the kernel sources (names and contents): ties a counter reading to the code it measured."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(CSRC, name), "rb").read())
    return h.hexdigest()[:16]


def _instance(kernel, head_dim, causal):
    sym = KERNEL_SYMBOL[kernel]
    if kernel == "dq" and head_dim != 80:
        sym = "dq_kernel_direct"        # head_dim 80 alone keeps the phased dQ kernel
    return f"{sym}<{head_dim}, {'true' if causal else 'false'}>"


def measured_traffic(kernel, head_dim, causal):
    """HBM bytes per launch of a kernel instance from the rocprofv3 --pmc readings that
    `bench.py --record-traffic` stored, or None when there is none for the kernel sources as they are now
    (a reading taken on other code says nothing about this code)."""
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None
    if rec.get("kernel_source_sha16") != kernel_source_hash():
        return None
    e = rec.get("kernels", {}).get(_instance(kernel, head_dim, causal))
    return None if e is None else int(e["bytes"])


def record_traffic(paths):
    """Reads the counter_collection.csv files of rocprofv3 --pmc runs of `bench.py --calibrate-copy`
    (FETCH_SIZE in one run, WRITE_SIZE in another), scales each counter by what it read for the 1 GiB
    device copy of the same run, and stores HBM bytes per launch per kernel instance in profiles/, together
    with the hash of the kernel sources they were measured on.  The kernel instances name the workload:
    <64, false> is the ViT batch (configs 2 and 5), <80, false> the long/short mix, <128, true> the LLM batch."""
    import csv
    import glob
    val = {}    # (counter, kernel name) -> [sum of readings (KiB), dispatch ids]
    largest_copy = {}   # counter -> largest single reading of a device-copy dispatch: the 1 GiB one
    for path in paths:
        files = glob.glob(os.path.join(path, "**", "*counter_collection.csv"), recursive=True) if os.path.isdir(path) else [path]
        for f in files:
            for row in csv.DictReader(open(f)):
                acc = val.setdefault((row["Counter_Name"], row["Kernel_Name"]), [0.0, set()])
                acc[0] += float(row["Counter_Value"])
                acc[1].add((f, row["Dispatch_Id"]))
                if "copyBuffer" in row["Kernel_Name"]:
                    c = row["Counter_Name"]
                    largest_copy[c] = max(largest_copy.get(c, 0.0), float(row["Counter_Value"]))
    factor = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        if largest_copy.get(counter, 0.0) < 1024.0:
            raise SystemExit(f"no device-copy kernel with a {counter} reading: profile `bench.py --calibrate-copy`")
        factor[counter] = float(1 << 30) / (largest_copy[counter] * 1024.0)   # true bytes per counted byte
    kernels = {}
    for (counter, name), (v, ids) in val.items():
        for sym in KERNEL_SYMBOLS_ALL:
            # demangled "va::fwd_kernel<64, false>(...)", or, where the profiler's demangler gave up, the
            # mangled "_ZN2va11dkdv_kernelILi64ELb0EEEv..."
            m = re.search(r"va::%s<(\d+), (true|false)>" % sym, name)
            if m:
                inst = f"{sym}<{m.group(1)}, {m.group(2)}>"
            else:
                m = re.search(r"\d+%sILi(\d+)ELb([01])E" % sym, name)
                if not m:
                    continue
                inst = f"{sym}<{m.group(1)}, {'true' if m.group(2) == '1' else 'false'}>"
            if counter not in factor:
                break
            e = kernels.setdefault(inst, {})
            e[counter.lower() + "_kib_per_dispatch"] = round(v / len(ids), 1)
            e["dispatches"] = len(ids)
            break
    for inst, e in kernels.items():
        if "fetch_size_kib_per_dispatch" in e and "write_size_kib_per_dispatch" in e:
            e["bytes"] = int(1024.0 * (e["fetch_size_kib_per_dispatch"] * factor["FETCH_SIZE"] +
                                       e["write_size_kib_per_dispatch"] * factor["WRITE_SIZE"]))
    out = {"kernel_source_sha16": kernel_source_hash(),
           "method": "rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE (KiB per dispatch, mean over the run's dispatches), "
                     "each times the factor that makes the same counter read 1 GiB for the 1 GiB device copy of the "
                     "same run",
           "calibration_true_bytes_per_counted_byte": {k: round(v, 4) for k, v in factor.items()},
           "kernels": {k: kernels[k] for k in sorted(kernels) if "bytes" in kernels[k]}}
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(json.dumps(out, indent=1))


def cpu_baseline(w, budget_flops=8e11):
    """The oracle, as it stands, on whole samples of the batch (shortest first) up to a flop budget."""
    import oracle
    from paper_2605_08962_amd import workloads as W
    order = np.argsort(w.lengths, kind="stable")
    per = 3.5 * 4.0 * w.head_dim * w.num_q_heads * w.lengths[order].astype(np.float64) ** 2
    if w.causal:
        per *= 0.5
    n = max(1, int(np.searchsorted(np.cumsum(per), budget_flops)))
    picks = order[:n]
    cu = w.cu_seqlens.astype(np.int64)
    idx = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in picks])
    lens = w.lengths[picks]
    cu_s = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q, k, v, do = (W.bf16_bits_to_f32(getattr(w, n_)[idx]) for n_ in ("q", "k", "v", "dout"))
    t0 = time.perf_counter()
    oracle.fwd(q, k, v, cu_s, w.causal, w.scale)
    oracle.bwd(q, k, v, do, cu_s, w.causal, w.scale)
    dt = time.perf_counter() - t0
    flops = float(per[:n].sum())
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"forward+backward of the {n} shortest samples ({int(lens.sum())} tokens, "
                      f"{flops:.3e} useful flop) of the same batch, all heads, {dt:.1f} s"}


def report(args, torch, binding, W, to_gpu_bf16):
    """Per-config table: median duration of the whole forward call and of the whole backward call."""
    cases = [("2", W.make(2, with_dout=True)), ("3", W.make(3, with_dout=True)), ("3-short", None),
             ("4", W.make(4, with_dout=True)), ("5", W.make(5, with_dout=True))]
    w3 = cases[1][1]
    short = w3.lengths[w3.lengths < w3.lengths.max()]
    cases[2] = ("3-short", W.make_custom(short, w3.num_q_heads, w3.num_kv_heads, w3.head_dim, w3.causal,
                                         seed=w3.seed, with_dout=True, scale=w3.scale))
    print("| config | mask | B | T | Hq/Hkv | D | pass | median ms | useful TFLOP/s | % of 2.5 PFLOP/s "
          "| shader clock GHz | % of the MFMA peak at that clock | min HBM GB | GB/s at min bytes |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|", flush=True)
    for name, w in cases:
        q, k, v, do = (to_gpu_bf16(getattr(w, n)) for n in ("q", "k", "v", "dout"))
        cu = torch.from_numpy(w.cu_seqlens).cuda()
        T = w.total_tokens
        longest = int(w.lengths.max())      # the max_seqlen a caller of a varlen interface passes along
        p = binding.make_params(T, w.num_seqs, w.num_q_heads, w.num_kv_heads, w.head_dim, w.causal, w.scale,
                                max_seqlen=longest)
        o = torch.empty_like(q)
        lse = torch.empty((w.num_q_heads, T), dtype=torch.float32, device="cuda")
        ws_f = torch.empty(binding.fwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(binding.bwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

        def fwd():
            binding.varlen_attn_fwd(q, k, v, cu, w.causal, w.scale, out=o, lse=lse, workspace=ws_f, max_seqlen=longest)

        def bwd():
            binding.varlen_attn_bwd(do, q, k, v, o, lse, cu, w.causal, w.scale, dq=dq, dk=dk, dv=dv,
                                    workspace=ws_b)

        e = 2 * w.head_dim * T
        qo, kv = e * w.num_q_heads, e * w.num_kv_heads
        stat = 4 * T * w.num_q_heads
        # forward: read Q, K, V, write O, LSE; backward: read Q, K, V, O, dO, LSE, write dQ, dK, dV
        min_bytes = {"fwd": 2 * qo + 2 * kv + stat, "bwd": 4 * qo + 4 * kv + stat}
        for pname, fn, flops in (("fwd", fwd, w.fwd_flops()), ("bwd", bwd, w.bwd_flops())):
            for _ in range(args.warmup):
                fn()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                  for _ in range(args.steps)]
            # the clock the pass's kernels run at during the timed calls: shader cycles over 100 MHz ticks,
            # summed over their workgroups (two clock reads and two atomics per workgroup)
            clocks = torch.zeros(6, dtype=torch.int64, device="cuda")
            binding.profile_clock_probe(clocks)
            for a, b in ev:
                a.record()
                fn()
                b.record()
            torch.cuda.synchronize()
            binding.profile_clock_probe(None)
            ms = float(np.median([a.elapsed_time(b) for a, b in ev]))
            tf = flops / (ms * 1e-3) / 1e12
            ck = clocks.cpu().tolist()
            ghz = 0.1 * sum(ck[1::2]) / max(sum(ck[0::2]), 1)
            peak_at_clock = 256 * 4 * 1024 * ghz * 1e-3   # TFLOP/s: CUs x SIMDs x bf16 flop per cycle x GHz
            print(f"| {name} | {'causal' if w.causal else 'full'} | {w.num_seqs} | {T} | "
                  f"{w.num_q_heads}/{w.num_kv_heads} | {w.head_dim} | {pname} | {ms:.3f} | {tf:.1f} | "
                  f"{100 * tf / PEAK_BF16_TFLOPS:.1f} | {ghz:.2f} | {100 * tf / peak_at_clock:.1f} | "
                  f"{min_bytes[pname] / 1e9:.3f} | {min_bytes[pname] / (ms * 1e-3) / 1e9:.0f} |", flush=True)
        del q, k, v, do, o, lse, ws_f, ws_b, dq, dk, dv
        torch.cuda.empty_cache()


def balance(args, torch, binding, W, ranks=8):
    """What the partitioner buys: time of the slowest rank's share over the mean share time."""
    print("| batch | assignment | predicted max/mean (sum L^2) | measured max ms | mean ms | measured max/mean |")
    print("|---|---|---|---|---|---|", flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    for cfg in (2, 3):
        w = W.make(cfg, lengths_only=True)
        lengths = w.lengths.astype(np.int64)
        n = lengths.size
        assignments = {"as drawn (contiguous chunks)": np.arange(n) * ranks // n}
        for name, method in (("greedy LPT", binding.PARTITION_LPT), ("Karmarkar-Karp", binding.PARTITION_KARMARKAR_KARP)):
            assignments[name + ", any counts"] = binding.balance_partition(lengths, ranks, method)[0]
            if n % ranks == 0:
                assignments[name + f", {n // ranks} per rank"] = binding.balance_partition(
                    lengths, ranks, method, equal_counts=True)[0]
        for name, bin_of in assignments.items():
            cost = np.bincount(bin_of, weights=lengths.astype(np.float64) ** 2, minlength=ranks)
            times = []
            for r in range(ranks):
                Ls = lengths[bin_of == r]
                if Ls.size == 0:
                    times.append(0.0)
                    continue
                T = int(Ls.sum())
                mk = lambda h: torch.randn((T, h, w.head_dim), device="cuda", dtype=torch.bfloat16, generator=gen)
                q, k, v, do = mk(w.num_q_heads), mk(w.num_kv_heads), mk(w.num_kv_heads), mk(w.num_q_heads)
                cu = torch.from_numpy(np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)).cuda()
                o, lse = binding.varlen_attn_fwd(q, k, v, cu, w.causal, w.scale)

                def step():
                    binding.varlen_attn_fwd(q, k, v, cu, w.causal, w.scale, out=o, lse=lse)
                    binding.varlen_attn_bwd(do, q, k, v, o, lse, cu, w.causal, w.scale)
                step()
                ev = []
                for _ in range(max(3, args.steps // 4)):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    step()
                    b.record()
                    ev.append((a, b))
                torch.cuda.synchronize()
                times.append(float(np.median([a.elapsed_time(b) for a, b in ev])))
                del q, k, v, do, o, lse
            times = np.asarray(times)
            print(f"| {w.name} ({n} samples, {ranks} ranks) | {name} | {cost.max() / cost.mean():.3f} | "
                  f"{times.max():.3f} | {times.mean():.3f} | {times.max() / times.mean():.3f} |", flush=True)
        torch.cuda.empty_cache()


def lssp(args, torch, binding, W, ranks=8, model_heads=16):
    """Section 4.1.1, long-short sequence parallelism, emulated on one GPU (no all-to-all): the time of
    the attention layers of the slowest rank, as a function of the length threshold."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4321)
    w = W.make(3, lengths_only=True)
    rng = np.random.Generator(np.random.PCG64(2003))
    mixes = {"long_short_mix_d80 (1 x 65536 + 256 x 64..1024)": w.lengths.astype(np.int64),
             "log-uniform 256..32768, 96 samples": np.floor(np.exp(rng.uniform(np.log(256), np.log(32768), 96))).astype(np.int64)}

    def run(Ls, heads):
        if Ls.size == 0:
            return 0.0
        T = int(Ls.sum())
        mk = lambda: torch.randn((T, heads, w.head_dim), device="cuda", dtype=torch.bfloat16, generator=gen)
        q, k, v, do = mk(), mk(), mk(), mk()
        cu = torch.from_numpy(np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)).cuda()
        o, lse = binding.varlen_attn_fwd(q, k, v, cu, False, w.scale)

        def step():
            binding.varlen_attn_fwd(q, k, v, cu, False, w.scale, out=o, lse=lse)
            binding.varlen_attn_bwd(do, q, k, v, o, lse, cu, False, w.scale)
        step()
        ev = []
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            step()
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in ev]))

    print("| microbatch of the node | threshold | samples in SP state | slowest rank, DP state ms | SP state ms | total ms |")
    print("|---|---|---|---|---|---|", flush=True)
    for name, lengths in mixes.items():
        for eta in (0, 1024, 2048, 4096, 8192, 16384, 1 << 30):
            long_ = lengths[lengths > eta]
            short = lengths[lengths <= eta]
            t_dp = 0.0
            if short.size:
                # data-parallel state: whole samples, balanced over the ranks; the slowest rank counts
                bin_of, cost = binding.balance_partition(short, ranks, binding.PARTITION_KARMARKAR_KARP)
                t_dp = run(short[bin_of == int(np.argmax(cost))], model_heads)
            # sequence-parallel state: every rank holds all tokens of the long samples for its heads
            t_sp = run(long_, model_heads // ranks)
            label = "all SP" if eta == 0 else ("all DP" if eta == 1 << 30 else str(eta))
            print(f"| {name} | {label} | {long_.size} of {lengths.size} | {t_dp:.3f} | {t_sp:.3f} | {t_dp + t_sp:.3f} |",
                  flush=True)
        torch.cuda.empty_cache()


def short_regime(args, torch, binding):
    """The short-sequence regime: equal-length samples of 64..2048 tokens (about 84k tokens per batch, 16
    heads), forward and backward, as HBM GB/s at the minimum bytes (every input read once, every output
    written once) next to useful TFLOP/s.  Median of HIP events over args.steps calls."""
    print("| D | L | samples | pass | us | GB/s at min bytes | % of 8 TB/s | useful TFLOP/s |")
    print("|---|---|---|---|---|---|---|---|")
    H = 16
    for D in (64, 80, 128):
        for L in (64, 128, 256, 512, 1024, 2048):
            B = 84000 // L
            T = B * L
            g = torch.Generator(device="cuda"); g.manual_seed(D + L)
            q, k, v, do = (torch.randn((T, H, D), device="cuda", dtype=torch.bfloat16, generator=g) for _ in range(4))
            cu = torch.arange(0, T + 1, L, dtype=torch.int32, device="cuda")
            scale = D ** -0.5
            p = binding.make_params(T, B, H, H, D, False, scale, max_seqlen=L)
            ws_f = torch.empty(binding.fwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
            ws_b = torch.empty(binding.bwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
            o = torch.empty_like(q)
            lse = torch.empty((H, T), dtype=torch.float32, device="cuda")
            dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
            # (a caller of a varlen interface knows its longest sample; the hint selects the lean forward)
            fns = (("fwd", lambda: binding.varlen_attn_fwd(q, k, v, cu, False, scale, out=o, lse=lse, workspace=ws_f,
                                                           max_seqlen=L),
                    2 * D * T * 4 * H + 4 * T * H, 1.0),
                   ("bwd", lambda: binding.varlen_attn_bwd(do, q, k, v, o, lse, cu, False, scale, dq=dq, dk=dk, dv=dv,
                                                           workspace=ws_b),
                    2 * D * T * 8 * H + 4 * T * H, 2.5))
            for name, fn, nbytes, mult in fns:
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                ts = []
                for _ in range(args.steps):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(); fn(); e1.record(); torch.cuda.synchronize()
                    ts.append(e0.elapsed_time(e1))
                ms = float(np.median(ts))
                flops = mult * 4.0 * D * H * B * L * L
                print(f"| {D} | {L} | {B} | {name} | {ms * 1e3:.0f} | {nbytes / ms / 1e6:.0f} | "
                      f"{100 * nbytes / ms / 1e6 / 8000:.0f} | {flops / ms / 1e9:.0f} |", flush=True)


def small_launch(args, torch, binding, W):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)

    def timed(fn, n=max(5, 20)):
        fn()
        ev = []
        for _ in range(n):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in ev]))

    print("| one sample of | heads (q/kv) | D | mask | workgroups unsplit | unsplit ms | automatic ms | speed-up |")
    print("|---|---|---|---|---|---|---|---|", flush=True)
    for L, Hq, Hkv, D, causal in ((2048, 2, 2, 128, True), (4096, 2, 2, 128, True), (8192, 2, 2, 80, False),
                                  (8192, 4, 1, 128, True), (16384, 2, 2, 80, False), (32768, 2, 2, 80, False),
                                  (65536, 2, 2, 80, False)):
        mk = lambda h: torch.randn((L, h, D), device="cuda", dtype=torch.bfloat16, generator=gen)
        q, k, v = mk(Hq), mk(Hkv), mk(Hkv)
        cu = torch.tensor([0, L], dtype=torch.int32, device="cuda")
        scale = D ** -0.5
        o = torch.empty_like(q)
        lse = torch.empty((Hq, L), dtype=torch.float32, device="cuda")
        res = []
        for splits in (1, 0):
            p = binding.make_params(L, 1, Hq, Hkv, D, causal, scale, splits)
            ws = torch.empty(binding.fwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
            res.append(timed(lambda: binding.varlen_attn_fwd(q, k, v, cu, causal, scale, out=o, lse=lse,
                                                             workspace=ws, kv_splits=splits)))
        print(f"| {L} tokens | {Hq}/{Hkv} | {D} | {'causal' if causal else 'full'} | {(L // 128) * Hq} | "
              f"{res[0]:.3f} | {res[1]:.3f} | {res[0] / res[1]:.2f}x |", flush=True)
    print()
    print("| merge of | tokens x heads x D | algorithmic bytes | ms | GB/s | fraction of 8 TB/s |")
    print("|---|---|---|---|---|---|", flush=True)
    for P, T, H, D in ((2, 178572, 16, 64), (4, 178572, 16, 64), (2, 32768, 32, 128), (8, 65536, 2, 80)):
        parts = torch.randn((P, T, H, D), device="cuda", dtype=torch.bfloat16, generator=gen)
        lses = torch.randn((P, H, T), device="cuda", dtype=torch.float32, generator=gen)
        o = torch.empty((T, H, D), device="cuda", dtype=torch.bfloat16)
        lse = torch.empty((H, T), device="cuda", dtype=torch.float32)
        ms = timed(lambda: binding.varlen_attn_merge(parts, lses, out=o, lse=lse))
        nbytes = (P + 1) * T * H * (2 * D + 4)  # every part read once, the result written once
        print(f"| {P} parts | {T} x {H} x {D} | {nbytes / 1e9:.3f} GB | {ms:.4f} | {nbytes / ms / 1e6:.0f} | "
              f"{nbytes / ms / 1e6 / 8000:.3f} |", flush=True)


def measure(args, torch, binding, to_gpu_bf16, w, with_bwd, steps, warmup, settle_s):
    """W warm-up steps, then further untimed steps until settle_s seconds of continuous load have passed (the
    chip lowers its clock under matrix-core load; a timed region that starts cold flatters it), then exactly
    `steps` timed steps between two synchronisations.  Per-kernel durations from HIP events the library records
    around each launch on the caller's stream."""
    q, k, v, do = (to_gpu_bf16(getattr(w, n)) for n in ("q", "k", "v", "dout"))
    cu = torch.from_numpy(w.cu_seqlens).cuda()
    T = w.total_tokens
    p = binding.make_params(T, w.num_seqs, w.num_q_heads, w.num_kv_heads, w.head_dim, w.causal, w.scale)
    o = torch.empty_like(q)
    lse = torch.empty((w.num_q_heads, T), dtype=torch.float32, device="cuda")
    ws_f = torch.empty(binding.fwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(binding.bwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

    def step():
        binding.varlen_attn_fwd(q, k, v, cu, w.causal, w.scale, out=o, lse=lse, workspace=ws_f)
        if with_bwd:
            binding.varlen_attn_bwd(do, q, k, v, o, lse, cu, w.causal, w.scale, dq=dq, dk=dk, dv=dv,
                                    workspace=ws_b)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < settle_s:
        for _ in range(4):
            step()
        torch.cuda.synchronize()
    clocks = torch.zeros(6, dtype=torch.int64, device="cuda")
    binding.profile_clock_probe(clocks)
    binding.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    binding.profile_enable(False)
    binding.profile_clock_probe(None)
    prof = binding.profile_read()
    ck = clocks.cpu().tolist()

    fwd_flops = w.fwd_flops()
    step_flops = fwd_flops * (3.5 if with_bwd else 1.0)
    ms = dt * 1e3 / steps
    value = step_flops / (ms * 1e-3) / 1e12
    # algorithmic flops per launch: forward = F; dK/dV kernel = S, dP, dV, dK = 4 of the backward's 5
    # GEMMs = 2.0 F; dQ kernel = the dQ GEMM = 0.5 F (its recomputation of S and dP is not counted).
    algo = {"fwd": fwd_flops, "dkdv": 2.0 * fwd_flops, "dq": 0.5 * fwd_flops}
    kern = {n: (prof[n][0] / prof[n][1]) for n in algo if prof[n][1] > 0}
    dom = max(kern, key=lambda n: kern[n] * prof[n][1])
    achieved = algo[dom] / (kern[dom] * 1e-3) / 1e12
    res = {
        "passes": "fwd+bwd" if with_bwd else "fwd", "ms_per_step": round(ms, 4), "tflops": round(value, 2),
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "kernels_ms": {n: round(prof[n][0] / max(prof[n][1], 1), 4) for n in prof if prof[n][1] > 0},
        "fwd_tflops": round(fwd_flops / (kern["fwd"] * 1e-3) / 1e12, 2),
        "roofline": {"kernel": _instance(dom, w.head_dim, w.causal), "bound": "mfma", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": measured_traffic(dom, w.head_dim, w.causal)},
        # average shader clock each compute kernel ran at (cycle counter over the 100 MHz constant clock)
        "shader_clock_ghz": {n: round(0.1 * ck[2 * i + 1] / ck[2 * i], 3)
                             for i, n in enumerate(("fwd", "dkdv", "dq")) if ck[2 * i] > 0},
    }
    if with_bwd:
        bwd_ms = sum(kern[n] for n in ("dkdv", "dq"))
        res["bwd_tflops"] = round(2.5 * fwd_flops / (bwd_ms * 1e-3) / 1e12, 2)
    del q, k, v, do, o, lse, ws_f, ws_b, dq, dk, dv
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, choices=[2, 3, 4, 5],
                    help="5 (default): ViT batch forward+backward; 2, 3, 4: forward only on that config")
    ap.add_argument("--passes", choices=["fwd", "fwd+bwd"], default=None,
                    help="override what a step is (default: fwd+bwd for config 5, fwd otherwise)")
    ap.add_argument("--report", action="store_true",
                    help="instead of the one JSON line: time forward and backward separately on configs "
                         "2, 3, 3 without its long sample, 4 and 5 (median over --steps calls, HIP events "
                         "around the whole library call) and print a markdown table")
    ap.add_argument("--balance", action="store_true",
                    help="instead of the one JSON line: split the ViT batch's 64 images (and the long/short "
                         "mix) over 8 ranks as drawn, by greedy LPT and by Karmarkar-Karp differencing "
                         "(library's host-side partitioner, cost = L^2), run forward+backward on every "
                         "rank's share on this GPU and print max / mean share time as a markdown table")
    ap.add_argument("--lssp", action="store_true",
                    help="instead of the one JSON line: long-short sequence parallelism as ONE rank of an 8-rank "
                         "node executes it: samples longer than a threshold run in the sequence-parallel state "
                         "(full length, 1/8 of the heads), the others in the data-parallel state (this rank's "
                         "balanced share, all heads); sweeps the threshold and prints a markdown table")
    ap.add_argument("--small-launch", action="store_true",
                    help="instead of the one JSON line: forward on launches too small to fill the GPU with and "
                         "without splitting each query tile's keys over several workgroups, and the merge "
                         "primitive's HBM rate; prints markdown tables")
    ap.add_argument("--short-regime", action="store_true",
                    help="equal-length samples of 64..2048 tokens: HBM GB/s at the minimum bytes and useful "
                         "TFLOP/s, forward and backward; prints a markdown table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="leave the per-config list (configs 2, 3, 4) out of the JSON line")
    ap.add_argument("--settle-s", type=float, default=1.0,
                    help="seconds of untimed steps after the warm-up, so that the timed steps run at the clock "
                         "the chip settles at under sustained load (default 1.0)")
    ap.add_argument("--record-traffic", nargs="+", metavar="DIR",
                    help="no GPU work: read rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE output directories of "
                         "`bench.py --calibrate-copy` runs and store HBM bytes per launch per kernel in "
                         "profiles/hbm_traffic_per_kernel.json, which later runs report as roofline.traffic")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy, as the known-size reference that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.record_traffic:
        record_traffic(args.record_traffic)
        return
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on one GPU only (no sharding, no collectives); "
                         "use --gpus 1\n")
        sys.exit(2)

    import torch
    from paper_2605_08962_amd import binding, workloads as W
    from tests._util import to_gpu_bf16
    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(1)
    binding.load()
    if args.report:
        report(args, torch, binding, W, to_gpu_bf16)
        return
    if args.balance:
        balance(args, torch, binding, W)
        return
    if args.lssp:
        lssp(args, torch, binding, W)
        return
    if args.small_launch:
        small_launch(args, torch, binding, W)
        return
    if args.short_regime:
        short_regime(args, torch, binding)
        return

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.zero_()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    with_bwd = (args.passes == "fwd+bwd") if args.passes else args.config == 5
    w = W.make(args.config, with_dout=True)
    head = measure(args, torch, binding, to_gpu_bf16, w, with_bwd, args.steps, args.warmup, args.settle_s)
    out = {
        "metric": METRIC, "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "num_seqs": w.num_seqs, "total_tokens": w.total_tokens,
                   "q_heads": w.num_q_heads, "kv_heads": w.num_kv_heads, "head_dim": w.head_dim,
                   "causal": w.causal, "passes": head["passes"], "seed": w.seed},
        "pct_of_bf16_mfma_peak": head["pct_of_bf16_mfma_peak"],
        "settle_s": args.settle_s,
        "kernels_ms": head["kernels_ms"], "fwd_tflops": head["fwd_tflops"],
        "roofline": head["roofline"], "shader_clock_ghz": head["shader_clock_ghz"],
    }
    if "bwd_tflops" in head:
        out["bwd_tflops"] = head["bwd_tflops"]
    # the other long-sequence configurations, each as a forward-only step and as a forward+backward step
    if args.config == 5 and args.passes is None and not args.headline_only:
        out["configs"] = []
        for cfg in (2, 3, 4):
            wc = W.make(cfg, with_dout=True)
            for wb in (False, True):
                if cfg == 2 and wb:
                    continue        # config 2 forward+backward IS the headline step (config 5)
                r = measure(args, torch, binding, to_gpu_bf16, wc, wb, args.steps, args.warmup, min(args.settle_s, 0.5))
                r.update({"workload": wc.name, "head_dim": wc.head_dim, "causal": wc.causal,
                          "total_tokens": wc.total_tokens, "num_seqs": wc.num_seqs})
                out["configs"].append(r)
            del wc
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
