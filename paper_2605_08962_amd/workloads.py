"""Seeded synthetic inputs for varlen packed attention.

This module serves both the HIP path's tests/benchmark and the CPU oracle's tests.  It
holds no attention arithmetic: only sequence-length recipes and i.i.d. N(0,1) tensors
rounded to bf16.  The recipes stand in for the paper's workloads (Section 2.2: ViT
tokens from 14x14-pixel patches at dynamic resolution, mean encoded lengths of a few
hundred to a few thousand tokens with rare very long samples; Section 4.1.1: a
microbatch that mixes one long sample with many short ones; Table 1: packed LLM
sequences of 8K-32K tokens).  The datasets themselves are not used.

Draw order for every workload: lengths, then Q, K, V, then dO, all from one
numpy PCG64 generator seeded with the workload's seed.
"""
from dataclasses import dataclass, field
import math

import numpy as np

CONFIG_NAMES = {
    1: "tiny_noncausal_d64",
    2: "vit_dynamic_resolution_d64",
    3: "long_short_mix_d80",
    4: "llm_causal_gqa_d128",
    5: "vit_dynamic_resolution_d64_fwd_bwd",
}


def f32_to_bf16_bits(x):
    """Round float32 to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits):
    """Exact float32 value of bf16 bit patterns."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    name: str
    lengths: np.ndarray            # int64 [B]
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    causal: bool
    scale: float
    seed: int
    q: np.ndarray = None           # uint16 bf16 bits [T, Hq, D]
    k: np.ndarray = None           # uint16 [T, Hkv, D]
    v: np.ndarray = None           # uint16 [T, Hkv, D]
    dout: np.ndarray = None        # uint16 [T, Hq, D] or None
    extra: dict = field(default_factory=dict)

    @property
    def cu_seqlens(self):
        cu = np.zeros(len(self.lengths) + 1, dtype=np.int64)
        np.cumsum(self.lengths, out=cu[1:])
        assert cu[-1] < 2 ** 31
        return cu.astype(np.int32)

    @property
    def total_tokens(self):
        return int(np.sum(self.lengths))

    @property
    def num_seqs(self):
        return len(self.lengths)

    def f32(self, name):
        return bf16_bits_to_f32(getattr(self, name))

    def fwd_flops(self):
        """Useful forward flops: 4*D*Hq*sum(L^2), or 4*D*Hq*sum(L(L+1)/2) under the causal mask."""
        L = self.lengths.astype(np.float64)
        pairs = np.sum(L * (L + 1) / 2) if self.causal else np.sum(L * L)
        return 4.0 * self.head_dim * self.num_q_heads * float(pairs)

    def bwd_flops(self):
        return 2.5 * self.fwd_flops()

    def fwd_min_bytes(self):
        """Q, K, V read once, O and LSE written once, cu_seqlens read."""
        T, D = self.total_tokens, self.head_dim
        return 2 * D * T * (2 * self.num_q_heads + 2 * self.num_kv_heads) + 4 * T * self.num_q_heads + 4 * (self.num_seqs + 1)


def _normal_bf16(rng, shape, gain=1.0):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if gain != 1.0:
        x *= np.float32(gain)
    return f32_to_bf16_bits(x)


def _fill(w, rng, with_dout, q_gain=1.0):
    T = w.total_tokens
    w.q = _normal_bf16(rng, (T, w.num_q_heads, w.head_dim), q_gain)
    w.k = _normal_bf16(rng, (T, w.num_kv_heads, w.head_dim))
    w.v = _normal_bf16(rng, (T, w.num_kv_heads, w.head_dim))
    if with_dout:
        w.dout = _normal_bf16(rng, (T, w.num_q_heads, w.head_dim))
    return w


def lengths_vit(rng, n_images=64):
    """H, W = 28*kh, 28*kw with kh, kw uniform over the integers 8..48 (224..1344 pixels);
    tokens = (H/14)*(W/14) = 4*kh*kw, in 256..9216.  Order as drawn."""
    kh = rng.integers(8, 49, size=n_images)
    kw = rng.integers(8, 49, size=n_images)
    return (2 * kh) * (2 * kw)


def lengths_long_short(rng, long_len=65536, n_short=256, lo=64, hi=1024, long_pos="first"):
    """One long sample plus n_short lengths floor(exp(U[ln lo, ln hi]))."""
    u = rng.uniform(math.log(lo), math.log(hi), size=n_short)
    short = np.floor(np.exp(u)).astype(np.int64)
    short = np.clip(short, lo, hi)
    pos = {"first": 0, "middle": n_short // 2, "last": n_short}[long_pos]
    return np.concatenate([short[:pos], [long_len], short[pos:]]).astype(np.int64)


def lengths_llm_pack(rng, budget=32768, median=2048, sigma=1.0, lo=128, hi=16384):
    """Lognormal lengths clamped to [lo, hi], appended until the token budget is met; the last
    one is cut to the remainder and merged into its predecessor when shorter than lo."""
    out, total = [], 0
    while total < budget:
        n = int(round(math.exp(rng.normal(math.log(median), sigma))))
        n = max(lo, min(hi, n))
        n = min(n, budget - total)
        if n < lo and out:
            out[-1] += n
        else:
            out.append(n)
        total += n
    return np.asarray(out, dtype=np.int64)


def make(config, seed=None, with_dout=None, long_pos="first", lengths_only=False):
    """Build BASELINE config 1..5.  lengths_only=True skips the tensors (for host-side tests)."""
    if config not in CONFIG_NAMES:
        raise ValueError(f"unknown config {config}")
    base = 2 if config == 5 else config
    seed = (1000 + base) if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    if base == 1:
        L, Hq, Hkv, D, causal = np.array([16, 37, 64, 129], dtype=np.int64), 2, 2, 64, False
    elif base == 2:
        L, Hq, Hkv, D, causal = lengths_vit(rng), 16, 16, 64, False
    elif base == 3:
        L, Hq, Hkv, D, causal = lengths_long_short(rng, long_pos=long_pos), 16, 16, 80, False
    else:
        L, Hq, Hkv, D, causal = lengths_llm_pack(rng), 32, 8, 128, True
    w = Workload(CONFIG_NAMES[config], np.asarray(L, dtype=np.int64), Hq, Hkv, D, causal,
                 1.0 / math.sqrt(D), seed)
    if lengths_only:
        return w
    if with_dout is None:
        with_dout = config == 5
    return _fill(w, rng, with_dout)


def make_custom(lengths, num_q_heads, num_kv_heads, head_dim, causal, seed, with_dout=False,
                scale=None, q_gain=1.0, name="custom"):
    """Arbitrary lengths/heads with the same value recipe (q_gain scales Q for peaky softmax)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w = Workload(name, np.asarray(lengths, dtype=np.int64), num_q_heads, num_kv_heads, head_dim,
                 bool(causal), (1.0 / math.sqrt(head_dim)) if scale is None else float(scale), seed)
    return _fill(w, rng, with_dout, q_gain)
