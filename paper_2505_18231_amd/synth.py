"""Seeded synthetic inputs for the coded-KV hot path.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no normalisation, rotation, quantisation or attention), so
both the CPU oracle's tests and the HIP path's tests may feed from it.

Streams are counter-based (Philox) and keyed by (seed, tensor tag, sequence,
kv-head), so any (sequence, head) unit can be regenerated alone.

Value recipe (stand-in for real model activations, which need weights):
  K[t][c] = scale_c * N(0,1) + bias_c,  scale_c = exp(N(0,1)),  bias_c ~ N(0, std 2),
            two seeded "outlier" channels per head get bias += 20;
  V ~ N(0,1);  q ~ N(0,1);  everything rounded to fp16.
"""
from __future__ import annotations

import numpy as np

HEAD_DIM = 128

_TAG = {"k": 1, "v": 2, "q": 3, "kstat": 4, "len": 5, "cb": 6, "misc": 7}


def _rng(seed: int, tag: str, b: int = 0, h: int = 0, extra: int = 0) -> np.random.Generator:
    stream = (_TAG[tag] << 56) | ((extra & 0xFFFF) << 40) | ((b & 0xFFFFF) << 20) | (h & 0xFFFFF)
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), stream]))


def channel_stats(seed: int, b: int, h: int, d: int = HEAD_DIM, per_seq: bool = False):
    """Per-channel (scale, bias) of the synthetic keys for kv-head h.

    per_seq=False: statistics depend on the head only (shared by all sequences);
    per_seq=True : biases are redrawn for every sequence b (stresses the Shift step).
    """
    g = _rng(seed, "kstat", 0, h)
    scale = np.exp(g.standard_normal(d))
    bias = 2.0 * g.standard_normal(d)
    outl = g.choice(d, size=2, replace=False)
    if per_seq:
        g2 = _rng(seed, "kstat", b + 1, h)
        bias = 2.0 * g2.standard_normal(d)
        outl = g2.choice(d, size=2, replace=False)
    bias[outl] += 20.0
    return scale, bias


def make_k(seed: int, b: int, h: int, length: int, d: int = HEAD_DIM, per_seq: bool = False,
           start: int = 0) -> np.ndarray:
    """Keys of one (sequence, kv-head) unit, tokens [start, start+length): fp16 [length][d]."""
    scale, bias = channel_stats(seed, b, h, d, per_seq)
    z = _rng(seed, "k", b, h, extra=((start % 65535) + 1) if start else 0)
    x = z.standard_normal((length, d), dtype=np.float32)
    return (x * scale.astype(np.float32) + bias.astype(np.float32)).astype(np.float16)


def make_v(seed: int, b: int, h: int, length: int, d: int = HEAD_DIM, start: int = 0) -> np.ndarray:
    """Values of one (sequence, kv-head) unit: fp16 [length][d], N(0,1)."""
    z = _rng(seed, "v", b, h, extra=((start % 65535) + 1) if start else 0)
    return z.standard_normal((length, d), dtype=np.float32).astype(np.float16)


def make_kv(seed: int, batch: int, n_kv_heads: int, length: int, d: int = HEAD_DIM,
            per_seq: bool = False):
    """K, V fp16 arrays [batch][n_kv_heads][length][d]."""
    k = np.empty((batch, n_kv_heads, length, d), dtype=np.float16)
    v = np.empty((batch, n_kv_heads, length, d), dtype=np.float16)
    for b in range(batch):
        for h in range(n_kv_heads):
            k[b, h] = make_k(seed, b, h, length, d, per_seq)
            v[b, h] = make_v(seed, b, h, length, d)
    return k, v


def make_q(seed: int, batch: int, n_q_heads: int, d: int = HEAD_DIM, step: int = 0) -> np.ndarray:
    """Decode queries fp16 [batch][n_q_heads][d], N(0,1)."""
    g = _rng(seed, "q", 0, 0, extra=step)
    return g.standard_normal((batch, n_q_heads, d), dtype=np.float32).astype(np.float16)


def ragged_lengths(seed: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """Sequence lengths uniform in [lo, hi], int32 [batch]."""
    g = _rng(seed, "len")
    return g.integers(lo, hi + 1, size=batch).astype(np.int32)


def codebook_samples(seed: int, n: int, sub_dim: int) -> np.ndarray:
    """Standard-normal training vectors for the codebook: fp32 [n][sub_dim]."""
    g = _rng(seed, "cb", 0, sub_dim)
    return g.standard_normal((n, sub_dim), dtype=np.float32)


def rope_inv_freq(base: float = 10000.0, d: int = HEAD_DIM) -> np.ndarray:
    """Rotary-embedding frequencies of a model configuration: fp32 [d/2], base ** (-2 i / d)."""
    return (float(base) ** (-np.arange(d // 2, dtype=np.float64) * 2.0 / d)).astype(np.float32)


def shuffled_page_table(seed: int, batch: int, pages_per_seq: int) -> np.ndarray:
    """A permutation of physical pages: int32 [batch][pages_per_seq] (for the paged layout)."""
    g = _rng(seed, "misc", 0, 0, extra=1)
    return g.permutation(batch * pages_per_seq).astype(np.int32).reshape(batch, pages_per_seq)


# The five workload shapes (index = position in the configuration list this build targets).
CONFIGS = {
    "C0": dict(name="tiny-1bit", batch=1, n_q_heads=1, n_kv_heads=1, length=1024, sub_dim=8,
               seed=0x5EED0000),
    "C1": dict(name="llama3-8b-gqa-2bit", batch=8, n_q_heads=32, n_kv_heads=8, length=8192,
               sub_dim=4, seed=0x5EED0001),
    "C2": dict(name="long-context-1bit", batch=1, n_q_heads=32, n_kv_heads=8, length=131072,
               sub_dim=8, seed=0x5EED0002),
    "C3": dict(name="mha-large-batch-2bit", batch=64, n_q_heads=32, n_kv_heads=32, length=32768,
               sub_dim=4, seed=0x5EED0003, per_seq=True),
    "C4": dict(name="ragged-paged", batch=32, n_q_heads=32, n_kv_heads=8, len_lo=512,
               len_hi=16384, page_size=256, append_steps=16, seed=0x5EED0004),
}
