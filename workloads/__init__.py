"""Seeded synthetic inputs shaped like the long-context decode workloads.

This module only draws random numbers and rounds them to bfloat16.  It holds
none of the method's arithmetic and is the one piece of code that both the CPU
oracle's tests and the GPU path's tests/benchmark use, so that both sides see
the same input bits.

All tensors are numpy ``uint16`` arrays of bfloat16 bit patterns:

* ``k``, ``v``  : ``[Hkv, total, D]`` (head-major; rows of one head are contiguous)
* ``qwin``      : ``[B, Hq, W, D]``   observation-window queries
* ``q``         : ``[B, Hq, D]``      the decode-step query
* ``cu``        : ``int32 [B+1]``     prefix sums of the sequence lengths

Recipe (values drawn in float32 from a Philox counter-based generator keyed by
the seed, rounded once to bfloat16, round-to-nearest-even):

* K, V ~ N(0,1); ``n_outlier`` channel indices are drawn once per KV head and
  K and V are multiplied by ``outlier_scale`` in those channels for every token;
* optional log-normal jitter: each K row (token, head) is multiplied by
  ``exp(jitter_sigma * z)``, z ~ N(0,1);
* optional quiet channels (the top-p benchmark): a fraction ``quiet_fraction`` of the K channels of every
  KV head, drawn once per head from a stream of its own, is scaled by ``quiet_scale * exp(0.5 z)`` - key
  caches concentrate their magnitude in a minority of channels, and this is what lets a 99 % saliency
  threshold drop more than half of them (0.6 and 0.008 reproduce the paper's overall ratio of 0.58 for that
  variant); 0 leaves every other workload's bits as they were;
* Q_win and q ~ N(0,1).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    keep: int
    seqlens: np.ndarray            # int64 [B]
    n_outlier: int = 0
    outlier_scale: float = 1.0
    jitter_sigma: float = 0.0
    seed: int = 0
    extra: dict = field(default_factory=dict)
    quiet_fraction: float = 0.0    # fraction of K channels per KV head that carry little magnitude (0: none)
    quiet_scale: float = 1.0

    @property
    def cu(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seqlens)]).astype(np.int32)

    @property
    def total(self) -> int:
        return int(np.sum(self.seqlens))


# The five configurations the benchmark definition names.  `keep` is the integer T.
def config(idx: int, **over) -> Workload:
    if idx == 1:     # tiny single-step case
        w = Workload("cfg1_tiny_1k_keep64", 1, 32, 8, 128, 32, 64, np.array([1024]),
                     n_outlier=4, outlier_scale=10.0, seed=0)
    elif idx == 2:   # Llama-3.1-8B-shaped, 32K context, 80 % pruned
        w = Workload("cfg2_llama8b_b8_32k_keep26", 8, 32, 8, 128, 32, 26, np.full(8, 32768),
                     n_outlier=8, outlier_scale=8.0, jitter_sigma=0.5, seed=2)
    elif idx == 3:   # prefill pruning only, 128K tokens
        w = Workload("cfg3_prune_131k", 1, 32, 8, 128, 64, 26, np.array([131072]),
                     n_outlier=8, outlier_scale=8.0, jitter_sigma=0.5, seed=3)
    elif idx == 4:   # ragged serving-style batch over an eviction-compressed cache
        rng = np.random.Generator(np.random.Philox(key=4))
        lens = rng.integers(512, 2049, size=64)
        w = Workload("cfg4_ragged_b64_keep64", 64, 32, 8, 128, 32, 64, lens,
                     n_outlier=4, outlier_scale=10.0, seed=4)
    elif idx == 5:   # Qwen3-32B-shaped, 128K context
        w = Workload("cfg5_qwen32b_b4_131k_keep26", 4, 64, 8, 128, 32, 26, np.full(4, 131072),
                     n_outlier=8, outlier_scale=10.0, jitter_sigma=0.5, seed=5)
    else:
        raise ValueError(idx)
    for key, val in over.items():
        setattr(w, key, val)
    return w


def small(name="small", batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, window=8, keep=26,
          seqlens=(200, 77), n_outlier=4, outlier_scale=8.0, jitter_sigma=0.5, seed=11) -> Workload:
    """A free-form small case for parity tests."""
    return Workload(name, batch, n_q_heads, n_kv_heads, head_dim, window, keep,
                    np.asarray(seqlens, dtype=np.int64), n_outlier, outlier_scale, jitter_sigma, seed)


@dataclass
class Tensors:
    k: np.ndarray
    v: np.ndarray
    qwin: np.ndarray
    q: np.ndarray
    cu: np.ndarray
    outlier_channels: np.ndarray   # int64 [Hkv, n_outlier]
    layout: str = "HND"


def generate(w: Workload, chunk_tokens: int = 1 << 16) -> Tensors:
    """Draw the tensors of a workload.  Deterministic in (w.seed, shape parameters)."""
    hkv, d, total = w.n_kv_heads, w.head_dim, w.total
    root = np.random.SeedSequence(entropy=int(w.seed), spawn_key=(0x5AA7C,))
    s_out, s_k, s_v, s_j, s_qw, s_q = root.spawn(6)

    rng = np.random.Generator(np.random.Philox(s_out))
    if w.n_outlier > 0:
        outl = np.stack([np.sort(rng.choice(d, size=w.n_outlier, replace=False)) for _ in range(hkv)])
    else:
        outl = np.zeros((hkv, 0), dtype=np.int64)
    chan_scale = np.ones((hkv, d), np.float32)
    for h in range(hkv):
        chan_scale[h, outl[h]] = np.float32(w.outlier_scale)

    k_scale = chan_scale.copy()
    if w.quiet_fraction > 0.0:
        rqc = np.random.Generator(np.random.Philox(np.random.SeedSequence(entropy=int(w.seed), spawn_key=(0x5AA7C, 0x51E7))))
        for h in range(hkv):
            quiet = rqc.random(d) < w.quiet_fraction
            k_scale[h, quiet] *= np.float32(w.quiet_scale) * np.exp(np.float32(0.5) * rqc.standard_normal(d, dtype=np.float32)[quiet])

    k = np.empty((hkv, total, d), np.uint16)
    v = np.empty((hkv, total, d), np.uint16)
    rk = np.random.Generator(np.random.Philox(s_k))
    rv = np.random.Generator(np.random.Philox(s_v))
    rj = np.random.Generator(np.random.Philox(s_j))
    for h in range(hkv):
        for t0 in range(0, total, chunk_tokens):
            n = min(chunk_tokens, total - t0)
            xk = rk.standard_normal((n, d), dtype=np.float32) * k_scale[h]
            if w.jitter_sigma > 0.0:
                z = rj.standard_normal((n, 1), dtype=np.float32)
                xk *= np.exp(np.float32(w.jitter_sigma) * z)
            k[h, t0:t0 + n] = f32_to_bf16_bits(xk)
            xv = rv.standard_normal((n, d), dtype=np.float32) * chan_scale[h]
            v[h, t0:t0 + n] = f32_to_bf16_bits(xv)

    rq = np.random.Generator(np.random.Philox(s_qw))
    qwin = f32_to_bf16_bits(rq.standard_normal((w.batch, w.n_q_heads, w.window, d), dtype=np.float32))
    rq1 = np.random.Generator(np.random.Philox(s_q))
    q = f32_to_bf16_bits(rq1.standard_normal((w.batch, w.n_q_heads, d), dtype=np.float32))
    return Tensors(k, v, qwin, q, w.cu, outl, "HND")


def checksum(x: np.ndarray) -> int:
    """Order-dependent 64-bit checksum of a tensor's bytes (detects a generator change)."""
    b = np.ascontiguousarray(x).reshape(-1).view(np.uint8).astype(np.uint64)
    idx = (np.arange(b.size, dtype=np.uint64) % np.uint64(65521)) + np.uint64(1)
    return int(np.sum(b * idx, dtype=np.uint64))
