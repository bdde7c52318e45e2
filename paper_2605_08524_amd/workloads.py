"""Seeded synthetic inputs for the block-attention path.

This module only draws numbers: sequence lengths, block ownership and bf16
tensors.  It holds none of the method's arithmetic (no planning, no attention,
no merging) so that the CPU oracle and the HIP library can both be fed from it
without sharing anything else.  All randomness comes from
``numpy.random.default_rng(seed)`` (PCG64); the draw order is fixed:
lengths / ownership first, then Q, K, V, dO, each from its own child stream so
that a tensor can be regenerated alone.

Workload shapes follow the paper's evaluation set-up (Evaluation: setup;
Appendix "Evaluation on Additional Workloads"): causal attention, log-normal
sequence lengths, GQA head shapes of a Llama-3-70B-like model, tens of
thousands of tokens per worker, fixed-size blocks, coalesce degree 16.  The
paper's own length trace is not public; the log-normal draw stands in for it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

__all__ = [
    "Workload", "make_workload", "custom_workload", "bf16_bits", "bf16_to_f32",
    "draw_tensor", "CONFIG_NAMES",
]

CONFIG_NAMES = {
    1: "cfg1-tiny-fwd",
    2: "cfg2-packed-varlen-fwd",
    3: "cfg3-long-sequence-share-fwd",
    4: "cfg4-multimodal-mix-fwd",
    5: "cfg5-training-step-fwd-bwd",
}


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32 values (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def draw_tensor(seed: int, stream: int, shape, chunk_rows: int = 1 << 14) -> np.ndarray:
    """N(0,1) in fp32 rounded to bf16 bits; drawn in row chunks from
    ``default_rng([seed, stream])`` so the bits depend only on (seed, stream, shape)."""
    rng = np.random.default_rng([int(seed), int(stream)])
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.uint16)
    rows = shape[0]
    inner = shape[1:]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = bf16_bits(rng.standard_normal((r1 - r0,) + inner, dtype=np.float32))
    return out


@dataclass
class Workload:
    """One worker's share: what it owns, how it is blocked, and the tensor recipe."""
    name: str
    seed: int
    seq_lens: np.ndarray            # int32 [n_seqs]: full length of every sequence whose KV is resident
    block_size: int
    causal: int
    coalesce: int                   # c >= 1; 0 = all KV blocks of a Q block in one slot
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    q_owned: Optional[np.ndarray] = None   # int32 [n, 2] of (seq, idx_in_seq), canonical order; None = all
    notes: str = ""
    _cache: dict = field(default_factory=dict, repr=False)

    @property
    def t_kv(self) -> int:
        return int(np.sum(self.seq_lens, dtype=np.int64))

    @property
    def t_q(self) -> int:
        if self.q_owned is None:
            return self.t_kv
        bs = self.block_size
        tot = 0
        for s, i in self.q_owned:
            L = int(self.seq_lens[s])
            tot += min(bs, L - int(i) * bs)
        return tot

    # Streams: 1 = Q, 2 = K, 3 = V, 4 = dO.
    def q(self) -> np.ndarray:
        return self._get("q", 1, (self.t_q, self.n_q_heads, self.head_dim))

    def k(self) -> np.ndarray:
        return self._get("k", 2, (self.t_kv, self.n_kv_heads, self.head_dim))

    def v(self) -> np.ndarray:
        return self._get("v", 3, (self.t_kv, self.n_kv_heads, self.head_dim))

    def d_o(self) -> np.ndarray:
        return self._get("do", 4, (self.t_q, self.n_q_heads, self.head_dim))

    def _get(self, key, stream, shape):
        if key not in self._cache:
            self._cache[key] = draw_tensor(self.seed, stream, shape)
        return self._cache[key]

    def drop_tensors(self):
        self._cache.clear()


def _lognormal_lengths(rng, total, median, sigma, lo, hi):
    """Draw clip(round(exp(N(ln median, sigma))), lo, hi) until the sum reaches
    `total`; the last length is truncated so the sum is exactly `total`."""
    out = []
    acc = 0
    while acc < total:
        L = int(np.clip(np.rint(np.exp(rng.normal(np.log(median), sigma))), lo, hi))
        L = min(L, total - acc)
        out.append(L)
        acc += L
    return np.asarray(out, dtype=np.int32)


def make_workload(config: int, seed: int = 0) -> Workload:
    """The five benchmark configurations (1-based)."""
    rng = np.random.default_rng([int(seed), 0])
    if config == 1:
        while True:
            lens = rng.integers(100, 1025, size=8)
            if int(lens.sum()) <= 4096:
                break
        return Workload(CONFIG_NAMES[1], seed, lens.astype(np.int32), 128, 1, 0, 4, 4, 64,
                        notes="8 seqs uniform[100,1024], redrawn until sum<=4096; MHA 4 heads d=64")
    if config in (2, 5):
        lens = _lognormal_lengths(rng, 65536, 2048.0, 1.0, 16, 32768)
        return Workload(CONFIG_NAMES[config], seed, lens, 1024, 1, 16, 32, 8, 128,
                        notes="64K tokens, lognormal(median 2K, sigma 1.0) clipped [16,32K]; GQA 32/8 d=128")
    if config == 3:
        L, bs = 1 << 20, 2048
        nb = L // bs
        low = np.sort(rng.choice(nb // 2, size=32, replace=False))
        idx = np.sort(np.concatenate([low, nb - 1 - low]))
        owned = np.stack([np.zeros_like(idx), idx], axis=1).astype(np.int32)
        return Workload(CONFIG_NAMES[3], seed, np.asarray([L], dtype=np.int32), bs, 1, 16, 32, 8, 128,
                        q_owned=owned,
                        notes="one 1M-token sequence, 64 owned Q blocks = 32 zig-zag pairs (i, 511-i)")
    if config == 4:
        bs = 256
        total, short_total = 131072, 117964
        lens = []
        acc = 0
        while acc < short_total:
            L = int(rng.integers(64, 1025))
            L = min(L, short_total - acc)
            lens.append(L)
            acc += L
        long_len = int(rng.integers(65536, 262145))
        tail = total - short_total
        lens.append(long_len)
        lens = np.asarray(lens, dtype=np.int32)
        owned = []
        for s, L in enumerate(lens[:-1]):
            for i in range((int(L) + bs - 1) // bs):
                owned.append((s, i))
        # tail of the long sequence: the last blocks covering (at least) `tail` tokens
        nb_long = (long_len + bs - 1) // bs
        got = 0
        first = nb_long
        while got < tail:
            first -= 1
            got += min(bs, long_len - first * bs)
        for i in range(first, nb_long):
            owned.append((len(lens) - 1, i))
        return Workload(CONFIG_NAMES[4], seed, lens, bs, 1, 16, 16, 16, 128,
                        q_owned=np.asarray(owned, dtype=np.int32),
                        notes="90% short seqs uniform[64,1024] owned whole + tail blocks of one long seq "
                              "uniform[64K,256K] whose earlier KV is resident; MHA 16 heads d=128")
    raise ValueError(f"unknown config {config}")


def short_mix_workload(seed: int = 0, total: int = 65536, lo: int = 16, hi: int = 256, block_size: int = 1024) -> Workload:
    """A batch of short sequences only (lengths uniform in [lo, hi), all shorter than a block), the case the paper's
    sharding policy packs into shared blocks; model shape of the training configuration."""
    rng = np.random.default_rng([int(seed), 3])
    lens, acc = [], 0
    while acc < total:
        L = min(int(rng.integers(lo, hi)), total - acc)
        lens.append(L)
        acc += L
    return Workload("short-mix", seed, np.asarray(lens, dtype=np.int32), int(block_size), 1, 16, 32, 8, 128,
                    notes=f"{total} tokens of sequences uniform[{lo},{hi}); GQA 32/8 d=128")


def custom_workload(seq_lens, block_size, causal=1, coalesce=0, n_q_heads=4, n_kv_heads=4,
                    head_dim=64, q_owned=None, seed=0, name="custom") -> Workload:
    return Workload(name, seed, np.asarray(seq_lens, dtype=np.int32), int(block_size), int(causal),
                    int(coalesce), int(n_q_heads), int(n_kv_heads), int(head_dim),
                    q_owned=None if q_owned is None else np.asarray(q_owned, dtype=np.int32).reshape(-1, 2))


def length_trace(kind: str, total_tokens: int, seed: int = 0) -> np.ndarray:
    """Sequence lengths of one global batch for the scheduling experiments (paper, appendix
    "Synthetic Workloads"): lognormal lengths clipped to [1K, 512K], drawn until `total_tokens`
    is reached (the last one truncated).
      "lognormal": sigma 0.7, mean length 16K (the less long-tailed trace);
      "bimodal"  : each length from sigma 0.5 / mean 16K or sigma 0.5 / mean 64K with equal odds.
    The mean of a lognormal is exp(mu + sigma^2 / 2), which fixes mu."""
    rng = np.random.default_rng([int(seed), 7])
    out, acc = [], 0
    while acc < total_tokens:
        if kind == "lognormal":
            sigma, mean = 0.7, 16384.0
        elif kind == "bimodal":
            sigma, mean = 0.5, (16384.0 if rng.random() < 0.5 else 65536.0)
        else:
            raise ValueError(f"unknown trace kind {kind}")
        mu = np.log(mean) - 0.5 * sigma * sigma
        L = int(np.clip(np.rint(np.exp(rng.normal(mu, sigma))), 1024, 524288))
        L = min(L, total_tokens - acc)
        out.append(L)
        acc += L
    return np.asarray(out, dtype=np.int32)
