"""Seeded synthetic inputs for the polar-quantized key-cache path.

This module only *draws inputs*: post-RoPE keys with outlier channels, queries,
fp16 values, ragged sequence lengths and page tables.  It holds none of the
method's arithmetic (no polar transform, no quantizer, no packing, no
attention) and imports neither the CPU oracle nor the HIP binding, so both can
be fed the same bytes.

Why these shapes: the paper measures on the attention shape of Llama-2-7B
(32 heads, MHA) and Llama-3.1-8B (32 query heads over 8 KV heads, head_dim
128; Section 5.2 "Superior efficiency", Appendix B.2) and states that key
outliers sit in one coordinate of a RoPE pair (Section 3.1, Figure 1).  The
generator reproduces that structure: i.i.d. N(0,1) keys, a few pair indices
per head scaled in ONE coordinate before the rotation, then rotate-half RoPE
(pair = dims (i, i+d/2), footnote 2 of Section 3.1; frequencies
phi_i = base^(-2i/d), Eq. 1) at the token's true position.

Every tensor of every sequence has its own counter-derived random stream, so a
test can regenerate one sequence of a large workload without drawing the rest.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Tuple

import numpy as np

SEED_BASE = 20250200

# tags that separate the random streams of one workload
_KEYS, _VALUES, _QUERY, _OUTLIERS, _LENGTHS, _PAGES = range(6)


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic decode (or encode) problem."""

    name: str
    index: int                 # selects the seed: SEED_BASE + index
    n_seqs: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    max_len: int               # context length (upper bound when ragged)
    min_len: int               # == max_len unless ragged
    r_bits: int
    t_bits: int
    group_tokens: int
    rope_base: float
    key_dtype: str             # "f16" | "f32"  (queries use the same)
    n_outlier_pairs: int       # pair indices per KV head that carry an outlier
    outlier_scale: float
    outlier_first_coord_only: bool
    shuffled_pages: bool       # page ids are a random permutation of the pool
    grouped_angles: bool = False   # angle quantizer: per-group min/scale instead of the uniform grid

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def n_pairs(self) -> int:
        return self.head_dim // 2

    @property
    def np_key_dtype(self):
        return np.float16 if self.key_dtype == "f16" else np.float32

    def scaled(self, **kw) -> "Workload":
        """Same recipe at another size (used by tests to shrink a config)."""
        return dataclasses.replace(self, **kw)


def _wl(name, index, S, Hq, Hkv, L, r, t, base, dt, nout, oscale, first_only,
        min_len=None, shuffled=False) -> Workload:
    return Workload(name=name, index=index, n_seqs=S, n_q_heads=Hq, n_kv_heads=Hkv,
                    head_dim=128, max_len=L, min_len=L if min_len is None else min_len,
                    r_bits=r, t_bits=t, group_tokens=128, rope_base=base, key_dtype=dt,
                    n_outlier_pairs=nout, outlier_scale=oscale,
                    outlier_first_coord_only=first_only, shuffled_pages=shuffled)


# "2% of the 64 pair indices" is 1.28; it is read as 2 pairs per KV head.
WORKLOADS: Dict[str, Workload] = {
    "tiny":   _wl("tiny", 1, 1, 1, 1, 4096, 4, 4, 1.0e4, "f32", 4, 10.0, True),
    "mha":    _wl("mha", 2, 8, 32, 32, 8192, 4, 4, 1.0e4, "f16", 2, 8.0, False),
    "gqa":    _wl("gqa", 3, 16, 32, 8, 32768, 4, 4, 5.0e5, "f16", 2, 8.0, False),
    "long33": _wl("long33", 4, 1, 32, 8, 131072, 3, 3, 5.0e5, "f16", 2, 8.0, False),
    "ragged": _wl("ragged", 5, 64, 32, 8, 16384, 4, 4, 5.0e5, "f16", 2, 8.0, False,
                  min_len=1024, shuffled=True),
    # prefill whose keys pq_encode_keys packs in the ragged config
    "prefill": _wl("prefill", 5, 1, 32, 8, 32768, 4, 4, 5.0e5, "f16", 2, 8.0, False),
}


def _rng(wl: Workload, tag: int, seq: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([wl.seed, tag, seq])
    return np.random.Generator(np.random.PCG64(ss))


def outlier_channels(wl: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """(pair index, coordinate) of each outlier, per KV head.

    Returns two int arrays of shape [n_kv_heads, n_outlier_pairs]; coordinate 0
    is dim j, coordinate 1 is dim j + d/2.  The same channels are used by every
    sequence of the workload (outlier channels are a property of the head).
    """
    rng = _rng(wl, _OUTLIERS)
    pairs = np.stack([rng.choice(wl.n_pairs, size=wl.n_outlier_pairs, replace=False)
                      for _ in range(wl.n_kv_heads)]).astype(np.int64)
    if wl.outlier_first_coord_only:
        coord = np.zeros_like(pairs)
    else:
        coord = rng.integers(0, 2, size=pairs.shape).astype(np.int64)
    return pairs, coord


def rope_tables(head_dim: int, base: float, positions: np.ndarray):
    """cos/sin of position * base^(-2i/d) for i < d/2, as float32 [len, d/2]."""
    half = head_dim // 2
    inv_freq = np.asarray(base, np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / head_dim)
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def apply_rope_rotate_half(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate each pair (x[..., i], x[..., i + d/2]) of a [len, heads, d] float32 array."""
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def seq_lengths(wl: Workload) -> np.ndarray:
    """Context length of each sequence, int32 [n_seqs]."""
    if wl.min_len == wl.max_len:
        return np.full(wl.n_seqs, wl.max_len, np.int32)
    rng = _rng(wl, _LENGTHS)
    return rng.integers(wl.min_len, wl.max_len + 1, size=wl.n_seqs).astype(np.int32)


def keys_for_seq(wl: Workload, seq: int, length: int) -> np.ndarray:
    """Post-RoPE keys of one sequence, [length, n_kv_heads, head_dim] in wl's key dtype."""
    rng = _rng(wl, _KEYS, seq)
    k = rng.standard_normal((length, wl.n_kv_heads, wl.head_dim), dtype=np.float32)
    pairs, coord = outlier_channels(wl)
    for h in range(wl.n_kv_heads):
        for p, c in zip(pairs[h], coord[h]):
            k[:, h, int(p) + int(c) * wl.n_pairs] *= np.float32(wl.outlier_scale)
    cos, sin = rope_tables(wl.head_dim, wl.rope_base, np.arange(length))
    return apply_rope_rotate_half(k, cos, sin).astype(wl.np_key_dtype)


def values_for_seq(wl: Workload, seq: int, length: int) -> np.ndarray:
    """fp16 N(0,1) values of one sequence, [length, n_kv_heads, head_dim]."""
    rng = _rng(wl, _VALUES, seq)
    return rng.standard_normal((length, wl.n_kv_heads, wl.head_dim), dtype=np.float32).astype(np.float16)


def queries(wl: Workload) -> np.ndarray:
    """One decode-step query per sequence, [n_seqs, n_q_heads, head_dim], N(0,1).

    A query that follows a context of L tokens sits at position L; N(0,1) is
    rotation invariant in each pair, so no rotation is applied to it.
    """
    rng = _rng(wl, _QUERY)
    q = rng.standard_normal((wl.n_seqs, wl.n_q_heads, wl.head_dim), dtype=np.float32)
    return q.astype(wl.np_key_dtype)


def page_table(wl: Workload, lens: np.ndarray) -> Tuple[np.ndarray, int]:
    """Block table int32 [n_seqs, max_pages_per_seq] (unused slots -1) and pool size in pages.

    Contiguous workloads use consecutive page ids; `shuffled_pages` draws a
    random permutation of the pool so that a sequence's pages are scattered.
    """
    g = wl.group_tokens
    n_pages = (lens.astype(np.int64) + g - 1) // g
    total = int(n_pages.sum())
    width = int(n_pages.max())
    ids = np.arange(total, dtype=np.int32)
    if wl.shuffled_pages:
        ids = _rng(wl, _PAGES).permutation(total).astype(np.int32)
    table = np.full((wl.n_seqs, width), -1, np.int32)
    o = 0
    for s, n in enumerate(n_pages):
        table[s, :n] = ids[o:o + n]
        o += int(n)
    return table, total
