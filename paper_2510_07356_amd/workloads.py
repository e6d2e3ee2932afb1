"""Seeded synthetic decode-attention inputs (numpy only).

This module serves both the HIP path's tests/benchmark and the CPU oracle and
therefore holds none of the method's arithmetic: it draws random numbers,
rounds them to bf16 bit patterns, lays them out as a KV cache and nothing else.

The workloads stand in for the paper's long reasoning traces (Section 3.3: a
32B grouped-query model sampled several times per task; Table 3: traces of
about 6-7 thousand tokens on average; Section 4.1: at most 32,768 tokens).
The traces themselves are not reproduced; only their shape is: head counts of
the 32B model (40 query / 8 KV heads of 128) or of the 8B comparands (32 / 8),
and KV lengths from 512 to 32,768 tokens.

Random streams: numpy PCG64 seeded with the list [seed, stream, sequence];
stream 0 = lengths, 1 = Q, 2 = K, 3 = V, 4 = outlier positions,
5 = block permutation.  fp32 normals are rounded to bf16 with
round-to-nearest-even and kept as uint16 bit patterns.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

try:                                    # optional accelerator for the bf16 rounding of big arrays
    import torch as _torch
except ImportError:                     # pragma: no cover
    _torch = None

BF16_POISON = np.uint16(0x7FC0)   # quiet NaN: any read of padding shows up in the output
PAGE = 16

_STREAM_LENS, _STREAM_Q, _STREAM_K, _STREAM_V, _STREAM_OUTLIER, _STREAM_PERM = range(6)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns
    (finite inputs; the draws are normal variates, never NaN or inf)."""
    x = np.asarray(x, dtype=np.float32)
    if _torch is not None and x.size >= 1 << 16:
        # same rounding, one fused pass instead of five numpy passes (see tests/test_workloads.py)
        t = _torch.from_numpy(np.ascontiguousarray(x)).to(_torch.bfloat16)
        return t.view(_torch.int16).numpy().view(np.uint16).reshape(x.shape)
    u = np.ascontiguousarray(x).reshape(-1).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.asarray(b, dtype=np.uint16)
    return (b.astype(np.uint32).reshape(-1) << np.uint32(16)).view(np.float32).reshape(b.shape)


@dataclass
class Workload:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    scale: float
    page_size: int                      # 0 = contiguous cache
    q: np.ndarray                       # [B, Hq, D] uint16
    k: np.ndarray                       # logical index [b|block, g, t|slot, d] uint16 (maybe a strided view)
    v: np.ndarray
    kv_lens: np.ndarray                 # [B] int32
    block_table: Optional[np.ndarray]   # [B, max_blocks] int32, -1 padded, or None
    layout: str                         # "head_major" or "token_major"

    @property
    def kv_tokens(self) -> int:
        return int(self.kv_lens.astype(np.int64).sum())

    @property
    def kv_bytes(self) -> int:
        """Algorithmic K+V bytes one attention call has to read."""
        return self.kv_tokens * 2 * self.num_kv_heads * self.head_dim * 2

    @property
    def max_kv_len(self) -> int:
        return int(self.kv_lens.max(initial=0))


def _rng(seed: int, stream: int, item: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream), int(item)])


def _normal_bits(seed: int, stream: int, item: int, shape, row_gain: Optional[np.ndarray] = None) -> np.ndarray:
    x = _rng(seed, stream, item).standard_normal(shape, dtype=np.float32)
    if row_gain is not None:            # shape [tokens]: scale whole key positions before rounding
        x *= row_gain[None, :, None]
    return f32_to_bf16_bits(x)


def _pool() -> ThreadPoolExecutor:
    return ThreadPoolExecutor(max_workers=max(1, min(16, len(os.sched_getaffinity(0)))))


def _as_layout(a_head_major: np.ndarray, layout: str) -> np.ndarray:
    """Return an array whose logical index is [b, g, t, d]; for token_major the
    memory order is [b, t, g, d] and the result is a strided view of it."""
    if layout == "head_major":
        return a_head_major
    if layout == "token_major":
        return np.ascontiguousarray(a_head_major.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    raise ValueError(layout)


def make_contiguous(name: str, seed: int, batch: int, num_q_heads: int, num_kv_heads: int,
                    kv_lens: Sequence[int], head_dim: int = 128, cache_len: Optional[int] = None,
                    layout: str = "head_major", outlier_fraction: float = 0.0,
                    outlier_gain: float = 8.0, scale: Optional[float] = None) -> Workload:
    kv_lens = np.asarray(kv_lens, dtype=np.int32)
    assert kv_lens.shape == (batch,)
    lmax = int(cache_len if cache_len is not None else max(int(kv_lens.max(initial=0)), 1))
    D, Hkv = head_dim, num_kv_heads
    q = _normal_bits(seed, _STREAM_Q, 0, (batch, num_q_heads, D))
    k = np.full((batch, Hkv, lmax, D), BF16_POISON, dtype=np.uint16)
    v = np.full((batch, Hkv, lmax, D), BF16_POISON, dtype=np.uint16)

    def fill(b: int) -> None:
        L = int(kv_lens[b])
        if L == 0:
            return
        gain = None
        if outlier_fraction > 0.0:
            n_out = int(round(outlier_fraction * L))
            pos = _rng(seed, _STREAM_OUTLIER, b).choice(L, size=n_out, replace=False)
            gain = np.ones(L, dtype=np.float32)
            gain[pos] = outlier_gain
        k[b, :, :L, :] = _normal_bits(seed, _STREAM_K, b, (Hkv, L, D), gain)
        v[b, :, :L, :] = _normal_bits(seed, _STREAM_V, b, (Hkv, L, D))

    with _pool() as ex:
        list(ex.map(fill, range(batch)))
    return Workload(name, batch, num_q_heads, Hkv, D,
                    float(np.float32(scale if scale is not None else 1.0 / math.sqrt(D))), 0,
                    q, _as_layout(k, layout), _as_layout(v, layout), kv_lens, None, layout)


def make_paged(name: str, seed: int, batch: int, num_q_heads: int, num_kv_heads: int,
               kv_lens: Sequence[int], head_dim: int = 128, page_size: int = PAGE,
               table_width: Optional[int] = None, spare_blocks: int = 3,
               layout: str = "head_major", permute: bool = True,
               scale: Optional[float] = None) -> Workload:
    """Paged cache: the blocks of all sequences live in one shared pool, in an
    order given by a seeded permutation.  Sequence b's i-th logical block is
    perm[off_b + i], off_b the running sum of block counts."""
    kv_lens = np.asarray(kv_lens, dtype=np.int32)
    assert kv_lens.shape == (batch,)
    D, Hkv, P = head_dim, num_kv_heads, page_size
    nblk = -(-kv_lens.astype(np.int64) // P)
    total = int(nblk.sum())
    off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
    pool_blocks = total + spare_blocks
    perm = _rng(seed, _STREAM_PERM).permutation(pool_blocks)[:total] if permute \
        else np.arange(total, dtype=np.int64)
    width = int(table_width if table_width is not None else max(int(nblk.max(initial=0)), 1))
    table = np.full((batch, width), -1, dtype=np.int32)
    q = _normal_bits(seed, _STREAM_Q, 0, (batch, num_q_heads, D))
    kp = np.full((pool_blocks, Hkv, P, D), BF16_POISON, dtype=np.uint16)
    vp = np.full((pool_blocks, Hkv, P, D), BF16_POISON, dtype=np.uint16)

    def fill(b: int) -> None:
        L, nb = int(kv_lens[b]), int(nblk[b])
        if L == 0:
            return
        blocks = perm[off[b]:off[b] + nb]
        table[b, :nb] = blocks
        for pool, stream in ((kp, _STREAM_K), (vp, _STREAM_V)):
            padded = np.full((Hkv, nb * P, D), BF16_POISON, dtype=np.uint16)
            padded[:, :L, :] = _normal_bits(seed, stream, b, (Hkv, L, D))
            pool[blocks] = padded.reshape(Hkv, nb, P, D).transpose(1, 0, 2, 3)

    with _pool() as ex:
        list(ex.map(fill, range(batch)))
    if layout == "token_major":      # memory order [block, slot, g, d], logical view unchanged
        kp = np.ascontiguousarray(kp.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
        vp = np.ascontiguousarray(vp.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    elif layout != "head_major":
        raise ValueError(layout)
    return Workload(name, batch, num_q_heads, Hkv, D,
                    float(np.float32(scale if scale is not None else 1.0 / math.sqrt(D))), P,
                    q, kp, vp, kv_lens, table, layout)


# ---------------------------------------------------------------------------
# The five named configurations
# ---------------------------------------------------------------------------

def ragged_lengths(seed: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """Uniform integers on [lo, hi], both ends included."""
    return _rng(seed, _STREAM_LENS).integers(lo, hi + 1, size=batch).astype(np.int32)


def lognormal_lengths(seed: int, batch: int, median: float, sigma: float, cap: int) -> np.ndarray:
    """exp(ln median + sigma z), z ~ N(0,1), rounded and clipped to [1, cap]."""
    z = _rng(seed, _STREAM_LENS).standard_normal(batch)
    return np.clip(np.rint(np.exp(math.log(median) + sigma * z)), 1, cap).astype(np.int32)


CONFIG_NAMES = ("single_seq_512", "uniform_b16_4096", "ragged_b64_1k_16k",
                "long_b8_32k_outliers", "paged_b128_lognormal")


def make_config(index: int, layout: str = "head_major") -> Workload:
    """index 0..4, in the order of CONFIG_NAMES."""
    if index == 0:
        return make_contiguous(CONFIG_NAMES[0], 0, 1, 40, 8, [512], layout=layout)
    if index == 1:
        return make_contiguous(CONFIG_NAMES[1], 1, 16, 40, 8, [4096] * 16, layout=layout)
    if index == 2:
        lens = ragged_lengths(2, 64, 1024, 16384)
        return make_contiguous(CONFIG_NAMES[2], 2, 64, 40, 8, lens, cache_len=16384, layout=layout)
    if index == 3:
        return make_contiguous(CONFIG_NAMES[3], 3, 8, 40, 8, [32768] * 8, layout=layout,
                               outlier_fraction=0.001, outlier_gain=8.0)
    if index == 4:
        lens = lognormal_lengths(4, 128, 6000.0, 0.6, 32768)
        return make_paged(CONFIG_NAMES[4], 4, 128, 32, 8, lens, table_width=32768 // PAGE,
                          layout=layout)
    raise IndexError(index)


# ---------------------------------------------------------------------------
# Shared-prefix batches: the samples drawn for one prompt share the prompt's K/V
# ---------------------------------------------------------------------------

@dataclass
class SharedPrefixWorkload:
    """`base` holds the queries and the per-sequence SUFFIX caches (kv_lens = suffix lengths);
    the prefix of group j is kp[j, :, :prefix_lens[j]] / vp[...], stored once per group."""
    base: Workload
    kp: np.ndarray                 # [groups, Hkv, Pmax, D] uint16
    vp: np.ndarray
    prefix_lens: np.ndarray        # [groups] int32
    group_start: np.ndarray        # [groups + 1] int32

    @property
    def logical_kv_bytes(self) -> int:
        """K+V bytes an implementation without sharing would read (every sequence its own prefix copy)."""
        m = np.diff(self.group_start).astype(np.int64)
        tokens = int((m * self.prefix_lens.astype(np.int64)).sum()) + self.base.kv_tokens
        return tokens * 2 * self.base.num_kv_heads * self.base.head_dim * 2

    @property
    def physical_kv_bytes(self) -> int:
        """K+V bytes that exist in memory: each prefix once, plus the suffixes."""
        tokens = int(self.prefix_lens.astype(np.int64)[np.diff(self.group_start) > 0].sum()) + self.base.kv_tokens
        return tokens * 2 * self.base.num_kv_heads * self.base.head_dim * 2

    def concatenated(self) -> Workload:
        """The same attention problem without sharing: one contiguous cache per sequence holding
        [prefix of its group ; its suffix].  This is what the oracle is given."""
        w = self.base
        B, Hkv, D = w.batch, w.num_kv_heads, w.head_dim
        group_of = np.repeat(np.arange(len(self.prefix_lens)), np.diff(self.group_start))
        full = self.prefix_lens[group_of].astype(np.int64) + w.kv_lens.astype(np.int64)
        lmax = max(int(full.max(initial=0)), 1)
        k = np.full((B, Hkv, lmax, D), BF16_POISON, dtype=np.uint16)
        v = np.full((B, Hkv, lmax, D), BF16_POISON, dtype=np.uint16)
        for b in range(B):
            j, P, S = int(group_of[b]), int(self.prefix_lens[group_of[b]]), int(w.kv_lens[b])
            k[b, :, :P] = self.kp[j, :, :P]
            v[b, :, :P] = self.vp[j, :, :P]
            for t in range(S):
                if w.page_size:
                    blk, slot = int(w.block_table[b, t // w.page_size]), t % w.page_size
                    k[b, :, P + t] = w.k[blk, :, slot]
                    v[b, :, P + t] = w.v[blk, :, slot]
                else:
                    break
            if not w.page_size:
                k[b, :, P:P + S] = w.k[b, :, :S]
                v[b, :, P:P + S] = w.v[b, :, :S]
        return Workload(w.name + "_concat", B, w.num_q_heads, Hkv, D, w.scale, 0, w.q, k, v,
                        full.astype(np.int32), None, "head_major")


def make_shared_prefix(name: str, seed: int, group_sizes: Sequence[int], prefix_lens: Sequence[int],
                       suffix_lens: Sequence[int], num_q_heads: int = 40, num_kv_heads: int = 8,
                       head_dim: int = 128, paged: bool = False, layout: str = "head_major",
                       prefix_cache_len: Optional[int] = None, **kw) -> SharedPrefixWorkload:
    group_sizes = np.asarray(group_sizes, dtype=np.int32)
    prefix_lens = np.asarray(prefix_lens, dtype=np.int32)
    batch = int(group_sizes.sum())
    assert len(prefix_lens) == len(group_sizes) and len(suffix_lens) == batch
    if paged:
        base = make_paged(name, seed, batch, num_q_heads, num_kv_heads, suffix_lens, head_dim=head_dim,
                          layout=layout, **kw)
    else:
        base = make_contiguous(name, seed, batch, num_q_heads, num_kv_heads, suffix_lens, head_dim=head_dim,
                               layout=layout, **kw)
    pmax = int(prefix_cache_len if prefix_cache_len is not None else max(int(prefix_lens.max(initial=0)), 1))
    kp = np.full((len(group_sizes), num_kv_heads, pmax, head_dim), BF16_POISON, dtype=np.uint16)
    vp = np.full_like(kp, BF16_POISON)
    for j, P in enumerate(prefix_lens):
        if P > 0:
            kp[j, :, :P] = _normal_bits(seed + 1000, _STREAM_K, j, (num_kv_heads, int(P), head_dim))
            vp[j, :, :P] = _normal_bits(seed + 1000, _STREAM_V, j, (num_kv_heads, int(P), head_dim))
    start = np.concatenate([[0], np.cumsum(group_sizes)]).astype(np.int32)
    return SharedPrefixWorkload(base, kp, vp, prefix_lens, start)


def make_sampling_batch(seed: int = 5, tasks: int = 12, samples: int = 5, prompt_median: float = 1800.0,
                        trace_median: float = 6000.0, sigma: float = 0.6, cap: int = 32768) -> SharedPrefixWorkload:
    """A decode batch shaped like the paper's trace synthesis: `tasks` prompts, `samples` traces
    per prompt (Section 3.3 draws 5 per task), prompt lengths lognormal around `prompt_median`
    tokens, generated-so-far lengths lognormal around `trace_median` (Table 3: 6-7 thousand
    tokens on average), total length capped at `cap` (Section 4.1)."""
    rng = _rng(seed, _STREAM_LENS)
    prompts = np.clip(np.rint(np.exp(math.log(prompt_median) + 0.3 * rng.standard_normal(tasks))), 16, cap // 4)
    traces = np.clip(np.rint(np.exp(math.log(trace_median) + sigma * rng.standard_normal(tasks * samples))), 1, None)
    traces = np.minimum(traces, cap - np.repeat(prompts, samples))
    return make_shared_prefix(f"sampling_{tasks}x{samples}", seed, [samples] * tasks, prompts.astype(np.int32),
                              traces.astype(np.int32))
