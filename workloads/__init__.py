"""Seeded synthetic workloads for the UniPrefill token-sparsification operator.

This module only *draws inputs*: sequence lengths, keep ratios, hidden states,
query/key projections and position ids, with the shapes of the paper's
long-context prefill experiments (4K-128K contexts, continuous batches, GQA
32/8 x 128 heads, block sizes 64/128, observation window n = 128 and A = 128
attention sinks -- Experimental Setup).  It holds none of the method's
arithmetic: no scoring, no selection, no compaction.  Both the CPU oracle's
tests and the HIP path's tests/bench draw their inputs here so that they see
byte-identical data.

The paper's own inputs are RULER prompts pushed through three real models;
neither the dataset nor the weights exist here, so these synthetic tensors
stand in for them.  No benchmark item is reproduced.

bfloat16 tensors are carried as ``uint16`` bit patterns (numpy has no bf16).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "Workload",
    "make_paged_cache",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "make_config",
    "make_custom",
    "CONFIG_NAMES",
]

N_OBS = 128   # observation window n (Experimental Setup)
N_SINK = 128  # attention sinks A (Experimental Setup)
HEAD_DIM = 128

CONFIG_NAMES = {
    1: "c1_4k_d1024_h8x8_G64_r0.5",
    2: "c2_32k_d4096_h32x8_G128_r0.3",
    3: "c3_16varlen_d4096_h32x8_G128",
    4: "c4_128k_d5120_h40x8_G128_r0.25_heavytail",
    5: "c5_64decode_8x8k_d4096_h32x8_G64_r0.4",
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even), return uint16 bits.

    NaN inputs map to the quiet NaN 0x7FC0 (sign preserved)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(x)
    if nan.any():
        rounded = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x0040), rounded)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    """One packed continuous-batching batch (all arrays are host numpy arrays).

    cu_seqlens : int32 [R+1]   packed row offsets, cu_seqlens[0] = 0
    keep_ratio : float32 [R]   per-request keep ratio in (0, 1]
    hidden     : uint16 [T, d]        bf16 bits
    q          : uint16 [T, Hq, D]    bf16 bits; rows outside each sequence's
                                      last n_obs tokens are NaN (never read)
    k          : uint16 [T, Hkv, D]   bf16 bits
    pos        : int32 [T]     position ids (data, gathered like a column)
    cu_seqlens_k : None, or int32 [R+1] when the requests follow earlier context: k is then
                   [Tk, Hkv, D], per request the keys of its earlier tokens, then of its own
    """

    name: str
    block_size: int
    n_obs: int
    n_sink: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    hidden_dim: int
    cu_seqlens: np.ndarray
    keep_ratio: np.ndarray
    hidden: np.ndarray
    q: np.ndarray
    k: np.ndarray
    pos: np.ndarray
    seed: int = 0
    notes: dict = field(default_factory=dict)
    cu_seqlens_k: np.ndarray | None = None

    @property
    def num_seqs(self) -> int:
        return int(self.cu_seqlens.shape[0] - 1)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


def _normal_bf16(rng: np.random.Generator, shape, chunk_rows: int = 1 << 15) -> np.ndarray:
    """~N(0,1) drawn as float32, rounded to bf16; drawn in row chunks to bound memory.

    The chunking does not change the stream: rows are drawn in order."""
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.uint16)
    rows = shape[0]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = f32_to_bf16_bits(rng.standard_normal((r1 - r0,) + shape[1:], dtype=np.float32))
    return out


def make_custom(
    *,
    name: str,
    seed: int,
    lengths,
    keep_ratio,
    hidden_dim: int,
    num_q_heads: int,
    num_kv_heads: int,
    block_size: int,
    n_obs: int = N_OBS,
    n_sink: int = N_SINK,
    head_dim: int = HEAD_DIM,
    k_row_lognormal: bool = False,
    pos_offsets=None,
    rng: np.random.Generator | None = None,
    earlier=None,
) -> Workload:
    """Draw one batch.  Draw order: hidden, q (window rows only), k, extra scales.

    (Lengths, ratios and position offsets are drawn by the caller from the same
    generator *before* this call when they are random.)

    ``earlier`` = tokens of earlier context per request (chunked prefill): k then has
    ``earlier[r] + lengths[r]`` rows per request and position ids start at ``earlier[r]``."""
    rng = np.random.default_rng(seed) if rng is None else rng
    lengths = np.asarray(lengths, dtype=np.int64)
    R = int(lengths.shape[0])
    cu = np.zeros(R + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lengths)
    T = int(cu[-1])
    ratio = np.asarray(keep_ratio, dtype=np.float32).reshape(R)
    cu_k = None
    Tk = T
    if earlier is not None:
        cu_k = np.zeros(R + 1, dtype=np.int32)
        cu_k[1:] = np.cumsum(lengths + np.asarray(earlier, dtype=np.int64))
        Tk = int(cu_k[-1])
        if pos_offsets is None:
            pos_offsets = [int(e) for e in earlier]

    hidden = _normal_bf16(rng, (T, hidden_dim))

    q = np.full((T, num_q_heads, head_dim), 0x7FC0, dtype=np.uint16)  # NaN: never read
    for r in range(R):
        n_eff = int(min(n_obs, lengths[r]))
        if n_eff:
            q[cu[r + 1] - n_eff:cu[r + 1]] = _normal_bf16(rng, (n_eff, num_q_heads, head_dim))

    if k_row_lognormal:
        kf = rng.standard_normal((Tk, num_kv_heads, head_dim), dtype=np.float32)
        z = rng.standard_normal(Tk, dtype=np.float32)
        kf *= np.exp(z)[:, None, None]
        k = f32_to_bf16_bits(kf)
        del kf
    else:
        k = _normal_bf16(rng, (Tk, num_kv_heads, head_dim))

    pos = np.empty(T, dtype=np.int32)
    for r in range(R):
        off = 0 if pos_offsets is None else int(pos_offsets[r])
        pos[cu[r]:cu[r + 1]] = np.arange(off, off + lengths[r], dtype=np.int32)

    return Workload(
        name=name, block_size=block_size, n_obs=n_obs, n_sink=n_sink,
        num_q_heads=num_q_heads, num_kv_heads=num_kv_heads, head_dim=head_dim,
        hidden_dim=hidden_dim, cu_seqlens=cu, keep_ratio=ratio,
        hidden=hidden, q=q, k=k, pos=pos, seed=seed, cu_seqlens_k=cu_k,
    )


def make_paged_cache(k: np.ndarray, cu_seqlens_k, kv_block_size: int, seed: int, spare_blocks: int = 3):
    """Lay packed keys out as a paged KV cache (input preparation only: a permuted copy).

    Returns (k_cache [num_blocks * B, ...] with unused rows NaN, block_table int32 [R, max_blocks]
    with unused entries -1).  Physical blocks are a seeded random permutation, a few stay unused."""
    ck = np.asarray(cu_seqlens_k, dtype=np.int64)
    B = int(kv_block_size)
    R = len(ck) - 1
    need = [int(-(-(ck[r + 1] - ck[r]) // B)) for r in range(R)]
    total = sum(need) + spare_blocks
    order = np.random.default_rng(seed).permutation(total)
    table = np.full((R, max(need + [1])), -1, dtype=np.int32)
    cache = np.full((total * B,) + k.shape[1:], 0x7FC0 if k.dtype == np.uint16 else np.nan, dtype=k.dtype)
    nxt = 0
    for r in range(R):
        for b in range(need[r]):
            phys = int(order[nxt]); nxt += 1
            table[r, b] = phys
            lo = int(ck[r]) + b * B
            hi = min(int(ck[r + 1]), lo + B)
            cache[phys * B:phys * B + (hi - lo)] = k[lo:hi]
    return cache, table


def make_config(idx: int, shrink: int = 1, hidden_dim: int | None = None) -> Workload:
    """The five benchmark workloads (seed = idx - 1).

    ``shrink`` divides every sequence length (kept >= 1) so that the CPU oracle
    can run structurally identical but smaller batches; shrink=1 is the full
    size.  ``hidden_dim`` overrides d (tests that do not need full-width rows).

    1: one 4096-token sequence, d=1024, 8/8 heads, G=64, ratio 0.5
    2: one 32768-token sequence, d=4096, 32/8 heads, G=128, ratio 0.3
    3: 16 requests, lengths U{2048..32768}, ratios U[0.2,0.6], d=4096, 32/8, G=128
    4: one 131072-token sequence, d=5120, 40/8 heads, G=128, ratio 0.25,
       every K row scaled by exp(z), z~N(0,1)  (heavy-tailed scores)
    5: 64 decode rows (length 1) then 8 prefill chunks of 8192-delta tokens,
       delta in [1,63] (ragged last blocks), d=4096, 32/8, G=64, ratio 0.4;
       chunk positions start at a seeded offset (positions are data)
    """
    if idx not in CONFIG_NAMES:
        raise ValueError(f"unknown config {idx}")
    seed = idx - 1
    rng = np.random.default_rng(seed)
    name = CONFIG_NAMES[idx] + ("" if shrink == 1 else f"_shrink{shrink}")

    def sh(n):
        return max(1, int(n) // shrink)

    if idx == 1:
        return make_custom(name=name, seed=seed, rng=rng, lengths=[sh(4096)], keep_ratio=[0.5],
                           hidden_dim=hidden_dim or 1024, num_q_heads=8, num_kv_heads=8, block_size=64)
    if idx == 2:
        return make_custom(name=name, seed=seed, rng=rng, lengths=[sh(32768)], keep_ratio=[0.3],
                           hidden_dim=hidden_dim or 4096, num_q_heads=32, num_kv_heads=8, block_size=128)
    if idx == 3:
        lengths = rng.integers(2048, 32768, size=16, endpoint=True)
        ratios = rng.uniform(0.2, 0.6, size=16).astype(np.float32)
        lengths = [sh(x) for x in lengths]
        return make_custom(name=name, seed=seed, rng=rng, lengths=lengths, keep_ratio=ratios,
                           hidden_dim=hidden_dim or 4096, num_q_heads=32, num_kv_heads=8, block_size=128)
    if idx == 4:
        return make_custom(name=name, seed=seed, rng=rng, lengths=[sh(131072)], keep_ratio=[0.25],
                           hidden_dim=hidden_dim or 5120, num_q_heads=40, num_kv_heads=8, block_size=128,
                           k_row_lognormal=True)
    # idx == 5
    delta = rng.integers(1, 63, size=8, endpoint=True)
    starts = rng.integers(0, 1 << 16, size=8)
    chunk = [max(1, sh(8192) - int(d)) for d in delta]
    lengths = [1] * 64 + chunk
    pos_offsets = list(rng.integers(1, 1 << 16, size=64)) + [int(s) for s in starts]
    return make_custom(name=name, seed=seed, rng=rng, lengths=lengths, keep_ratio=[0.4] * 72,
                       hidden_dim=hidden_dim or 4096, num_q_heads=32, num_kv_heads=8, block_size=64,
                       pos_offsets=pos_offsets)
