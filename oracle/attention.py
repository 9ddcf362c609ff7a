"""fp64 softmax attention over a paged KV cache -- the plain definition.

The paper (Section 2.1) describes prefilling as computing
P(x_{n+1} | x_1..x_n) and decoding as P(x_{n+t+1} | x_1..x_{n+t}), and names a
paged KV cache as its substrate (Section 5.1); it states no attention formula.
The reading used here is standard scaled dot-product attention:

    s_j = scale * <q, k_j>                for every visible key j
    w_j = exp(s_j - max_j s_j)
    o   = (sum_j w_j v_j) / (sum_j w_j)

* A decoding request sees all ``seq_len`` cached tokens (the current token's
  K/V were appended by the caller).
* Token i of a prefill chunk of length Lq, whose sequence has ``seq_len``
  cached tokens after the chunk, sits at absolute position
  p = seq_len - Lq + i and sees keys 0..p inclusive.
* Query head h reads KV head h // (Hq // Hkv).
* seq_len == 0 gives an all-zero output row.
* A prefill chunk that is longer than the context it is said to end
  (seq_len < Lq) has no positions to give its tokens: all its output rows are
  zero and none of its cache blocks is looked at (the library's stated
  behaviour for that caller slip; the paper has nothing to say about it).

Everything is three plain passes in float64; no online update, no blocking.
Stored 16-bit values are widened exactly.  TEST INFRASTRUCTURE ONLY.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of fp16 / bf16 bit patterns (uint16)."""
    bits = np.asarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("storage arrays are uint16 bit patterns")
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown storage dtype {dtype!r}")


def softmax_weights(q: np.ndarray, keys: np.ndarray, scale: float) -> np.ndarray:
    """Normalised attention weights of one query over ``keys[S, D]`` (float64)."""
    s = np.float64(np.float32(scale)) * (keys @ q)        # pass 1: logits
    w = np.exp(s - s.max())                               # pass 2: shifted exponentials
    return w / w.sum()                                    # pass 3: normalise


def attend_one(q: np.ndarray, keys: np.ndarray, values: np.ndarray, scale: float) -> np.ndarray:
    """o[D] for one query vector over keys[S, D], values[S, D]; zeros when S == 0."""
    if keys.shape[0] == 0:
        return np.zeros(values.shape[1], dtype=np.float64)
    return softmax_weights(q, keys, scale) @ values


def gather_sequence(
    cache_bits: np.ndarray, block_row: np.ndarray, seq_len: int, kv_head: int, dtype: str
) -> np.ndarray:
    """The first ``seq_len`` cached rows [S, D] of one KV head, in token order."""
    block_size = cache_bits.shape[2]
    pos = np.arange(seq_len)
    blocks = np.asarray(block_row)[pos // block_size]
    return widen(cache_bits[blocks, kv_head, pos % block_size, :], dtype)


def paged_decode(
    q_bits: np.ndarray,          # [N, Hq, D] uint16
    k_bits: np.ndarray,          # [num_blocks, Hkv, Bs, D] uint16
    v_bits: np.ndarray,
    block_table: np.ndarray,     # [N, max_blocks] int32
    seq_lens: Sequence[int],     # [N]
    scale: float,
    dtype: str,
    rows: Sequence[Tuple[int, int]] | None = None,
) -> np.ndarray:
    """Decode attention, float64 [N, Hq, D].

    ``rows`` optionally restricts the work to some (request, q_head) pairs;
    the other output rows are left NaN so that nobody mistakes them for results.
    """
    n, hq, d = q_bits.shape
    hkv = k_bits.shape[1]
    group = hq // hkv
    out = np.full((n, hq, d), np.nan if rows is not None else 0.0, dtype=np.float64)
    todo = rows if rows is not None else [(r, h) for r in range(n) for h in range(hq)]
    cached: dict = {}
    for r, h in todo:
        g = h // group
        if (r, g) not in cached:
            cached.clear()  # keep one (request, kv head) in memory at a time
            s = int(seq_lens[r])
            cached[(r, g)] = (
                gather_sequence(k_bits, block_table[r], s, g, dtype),
                gather_sequence(v_bits, block_table[r], s, g, dtype),
            )
        keys, values = cached[(r, g)]
        out[r, h] = attend_one(widen(q_bits[r, h], dtype), keys, values, scale)
    return out


def paged_prefill_chunk(
    q_bits: np.ndarray,          # [T, Hq, D] uint16, chunks of all sequences concatenated
    cu_q_lens: Sequence[int],    # [N+1] prefix sums of the chunk lengths
    k_bits: np.ndarray,
    v_bits: np.ndarray,
    block_table: np.ndarray,
    seq_lens: Sequence[int],     # [N] context length after the chunk was appended
    scale: float,
    dtype: str,
    rows: Sequence[Tuple[int, int, int]] | None = None,
) -> np.ndarray:
    """Causal prefill-chunk attention, float64 [T, Hq, D].

    ``rows`` optionally restricts the work to some (sequence, chunk token i,
    q_head) triples; the others are left NaN.
    """
    t, hq, d = q_bits.shape
    hkv = k_bits.shape[1]
    group = hq // hkv
    n = len(cu_q_lens) - 1
    out = np.full((t, hq, d), np.nan if rows is not None else 0.0, dtype=np.float64)
    if rows is None:
        rows = [(r, i, h) for r in range(n)
                for h in range(hq) for i in range(int(cu_q_lens[r + 1]) - int(cu_q_lens[r]))]
    cached: dict = {}
    for r, i, h in rows:
        g = h // group
        s = int(seq_lens[r])
        lq = int(cu_q_lens[r + 1]) - int(cu_q_lens[r])
        if s < lq:                           # inconsistent sequence: zero rows, cache untouched
            out[int(cu_q_lens[r]) + i, h] = 0.0
            continue
        if (r, g) not in cached:
            cached.clear()
            cached[(r, g)] = (
                gather_sequence(k_bits, block_table[r], s, g, dtype),
                gather_sequence(v_bits, block_table[r], s, g, dtype),
            )
        keys, values = cached[(r, g)]
        p = s - lq + i                       # absolute position of chunk token i
        row = int(cu_q_lens[r]) + i
        out[row, h] = attend_one(widen(q_bits[row, h], dtype), keys[: p + 1], values[: p + 1], scale)
    return out


def kv_append(
    k_cache: np.ndarray,         # [num_blocks, Hkv, Bs, D] uint16, modified in place
    v_cache: np.ndarray,
    k_new: np.ndarray,           # [T, Hkv, D] uint16, new tokens of all sequences concatenated
    v_new: np.ndarray,
    cu_new_lens: Sequence[int],  # [N+1] prefix sums of the number of new tokens per sequence
    block_table: np.ndarray,
    seq_lens: Sequence[int],     # [N] context length AFTER the append
) -> None:
    """Write the K/V rows of newly processed tokens into the paged cache (the step that precedes attention).

    New token i of sequence r (of n_r = cu[r+1]-cu[r] new ones) gets absolute position p = seq_len_r - n_r + i
    and lands in block block_table[r][p // Bs], row p % Bs, for every KV head.  Pure data movement.
    """
    bs = k_cache.shape[2]
    for r in range(len(cu_new_lens) - 1):
        n_r = int(cu_new_lens[r + 1]) - int(cu_new_lens[r])
        for i in range(n_r):
            p = int(seq_lens[r]) - n_r + i
            blk = int(block_table[r][p // bs])
            t = int(cu_new_lens[r]) + i
            k_cache[blk, :, p % bs, :] = k_new[t]
            v_cache[blk, :, p % bs, :] = v_new[t]
