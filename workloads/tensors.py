"""Seeded block tables and Q/K/V arrays (numpy, host side).

Values are drawn i.i.d. N(0,1) in float32 and rounded once (to nearest, ties
to even) to the 16-bit storage type.  The rounded bit patterns are what every
consumer reads, so nobody rounds differently from anybody else.  Arrays in
the 16-bit storage types are carried as ``numpy.uint16`` bit patterns plus a
dtype tag ("f16" or "bf16"), because numpy has no bfloat16.

Paged layout (the same for K and V):
    cache[num_blocks, num_kv_heads, block_size, head_dim]
    block_table[num_seqs, max_blocks_per_seq]  (int32, physical block ids)
so token p of sequence r lives in block ``block_table[r, p // block_size]`` at
row ``p % block_size``.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def f32_to_storage_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to fp16 / bf16 and return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = x.view(np.uint32)
        rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        return (rounded >> np.uint32(16)).astype(np.uint16)
    raise ValueError(f"unknown storage dtype {dtype!r}")


def make_block_table(
    rng: np.random.Generator,
    seq_lens: Sequence[int],
    block_size: int,
    spare_blocks: int = 3,
    min_row_len: int = 0,
    pad_value: int = 0,
) -> Tuple[np.ndarray, int]:
    """Deal a random permutation of the physical blocks out to the sequences.

    Returns (block_table, num_blocks).  Entries past a sequence's last block
    hold ``pad_value``; a correct consumer never reads them.
    """
    need = [(int(s) + block_size - 1) // block_size for s in seq_lens]
    total = int(sum(need))
    num_blocks = total + spare_blocks
    perm = rng.permutation(num_blocks).astype(np.int32)
    width = max([min_row_len, 1] + need)
    table = np.full((len(need), width), pad_value, dtype=np.int32)
    at = 0
    for r, n in enumerate(need):
        table[r, :n] = perm[at:at + n]
        at += n
    return table, num_blocks


def make_qkv_numpy(
    rng: np.random.Generator,
    num_q_rows: int,
    num_q_heads: int,
    num_kv_heads: int,
    head_dim: int,
    num_blocks: int,
    block_size: int,
    dtype: str,
    chunk_blocks: int = 4096,
) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """q[num_q_rows, Hq, D], k_cache and v_cache[num_blocks, Hkv, Bs, D] as uint16 bits."""
    q = f32_to_storage_bits(rng.standard_normal((num_q_rows, num_q_heads, head_dim), dtype=np.float32), dtype)
    shape = (num_blocks, num_kv_heads, block_size, head_dim)
    k = np.empty(shape, dtype=np.uint16)
    v = np.empty(shape, dtype=np.uint16)
    for lo in range(0, num_blocks, chunk_blocks):
        hi = min(num_blocks, lo + chunk_blocks)
        sub = (hi - lo,) + shape[1:]
        k[lo:hi] = f32_to_storage_bits(rng.standard_normal(sub, dtype=np.float32), dtype)
        v[lo:hi] = f32_to_storage_bits(rng.standard_normal(sub, dtype=np.float32), dtype)
    return q, k, v


NAN_BITS = {"f16": 0x7E00, "bf16": 0x7FC0}


def poison_unused_rows(cache: np.ndarray, block_table: np.ndarray, seq_lens: Sequence[int], bits: int) -> None:
    """Overwrite, in place, every cache row that no valid token occupies.

    ``bits`` is the 16-bit pattern to write (``NAN_BITS[dtype]`` for a NaN).
    Used to check that rows past seq_len in a sequence's last block, and spare
    blocks, never influence a result.
    """
    num_blocks, _, block_size, _ = cache.shape
    used = np.zeros((num_blocks, block_size), dtype=bool)
    for r, s in enumerate(seq_lens):
        s = int(s)
        for b in range((s + block_size - 1) // block_size):
            n = min(block_size, s - b * block_size)
            used[int(block_table[r, b]), :n] = True
    for b in np.nonzero(~used.all(axis=1))[0]:
        cache[b][:, ~used[b], :] = np.uint16(bits)
