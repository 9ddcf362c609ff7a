"""Test-side helpers: packing dense K/V into a paged cache, dtype plumbing.  No attention math."""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

from workloads.tensors import f32_to_storage_bits, make_block_table


def pack_paged(
    keys: Sequence[np.ndarray],      # per sequence: float32 [S_r, Hkv, D]
    values: Sequence[np.ndarray],
    block_size: int,
    dtype: str,
    rng: np.random.Generator,
    spare_blocks: int = 2,
    fill_bits: int | None = None,
    pad_value: int = 0,
) -> Tuple[np.ndarray, np.ndarray, np.ndarray, List[int]]:
    """Scatter dense per-sequence K/V into a paged cache with a random block permutation."""
    seq_lens = [int(k.shape[0]) for k in keys]
    hkv, d = keys[0].shape[1], keys[0].shape[2]
    table, num_blocks = make_block_table(rng, seq_lens, block_size, spare_blocks, pad_value=pad_value)
    shape = (num_blocks, hkv, block_size, d)
    if fill_bits is None:
        kc = f32_to_storage_bits(rng.standard_normal(shape, dtype=np.float32), dtype)
        vc = f32_to_storage_bits(rng.standard_normal(shape, dtype=np.float32), dtype)
    else:
        kc = np.full(shape, fill_bits, dtype=np.uint16)
        vc = np.full(shape, fill_bits, dtype=np.uint16)
    for r, (k, v) in enumerate(zip(keys, values)):
        kb = f32_to_storage_bits(k, dtype)
        vb = f32_to_storage_bits(v, dtype)
        for p in range(seq_lens[r]):
            blk = int(table[r, p // block_size])
            kc[blk, :, p % block_size, :] = kb[p]
            vc[blk, :, p % block_size, :] = vb[p]
    return kc, vc, table, seq_lens


def bits_to_f64_via_torch(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Widen 16-bit storage through torch (independent of the oracle's own widening)."""
    import torch

    t = torch.from_numpy(bits.view(np.int16).copy())
    t = t.view(torch.float16 if dtype == "f16" else torch.bfloat16)
    return t.to(torch.float64).numpy()
