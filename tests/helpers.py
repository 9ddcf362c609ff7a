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


# ---- the floating-point bar of the GPU parity tests ---------------------------------------------------
TOL = {"f16": 2e-3, "bf16": 1e-2}          # max-abs against the unrounded fp64 oracle
_MANTISSA_BITS = {"f16": 10, "bf16": 7}


def elementwise_tolerance(want: np.ndarray, dtype: str) -> np.ndarray:
    """The bound every output element is held to.

    It is the flat max-abs tolerance wherever the output format can express a result that close.  From
    |o| >= 4 on it cannot: there the spacing of bf16 is 2^-5 (of fp16 2^-8), so even the correctly
    rounded exact result may be off by half of that, 1.56e-2 (1.95e-3).  Such elements -- a handful per
    million with N(0,1) values and very few keys -- are held to half a unit in the last place of the
    output format plus a fifth of the flat tolerance for the arithmetic before the final rounding.
    """
    a = np.maximum(np.abs(np.asarray(want, dtype=np.float64)), 2.0 ** -24)
    half_ulp = 0.5 * np.exp2(np.floor(np.log2(a)) - _MANTISSA_BITS[dtype])
    return np.maximum(TOL[dtype], half_ulp + 0.2 * TOL[dtype])


def within_tolerance(got: np.ndarray, want: np.ndarray, dtype: str) -> bool:
    got = np.asarray(got, dtype=np.float64)
    return bool(np.isfinite(got).all() and (np.abs(got - want) <= elementwise_tolerance(want, dtype)).all())
