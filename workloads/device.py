"""Device-side (torch) construction of the inputs of one serving step.

Only plumbing: block tables come from ``tensors.make_block_table``; Q/K/V are
drawn N(0,1) in float32 on the device with a seeded generator and rounded once
to the 16-bit storage type (large configurations), or uploaded from the numpy
generator (small ones).  Nothing here computes attention or counters.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from .batches import StepBatch
from .tensors import make_block_table, make_qkv_numpy
from .traces import SEED_BASE


def torch_dtype(tag: str):
    import torch

    return {"f16": torch.float16, "bf16": torch.bfloat16}[tag]


def bits_to_tensor(bits: np.ndarray, tag: str, device="cuda"):
    """uint16 bit patterns -> torch tensor of the storage dtype on ``device``."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch_dtype(tag))


def tensor_to_bits(t) -> np.ndarray:
    """torch fp16 / bf16 tensor (any device) -> uint16 bit patterns on the host."""
    import torch

    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@dataclass
class DeviceStep:
    batch: StepBatch
    # decode
    q: object                  # [Nd, Hq, D]
    seq_lens: object           # int32 [Nd]
    block_table: object        # int32 [Nd, max_blocks]
    # prefill (None when the step has no prefill)
    pf_q: Optional[object]     # [T, Hq, D]
    pf_cu_q_lens: Optional[object]
    pf_seq_lens: Optional[object]
    pf_block_table: Optional[object]
    pf_max_q_len: int
    # shared paged cache
    k_cache: object            # [num_blocks, Hkv, Bs, D]
    v_cache: object
    # counters
    counters: object           # int64 [num_clients]
    cu_client_ids: object      # int32 [Nd + Np]
    cu_n_in: object
    cu_n_out: object
    max_blocks_per_seq: int


def make_device_step(batch: StepBatch, device="cuda", host_random: bool = False, seed: Optional[int] = None) -> DeviceStep:
    """Allocate and fill every input of the step on ``device``.

    Decode and prefill sequences share one paged cache with a single random
    permutation of physical blocks; both block tables have the same row stride.
    """
    import torch

    sh = batch.shape
    seed = SEED_BASE + 100 * batch.config_id if seed is None else seed
    rng = np.random.default_rng(seed)
    all_lens = np.concatenate([batch.seq_lens, batch.pf_seq_lens]).astype(np.int64)
    table, num_blocks = make_block_table(rng, all_lens, sh.block_size, spare_blocks=3)
    nd, np_ = batch.num_decode, batch.num_prefill
    total_q = int(batch.pf_q_lens.sum()) if np_ else 0
    dt = torch_dtype(sh.dtype)
    if host_random:
        q_bits, k_bits, v_bits = make_qkv_numpy(rng, nd + total_q, sh.num_q_heads, sh.num_kv_heads, sh.head_dim,
                                                num_blocks, sh.block_size, sh.dtype)
        q_all = bits_to_tensor(q_bits, sh.dtype, device)
        k_cache = bits_to_tensor(k_bits, sh.dtype, device)
        v_cache = bits_to_tensor(v_bits, sh.dtype, device)
    else:
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        q_all = torch.randn((nd + total_q, sh.num_q_heads, sh.head_dim), generator=gen, device=device,
                            dtype=torch.float32).to(dt)
        shape = (num_blocks, sh.num_kv_heads, sh.block_size, sh.head_dim)
        k_cache = torch.empty(shape, device=device, dtype=dt)
        v_cache = torch.empty(shape, device=device, dtype=dt)
        step = max(1, (1 << 27) // (sh.num_kv_heads * sh.block_size * sh.head_dim))   # <= 512 MiB of fp32 at a time
        for lo in range(0, num_blocks, step):
            hi = min(num_blocks, lo + step)
            k_cache[lo:hi] = torch.randn((hi - lo,) + shape[1:], generator=gen, device=device, dtype=torch.float32).to(dt)
            v_cache[lo:hi] = torch.randn((hi - lo,) + shape[1:], generator=gen, device=device, dtype=torch.float32).to(dt)
    ids, n_in, n_out = batch.counter_update_args(first_chunk=(batch.meta.get("prefill_chunk", "0") == "0"))
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)
    table_t = i32(table)
    cu = np.concatenate([[0], np.cumsum(batch.pf_q_lens)]).astype(np.int32)
    return DeviceStep(
        batch=batch,
        q=q_all[:nd].contiguous(),
        seq_lens=i32(batch.seq_lens),
        block_table=table_t[:nd].contiguous(),
        pf_q=q_all[nd:].contiguous() if np_ else None,
        pf_cu_q_lens=i32(cu) if np_ else None,
        pf_seq_lens=i32(batch.pf_seq_lens) if np_ else None,
        pf_block_table=table_t[nd:].contiguous() if np_ else None,
        pf_max_q_len=int(batch.pf_q_lens.max()) if np_ else 0,
        k_cache=k_cache,
        v_cache=v_cache,
        counters=torch.from_numpy(np.ascontiguousarray(batch.counters_before, dtype=np.int64)).to(device),
        cu_client_ids=i32(ids),
        cu_n_in=i32(n_in),
        cu_n_out=i32(n_out),
        max_blocks_per_seq=int(table.shape[1]),
    )


def sequence_rows_to_host(cache, block_row, seq_len: int, kv_head: int) -> np.ndarray:
    """Copy the first ``seq_len`` cached rows of one KV head to the host as uint16 bits [S, D]."""
    bs = cache.shape[2]
    nb = (seq_len + bs - 1) // bs
    rows = cache[block_row[:nb].long(), kv_head]            # [nb, Bs, D] on the device
    return tensor_to_bits(rows.reshape(nb * bs, -1)[:seq_len])
