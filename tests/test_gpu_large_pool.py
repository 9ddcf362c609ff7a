"""KV pools of more than 2^31 elements per tensor: every entry point that addresses the paged cache is
checked with the blocks it uses spread up to the top of such a pool, so that an element or byte offset
computed in 32 bits anywhere on the path would read or write the wrong block.

The oracle never sees the large pool: it works on a compact cache holding the used blocks only, and the
device block table is the compact one mapped through a seeded injection into the large pool.
"""
import math
import sys

import numpy as np
import pytest

import paper_2401_00588_amd as vtc
from oracle import attention as OA
from oracle.counters import gather_slots as oracle_gather_slots
from tests.helpers import within_tolerance
from workloads import NAN_BITS, bits_to_tensor, make_block_table, make_qkv_numpy, tensor_to_bits

pytestmark = pytest.mark.gpu

SCALE = 1.0 / math.sqrt(128.0)


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch as t

    assert t.cuda.is_available(), "these tests need a GPU"
    vtc.load_library()
    return t


def _i32(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _spread(rng, num_compact, num_large):
    """Injection compact block id -> large-pool block id; the first and the last block of the pool are always used."""
    ids = rng.choice(np.arange(1, num_large - 1), size=num_compact - 2, replace=False)
    ids = np.concatenate([[0, num_large - 1], ids])
    rng.shuffle(ids)
    assert (ids >= num_large // 2).sum() > num_compact // 4      # a good share lies beyond 2^31 elements
    return ids.astype(np.int64)


def _large_pool(torch, compact_bits, ids, junk, num_large, dtype):
    """Uninitialised large device pool with the compact cache's blocks copied to their mapped places."""
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    pool = torch.empty((num_large,) + compact_bits.shape[1:], dtype=tdt, device="cuda")
    assert pool.numel() > 2 ** 31
    pool[torch.from_numpy(ids).cuda()] = bits_to_tensor(compact_bits, dtype)
    pool[junk] = float("nan")
    return pool


@pytest.mark.parametrize("dtype,hq,hkv,num_large", [("f16", 32, 32, 36000), ("bf16", 32, 8, 140000)])
def test_every_cache_access_is_64_bit_clean(torch, dtype, hq, hkv, num_large):
    say(f"large pool dtype={dtype} Hq={hq} Hkv={hkv} blocks={num_large}")
    rng = np.random.default_rng(97 + hkv)
    seq_lens = np.array([1, 16, 17, 200, 513, 1500, 64, 330], dtype=np.int32)
    n_new = np.array([1, 1, 17, 130, 256, 1, 0, 5], dtype=np.int32)       # tokens appended / prefilled this step
    table, nb = make_block_table(rng, seq_lens, 16)
    q_dec, k, v = make_qkv_numpy(rng, len(seq_lens), hq, hkv, 128, nb, 16, dtype)
    ids = _spread(rng, nb, num_large)
    big_table = ids[table].astype(np.int32)
    # entries past a sequence's last block name a free block that holds NaN only: a consumer that used them would show it
    junk = int(np.setdiff1d(np.arange(2, 64), ids)[0])
    for r, s_r in enumerate(seq_lens):
        big_table[r, (int(s_r) + 15) // 16:] = junk
    p = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE)

    # slots: bit-exact against the definition on the mapped table
    cu_s = np.concatenate([[0], np.cumsum(seq_lens)]).astype(np.int32)
    slots = torch.full((int(cu_s[-1]),), -1, dtype=torch.int32).cuda()
    vtc.vtc_debug_gather_slots(p, _i32(torch, big_table), _i32(torch, seq_lens), _i32(torch, cu_s),
                               int(seq_lens.max()), slots)
    assert slots.cpu().tolist() == oracle_gather_slots(big_table, seq_lens, 16)

    # append: the new rows start out as NaN in the device pool and must end up bit-identical to the oracle's append
    k_hole, v_hole = k.copy(), v.copy()
    new_k, new_v = [], []
    for r, (s, n) in enumerate(zip(seq_lens, n_new)):
        for pos in range(s - n, s):
            blk, row = table[r, pos // 16], pos % 16
            new_k.append(k[blk, :, row, :].copy())
            new_v.append(v[blk, :, row, :].copy())
            k_hole[blk, :, row, :] = NAN_BITS[dtype]
            v_hole[blk, :, row, :] = NAN_BITS[dtype]
    new_k, new_v = np.stack(new_k), np.stack(new_v)
    cu_n = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    kc = _large_pool(torch, k_hole, ids, junk, num_large, dtype)
    vc = _large_pool(torch, v_hole, ids, junk, num_large, dtype)
    say("  append")
    vtc.vtc_kv_append(p, bits_to_tensor(new_k, dtype), bits_to_tensor(new_v, dtype), _i32(torch, cu_n),
                      int(n_new.max()), kc, vc, _i32(torch, big_table), _i32(torch, seq_lens))
    torch.cuda.synchronize()
    k_or, v_or = k_hole.copy(), v_hole.copy()
    OA.kv_append(k_or, v_or, new_k, new_v, cu_n, table, seq_lens)
    assert np.array_equal(k_or, k) and np.array_equal(v_or, v)
    sel = torch.from_numpy(ids).cuda()
    assert np.array_equal(tensor_to_bits(kc[sel]), k_or) and np.array_equal(tensor_to_bits(vc[sel]), v_or)

    say("  decode")
    out = vtc.vtc_attn_decode(p, bits_to_tensor(q_dec, dtype), kc, vc, _i32(torch, big_table), _i32(torch, seq_lens))
    torch.cuda.synchronize()
    want = OA.paged_decode(q_dec, k, v, table, seq_lens, SCALE, dtype)
    assert within_tolerance(OA.widen(tensor_to_bits(out), dtype), want, dtype)

    say("  prefill chunk")
    q_pf = make_qkv_numpy(rng, int(cu_n[-1]), hq, hkv, 128, 1, 16, dtype)[0]
    out = vtc.vtc_attn_prefill_chunk(p, bits_to_tensor(q_pf, dtype), _i32(torch, cu_n), int(n_new.max()), kc, vc,
                                     _i32(torch, big_table), _i32(torch, seq_lens))
    torch.cuda.synchronize()
    want = OA.paged_prefill_chunk(q_pf, cu_n, k, v, table, seq_lens, SCALE, dtype)
    assert within_tolerance(OA.widen(tensor_to_bits(out), dtype), want, dtype)
