"""KV blocks of fewer than 16 tokens -- the paper's own system pages its cache one token at a time (Section 5.1) --
through the C ABI against the CPU oracle (needs an MI355X).  These sizes take the library's general path: the
same entry points, same results, no tuning."""
import math
import sys

import numpy as np
import pytest

import paper_2401_00588_amd as vtc
from oracle import attention as OA
from oracle.counters import counter_update as oracle_counter_update
from oracle.counters import gather_slots as oracle_gather_slots
from tests.helpers import check_both_outputs
from workloads import (NAN_BITS, bits_to_tensor, make_block_table, make_qkv_numpy, poison_unused_rows, tensor_to_bits)

pytestmark = pytest.mark.gpu
SCALE = 1.0 / math.sqrt(128.0)
SEQ = [1, 2, 3, 15, 16, 17, 33, 100, 0, 257, 40]


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


@pytest.mark.parametrize("bs", [1, 2, 4, 8])
@pytest.mark.parametrize("dtype,hq,hkv", [("f16", 4, 4), ("bf16", 8, 2)])
def test_decode_with_small_blocks(torch, bs, dtype, hq, hkv):
    say(f"decode block size {bs} dtype={dtype} Hq={hq} Hkv={hkv}")
    rng = np.random.default_rng(100 + bs)
    table, nb = make_block_table(rng, SEQ, bs, min_row_len=300)
    q, k, v = make_qkv_numpy(rng, len(SEQ), hq, hkv, 128, nb, bs, dtype)
    poison_unused_rows(k, table, SEQ, NAN_BITS[dtype])
    poison_unused_rows(v, table, SEQ, NAN_BITS[dtype])
    args = (bits_to_tensor(q, dtype), bits_to_tensor(k, dtype), bits_to_tensor(v, dtype), _i32(torch, table), _i32(torch, SEQ))
    mk = lambda o: vtc.make_params(hq, hkv, 128, bs, table.shape[1], dtype, SCALE, o)
    out16 = vtc.vtc_attn_decode(mk(None), *args)
    out32 = vtc.vtc_attn_decode(mk("f32"), *args)
    torch.cuda.synchronize()
    want = OA.paged_decode(q, k, v, table, SEQ, SCALE, dtype)
    got = check_both_outputs(out16, out32, want, dtype, f"decode, block size {bs}")
    assert (got[8] == 0).all()
    # the entry point without a workspace and the fused step give the same rows; the step's charge is exact
    out_s = torch.empty_like(out16)
    vtc.vtc_attn_decode_static(mk(None), *args, out_s)
    counters = torch.tensor([3, 4], dtype=torch.int64).cuda()
    ids = rng.integers(0, 2, size=len(SEQ)).astype(np.int32)
    ones = np.ones(len(SEQ), dtype=np.int32)
    out_f = vtc.vtc_step_decode(mk(None), *args, counters, _i32(torch, ids), None, _i32(torch, ones), 1, 2)
    torch.cuda.synchronize()
    assert torch.equal(out_s.view(torch.int16), out16.view(torch.int16))
    assert torch.equal(out_f.view(torch.int16), out16.view(torch.int16))
    assert counters.cpu().tolist() == oracle_counter_update([3, 4], ids, None, ones, 1, 2)


@pytest.mark.parametrize("bs", [1, 4])
@pytest.mark.parametrize("dtype,hq,hkv", [("bf16", 8, 2), ("f16", 4, 4)])
def test_prefill_chunk_with_small_blocks(torch, bs, dtype, hq, hkv):
    say(f"prefill block size {bs} dtype={dtype} Hq={hq} Hkv={hkv}")
    rng = np.random.default_rng(200 + bs)
    q_lens = [1, 5, 33, 64, 20, 7]
    seq = [1, 5, 90, 64, 10, 0]                 # the last two are shorter than their chunks: zero rows
    table, nb = make_block_table(rng, seq, bs, min_row_len=100, pad_value=1 << 28)
    table[4, :] = 1 << 28
    cu = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    q, k, v = make_qkv_numpy(rng, int(cu[-1]), hq, hkv, 128, nb, bs, dtype)
    args = (bits_to_tensor(q, dtype), _i32(torch, cu), max(q_lens), bits_to_tensor(k, dtype), bits_to_tensor(v, dtype),
            _i32(torch, table), _i32(torch, seq))
    mk = lambda o: vtc.make_params(hq, hkv, 128, bs, table.shape[1], dtype, SCALE, o)
    out16 = vtc.vtc_attn_prefill_chunk(mk(None), *args)
    out32 = vtc.vtc_attn_prefill_chunk(mk("f32"), *args)
    torch.cuda.synchronize()
    want = OA.paged_prefill_chunk(q, cu, k, v, table, seq, SCALE, dtype)
    got = check_both_outputs(out16, out32, want, dtype, f"prefill, block size {bs}")
    assert (got[cu[4]:] == 0).all() and np.abs(got[cu[2]:cu[3]]).sum() > 0


@pytest.mark.parametrize("bs", [1, 2, 8])
def test_append_and_slots_with_small_blocks(torch, bs):
    say(f"kv_append and slot indices, block size {bs}")
    rng = np.random.default_rng(300 + bs)
    hkv, dtype = 4, "bf16"
    seq = [5, 1, 40, 17]
    new = [2, 1, 40, 0]
    table, nb = make_block_table(rng, seq, bs)
    _, k, v = make_qkv_numpy(rng, 1, 4, hkv, 128, nb, bs, dtype)
    cu = np.concatenate([[0], np.cumsum(new)]).astype(np.int32)
    _, k_new, v_new = make_qkv_numpy(rng, 1, 4, hkv, 128, int(cu[-1]), 1, dtype)
    k_new, v_new = k_new[:, :, 0, :].copy(), v_new[:, :, 0, :].copy()          # [T, Hkv, D]
    p = vtc.make_params(4, hkv, 128, bs, table.shape[1], dtype, SCALE)
    kd, vd = bits_to_tensor(k, dtype), bits_to_tensor(v, dtype)
    vtc.vtc_kv_append(p, bits_to_tensor(k_new, dtype), bits_to_tensor(v_new, dtype), _i32(torch, cu), max(new), kd, vd,
                      _i32(torch, table), _i32(torch, seq))
    torch.cuda.synchronize()
    OA.kv_append(k, v, k_new, v_new, cu, table, seq)
    assert np.array_equal(tensor_to_bits(kd), k) and np.array_equal(tensor_to_bits(vd), v)
    cu_s = np.concatenate([[0], np.cumsum(seq)]).astype(np.int32)
    slots = torch.full((int(cu_s[-1]),), -1, dtype=torch.int32).cuda()
    vtc.vtc_debug_gather_slots(p, _i32(torch, table), _i32(torch, seq), _i32(torch, cu_s), max(seq), slots)
    assert slots.cpu().tolist() == oracle_gather_slots(table, seq, bs)
