"""Parity of the HIP path with the CPU oracle, through the C ABI (needs an MI355X).

Tolerances (max-abs against the *unrounded* fp64 oracle): 2e-3 for fp16 inputs, 1e-2
for bf16 inputs.  Every attention case runs twice on the same inputs: with fp32 output
rows, held to that flat bar on every element, and with output rows in the 16-bit
storage format, held to the flat bar for every |o| < 4 (beyond that the format's own
spacing exceeds it; tests/helpers.py prints how many elements that concerns) and
required to be the fp32 rows rounded once.  The benchmark configurations are compared
on every output element and must meet the flat bar throughout.  Counters and slot
indices are compared bit for bit.
"""
import math
import sys

import numpy as np
import pytest

import paper_2401_00588_amd as vtc
from oracle import attention as OA
from oracle.counters import counter_update as oracle_counter_update
from oracle.counters import gather_slots as oracle_gather_slots
from tests.helpers import (TOL, check_both_outputs, full_decode_oracle, full_prefill_oracle)
from workloads import (NAN_BITS, bits_to_tensor, make_block_table, make_device_step, make_qkv_numpy,
                       make_step_batch, poison_unused_rows, sequence_rows_to_host, tensor_to_bits)

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


# ------------------------------------------------------------------ counters
@pytest.mark.parametrize("n,clients,seed", [(8, 2, 0), (64, 2, 1), (256, 4, 2), (512, 27, 3), (272, 8, 4),
                                            (1, 1, 5), (5000, 27, 6), (20000, 5000, 7), (4097, 4096, 8)])
def test_counter_update_is_bit_exact(torch, n, clients, seed):
    say(f"counter_update n={n} clients={clients} seed={seed}")
    rng = np.random.default_rng(seed)
    ids = rng.integers(-2, clients + 2, size=n).astype(np.int32)       # some ids out of range on both sides
    n_in = rng.integers(0, 4097, size=n).astype(np.int32)
    n_out = rng.integers(0, 2, size=n).astype(np.int32)
    base = rng.integers(0, 1 << 40, size=clients).astype(np.int64)
    for w_p, w_q, use_in, use_out in ((1, 2, True, True), (1, 2, False, True), (3, 5, True, False), (7, 11, False, False)):
        c = torch.from_numpy(base.copy()).cuda()
        vtc.vtc_counter_update(c, _i32(torch, ids), _i32(torch, n_in) if use_in else None,
                               _i32(torch, n_out) if use_out else None, w_p, w_q)
        want = oracle_counter_update(base, ids, n_in if use_in else None, n_out if use_out else None, w_p, w_q)
        assert c.cpu().tolist() == want


def test_counter_update_negative_tokens_and_repeated_steps(torch):
    say("counter_update refunds / repeated steps")
    rng = np.random.default_rng(11)
    ids = rng.integers(0, 3, size=40).astype(np.int32)
    n_out = rng.integers(-50, 50, size=40).astype(np.int32)
    c = torch.zeros(3, dtype=torch.int64).cuda()
    want = [0, 0, 0]
    for _ in range(5):
        vtc.vtc_counter_update(c, _i32(torch, ids), None, _i32(torch, n_out), 1, 2)
        want = oracle_counter_update(want, ids, None, n_out, 1, 2)
    assert c.cpu().tolist() == want


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_counter_update_on_the_config_batches(torch, cfg):
    say(f"counter_update config {cfg}")
    b = make_step_batch(cfg)
    ids, n_in, n_out = b.counter_update_args()
    c = torch.from_numpy(b.counters_before.copy()).cuda()
    vtc.vtc_counter_update(c, _i32(torch, ids), _i32(torch, n_in), _i32(torch, n_out), b.w_p, b.w_q)
    want = oracle_counter_update(b.counters_before, ids, n_in, n_out, b.w_p, b.w_q)
    assert c.cpu().tolist() == want
    if b.counters_after is not None and b.num_prefill == 0:
        assert want == b.counters_after.tolist()        # what the CPU scheduler recorded for this step


# --------------------------------------------------------------------- slots
def test_gathered_slots_are_bit_exact(torch):
    say("gather_slots")
    rng = np.random.default_rng(21)
    seq = np.array([0, 1, 15, 16, 17, 255, 256, 257, 1000, 4096], dtype=np.int32)
    table, nb = make_block_table(rng, seq, 16)
    p = vtc.make_params(32, 8, 128, 16, table.shape[1], "bf16", SCALE)
    cu = np.concatenate([[0], np.cumsum(seq)]).astype(np.int32)
    out = torch.full((int(cu[-1]),), -1, dtype=torch.int32).cuda()
    vtc.vtc_debug_gather_slots(p, _i32(torch, table), _i32(torch, seq), _i32(torch, cu), int(seq.max()), out)
    assert out.cpu().tolist() == oracle_gather_slots(table, seq, 16)


# -------------------------------------------------------------------- decode
def _decode_case(torch, seq_lens, hq, hkv, dtype, seed, poison=False, min_row_len=0, scale=SCALE, label="decode",
                 workspace_bytes=None):
    """One decode call with 16-bit and one with fp32 output rows, both checked against the oracle."""
    rng = np.random.default_rng(seed)
    table, nb = make_block_table(rng, seq_lens, 16, min_row_len=min_row_len)
    q, k, v = make_qkv_numpy(rng, len(seq_lens), hq, hkv, 128, nb, 16, dtype)
    if poison:
        poison_unused_rows(k, table, seq_lens, NAN_BITS[dtype])
        poison_unused_rows(v, table, seq_lens, NAN_BITS[dtype])
    args = (bits_to_tensor(q, dtype), bits_to_tensor(k, dtype), bits_to_tensor(v, dtype), _i32(torch, table),
            _i32(torch, seq_lens))
    kw = {}
    if workspace_bytes is not None:
        kw["workspace"] = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda")
    out16 = vtc.vtc_attn_decode(vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, scale), *args, **kw)
    out32 = vtc.vtc_attn_decode(vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, scale, "f32"), *args, **kw)
    torch.cuda.synchronize()
    want = OA.paged_decode(q, k, v, table, seq_lens, scale, dtype)
    got = check_both_outputs(out16, out32, want, dtype, label)
    return got, want


RAGGED = [1, 2, 3, 4, 5, 15, 16, 17, 31, 32, 33, 100, 255, 256, 257, 300, 511, 512, 513, 700, 1023, 1025]


@pytest.mark.parametrize("dtype,hq,hkv", [("f16", 32, 32), ("bf16", 32, 8), ("f16", 8, 4), ("bf16", 16, 2),
                                          ("bf16", 4, 4), ("f16", 32, 8)])
def test_decode_ragged_lengths_match_the_oracle(torch, dtype, hq, hkv):
    say(f"decode ragged dtype={dtype} Hq={hq} Hkv={hkv}")
    got, want = _decode_case(torch, RAGGED, hq, hkv, dtype, seed=31)
    err = np.abs(got - want).max()
    say(f"  max abs err {err:.3e}  max |o| {np.abs(want).max():.3f}")


@pytest.mark.parametrize("dtype,hq,hkv", [("f16", 32, 32), ("bf16", 32, 8)])
def test_decode_ignores_rows_past_seq_len_and_handles_empty_sequences(torch, dtype, hq, hkv):
    say(f"decode poisoned tails dtype={dtype}")
    seq = [0, 1, 7, 16, 0, 250, 257, 17]
    got, want = _decode_case(torch, seq, hq, hkv, dtype, seed=32, poison=True, min_row_len=40)
    assert (got[0] == 0).all() and (got[4] == 0).all()


@pytest.mark.parametrize("n", [1, 5, 1500])
def test_decode_of_a_batch_with_no_tokens_at_all(torch, n):
    # every sequence empty: nothing to read, every output row is zero (both planning paths)
    say(f"decode of {n} empty sequences")
    rng = np.random.default_rng(40 + n)
    table, nb = make_block_table(rng, [0] * n, 16, min_row_len=3)
    q, k, v = make_qkv_numpy(rng, n, 8, 2, 128, nb, 16, "bf16")
    p = vtc.make_params(8, 2, 128, 16, table.shape[1], "bf16", SCALE)
    out = torch.full((n, 8, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    vtc.vtc_attn_decode(p, bits_to_tensor(q, "bf16"), bits_to_tensor(k, "bf16"), bits_to_tensor(v, "bf16"),
                        _i32(torch, table), _i32(torch, [0] * n), out=out)
    torch.cuda.synchronize()
    assert (tensor_to_bits(out) == 0).all()
    assert (OA.paged_decode(q, k, v, table, [0] * n, SCALE, "bf16") == 0).all()


@pytest.mark.parametrize("n,hq,hkv,dtype", [(2500, 4, 2, "bf16"), (9000, 2, 2, "f16")])
def test_decode_many_short_sequences(torch, n, hq, hkv, dtype):
    # more sequences than one planning pass (1024) and than the planner's on-chip prefix table (4096) hold;
    # many ranges then span several whole sequences, some of them empty
    say(f"decode {n} short sequences dtype={dtype}")
    rng = np.random.default_rng(n)
    seq = rng.integers(0, 49, size=n).astype(np.int32)
    seq[rng.integers(0, n, size=5)] = 700          # a few long ones, cut by several range boundaries
    got, want = _decode_case(torch, seq, hq, hkv, dtype, seed=n + 1)
    err = np.abs(got - want).max()
    say(f"  max abs err {err:.3e}")
    assert (got[seq == 0] == 0).all()


@pytest.mark.parametrize("dtype,hq,hkv", [("f16", 4, 4), ("bf16", 8, 2), ("bf16", 32, 8), ("f16", 16, 2)])
def test_decode_with_a_workspace_for_a_few_waves(torch, dtype, hq, hkv):
    # A workspace with room for about one wave per KV head: the call runs on that few waves, every one of them
    # closes hundreds of (sequence, kv head) pieces -- far more than it can park in LDS before writing them out --
    # and the long sequences are cut by several ranges.  Same results as with any other number of waves.
    say(f"decode on a few waves dtype={dtype} Hq={hq} Hkv={hkv}")
    rng = np.random.default_rng(77)
    n = 300
    seq = rng.integers(0, 41, size=n).astype(np.int32)
    seq[rng.integers(0, n, size=4)] = 333
    table_cols = (int(seq.max()) + 15) // 16
    p = vtc.make_params(hq, hkv, 128, 16, table_cols, dtype, SCALE)
    # sized for a single one-block sequence (one wave per KV head) plus this batch's per-sequence prefix
    small = vtc.vtc_attn_workspace_bytes(p, 1, 1) + 8 * n + 256
    assert small < vtc.vtc_attn_workspace_bytes(p, n, 0) // 8
    got, want = _decode_case(torch, seq, hq, hkv, dtype, seed=78, workspace_bytes=small)
    assert (got[seq == 0] == 0).all()


@pytest.mark.parametrize("seq,hq,hkv,dtype", [([1], 8, 8, "f16"), ([16, 1, 33, 0, 2], 8, 2, "bf16"),
                                              ([5] * 40, 32, 8, "bf16"), ([17, 16, 15] * 9, 4, 4, "f16"),
                                              ([1, 0, 0, 1, 0, 2000, 1, 1], 32, 32, "f16")])
def test_decode_ranges_of_a_block_or_two(torch, seq, hq, hkv, dtype):
    # The stream is cut by cost -- a block is one unit, beginning a (sequence, kv head) another -- and a batch this
    # small gets ranges of two or three units: a head's beginning plus its only block, the last block of one head
    # plus the beginning of the next, and cuts that fall on a beginning.  The long sequence of the last case is cut
    # into many ranges while its neighbours are one block each.
    say(f"decode tiny ranges {seq[:8]}... dtype={dtype} Hq={hq} Hkv={hkv}")
    got, want = _decode_case(torch, seq, hq, hkv, dtype, seed=900 + len(seq))
    assert (got[np.asarray(seq) == 0] == 0).all()


@pytest.mark.parametrize("n", [1, 63, 64, 65, 130, 1000, 1024, 1025])
def test_decode_batch_sizes_around_the_in_kernel_planning_limits(torch, n):
    # up to 1024 sequences every wave finds its own range (16 sequences per lane at most); one more
    # sequence and the planning kernel runs instead.  Lanes with no sequence, lanes whose sequences are
    # all empty, and the last partly filled lane are all present in these sizes.
    say(f"decode batch of {n} sequences")
    rng = np.random.default_rng(7000 + n)
    seq = rng.integers(0, 40, size=n).astype(np.int32)
    seq[rng.integers(0, n, size=max(1, n // 8))] = 0
    seq[rng.integers(0, n, size=2)] = 530
    got, want = _decode_case(torch, seq, 8, 2, "f16", seed=7100 + n)
    err = np.abs(got - want).max()
    say(f"  max abs err {err:.3e}")
    assert (got[seq == 0] == 0).all()


def test_decode_single_key_and_identical_keys(torch):
    say("decode closed forms on the GPU")
    rng = np.random.default_rng(33)
    seq = [1, 200]
    table, nb = make_block_table(rng, seq, 16)
    q, k, v = make_qkv_numpy(rng, 2, 32, 32, 128, nb, 16, "f16")
    for b in range(13):                         # sequence 1: every key identical -> mean of V
        k[table[1, b]] = k[table[1, 0], :, :1, :]
    p = vtc.make_params(32, 32, 128, 16, table.shape[1], "f16", SCALE)
    out = vtc.vtc_attn_decode(p, bits_to_tensor(q, "f16"), bits_to_tensor(k, "f16"), bits_to_tensor(v, "f16"),
                              _i32(torch, table), _i32(torch, seq))
    got = OA.widen(tensor_to_bits(out), "f16")
    v0 = OA.widen(v[table[0, 0], :, 0, :], "f16")
    assert np.array_equal(got[0], v0)           # one key: the value itself, exactly
    vals = np.stack([OA.gather_sequence(v, table[1], 200, h, "f16") for h in range(32)])  # [H, S, D]
    assert np.abs(got[1] - vals.mean(axis=1)).max() <= 1e-3


def _params_pair(st, scale=SCALE):
    sh = st.batch.shape
    mk = lambda out: vtc.make_params(sh.num_q_heads, sh.num_kv_heads, 128, 16, st.max_blocks_per_seq, sh.dtype, scale, out)
    return mk(None), mk("f32")


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_decode_configs_every_element(torch, cfg):
    # all five configurations at full size, in the launch configuration the benchmark times (caller-held
    # workspace), every output element against the oracle, with the flat tolerance on both output formats
    say(f"decode config {cfg}: every output element")
    b = make_step_batch(cfg)
    st = make_device_step(b, host_random=cfg <= 2)
    sh = b.shape
    p16, p32 = _params_pair(st)
    ws = torch.empty(vtc.vtc_attn_workspace_bytes(p16, b.num_decode, 0), dtype=torch.uint8, device="cuda")
    out16 = torch.full_like(st.q, float("nan"))
    out32 = torch.full(st.q.shape, float("nan"), dtype=torch.float32, device="cuda")
    vtc.vtc_attn_decode(p16, st.q, st.k_cache, st.v_cache, st.block_table, st.seq_lens, out=out16, workspace=ws)
    vtc.vtc_attn_decode(p32, st.q, st.k_cache, st.v_cache, st.block_table, st.seq_lens, out=out32, workspace=ws)
    torch.cuda.synchronize()
    want = full_decode_oracle(st, SCALE)
    say(f"  {want.shape[0]} requests x {want.shape[1]} heads, {int(b.seq_lens.sum())} context tokens, "
        f"max |o| {np.abs(want).max():.3f}")
    check_both_outputs(out16, out32, want, sh.dtype, f"cfg{cfg} decode", flat_only=True)
    # a second call into the same workspace gives the same bits (no stale state, deterministic order)
    out2 = torch.empty_like(st.q)
    vtc.vtc_attn_decode(p16, st.q, st.k_cache, st.v_cache, st.block_table, st.seq_lens, out=out2, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out16.view(torch.int16), out2.view(torch.int16))


# ------------------------------------------------------------------- prefill
def _prefill_case(torch, q_lens, seq_lens, hq, hkv, dtype, seed, poison=False, scale=SCALE, label="prefill"):
    """One prefill-chunk call with 16-bit and one with fp32 output rows, both checked against the oracle."""
    rng = np.random.default_rng(seed)
    table, nb = make_block_table(rng, seq_lens, 16)
    cu = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    q, k, v = make_qkv_numpy(rng, int(cu[-1]), hq, hkv, 128, nb, 16, dtype)
    if poison:
        poison_unused_rows(k, table, seq_lens, NAN_BITS[dtype])
        poison_unused_rows(v, table, seq_lens, NAN_BITS[dtype])
    args = (bits_to_tensor(q, dtype), _i32(torch, cu), int(max(q_lens)), bits_to_tensor(k, dtype),
            bits_to_tensor(v, dtype), _i32(torch, table), _i32(torch, seq_lens))
    out16 = vtc.vtc_attn_prefill_chunk(vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, scale), *args)
    out32 = vtc.vtc_attn_prefill_chunk(vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, scale, "f32"), *args)
    torch.cuda.synchronize()
    want = OA.paged_prefill_chunk(q, cu, k, v, table, seq_lens, scale, dtype)
    got = check_both_outputs(out16, out32, want, dtype, label)
    return got, want


PF_Q = [1, 5, 16, 17, 63, 64, 65, 100, 130, 256]
PF_S = [1, 5, 16, 40, 63, 200, 65, 100, 400, 512]


@pytest.mark.parametrize("dtype,hq,hkv", [("bf16", 8, 2), ("f16", 4, 4), ("bf16", 32, 8), ("f16", 8, 1)])
def test_prefill_chunk_ragged_matches_the_oracle(torch, dtype, hq, hkv):
    say(f"prefill ragged dtype={dtype} Hq={hq} Hkv={hkv}")
    got, want = _prefill_case(torch, PF_Q, PF_S, hq, hkv, dtype, seed=41, poison=True)
    err = np.abs(got - want)
    say(f"  max abs err {err.max():.3e}  max |o| {np.abs(want).max():.3f}")


@pytest.mark.parametrize("scale", [-0.07, 0.0, 0.4])
@pytest.mark.parametrize("dtype,hq,hkv", [("f16", 4, 4), ("bf16", 8, 2)])
def test_negative_zero_and_large_scales(torch, scale, dtype, hq, hkv):
    # the scale is the caller's: a negative one turns the softmax towards the smallest logits, zero makes every
    # visible key weigh the same, a large one lets a single key dominate; MHA (vector path) and GQA (matrix path)
    say(f"scale {scale} dtype={dtype} Hq={hq} Hkv={hkv}")
    got, want = _decode_case(torch, [1, 17, 100, 300, 0, 64], hq, hkv, dtype, seed=51, scale=scale)
    say(f"  decode max abs err {np.abs(got - want).max():.3e}")
    got, want = _prefill_case(torch, [5, 70, 33], [5, 150, 33], hq, hkv, dtype, seed=52, scale=scale)
    say(f"  prefill max abs err {np.abs(got - want).max():.3e}")


def test_decode_at_the_capacity_of_the_block_table(torch):
    # a context that fills every block of its table row, and one beyond it: lengths are clamped to the capacity
    say("decode at block-table capacity")
    rng = np.random.default_rng(53)
    cap = 5 * 16
    table, nb = make_block_table(rng, [cap, cap, 7], 16)
    assert table.shape[1] == 5
    q, k, v = make_qkv_numpy(rng, 3, 8, 2, 128, nb, 16, "f16")
    args = (bits_to_tensor(q, "f16"), bits_to_tensor(k, "f16"), bits_to_tensor(v, "f16"), _i32(torch, table),
            _i32(torch, [cap, cap + 1000, 7]))
    out16 = vtc.vtc_attn_decode(vtc.make_params(8, 2, 128, 16, 5, "f16", SCALE), *args)
    out32 = vtc.vtc_attn_decode(vtc.make_params(8, 2, 128, 16, 5, "f16", SCALE, "f32"), *args)
    torch.cuda.synchronize()
    want = OA.paged_decode(q, k, v, table, [cap, cap, 7], SCALE, "f16")
    check_both_outputs(out16, out32, want, "f16", "decode at capacity")


@pytest.mark.parametrize("chunk", [0, 1])
def test_prefill_config5_chunks_every_element_and_decode_consistency(torch, chunk):
    say(f"prefill config 5 chunk {chunk}: every output element")
    b = make_step_batch(5, prefill_chunk=chunk)
    st = make_device_step(b)
    sh = b.shape
    p16, p32 = _params_pair(st)
    out16 = torch.full_like(st.pf_q, float("nan"))
    out32 = torch.full(st.pf_q.shape, float("nan"), dtype=torch.float32, device="cuda")
    for p, out in ((p16, out16), (p32, out32)):
        vtc.vtc_attn_prefill_chunk(p, st.pf_q, st.pf_cu_q_lens, st.pf_max_q_len, st.k_cache, st.v_cache,
                                   st.pf_block_table, st.pf_seq_lens, out=out)
    torch.cuda.synchronize()
    want = full_prefill_oracle(st, SCALE)
    say(f"  {want.shape[0]} chunk tokens x {want.shape[1]} heads, max |o| {np.abs(want).max():.3f}")
    # a chunk token early in a first chunk sees only a few keys, so |o| >= 4 does occur here (chunk 0 only)
    check_both_outputs(out16, out32, want, sh.dtype, f"cfg5 prefill chunk {chunk}", flat_only=chunk == 1)
    # the last chunk token attends to the whole context: same answer as a decode call at that length
    last_rows = (st.pf_cu_q_lens[1:] - 1).long()
    q_last = st.pf_q[last_rows].contiguous()
    dec = vtc.vtc_attn_decode(p32, q_last, st.k_cache, st.v_cache, st.pf_block_table, st.pf_seq_lens)
    torch.cuda.synchronize()
    diff = (dec.double() - out32[last_rows].double()).abs().max().item()
    say(f"  prefill last row vs decode (fp32 rows): {diff:.3e}")
    assert diff <= 1e-3


@pytest.mark.parametrize("dtype,hq,hkv", [("bf16", 8, 2), ("f16", 4, 4)])
def test_prefill_chunk_longer_than_its_context_gives_zero_rows(torch, dtype, hq, hkv):
    # seq_lens[r] < chunk length (0 included) is a caller slip with a stated outcome: zero rows for that sequence,
    # and its block-table row -- here filled with an id far outside the cache -- is never followed
    say(f"prefill with inconsistent sequences dtype={dtype} Hq={hq} Hkv={hkv}")
    rng = np.random.default_rng(77)
    q_lens = [40, 33, 5, 100, 64]
    seq = [40, 20, 0, 99, 200]
    table, nb = make_block_table(rng, seq, 16, pad_value=1 << 30)
    table[1, :] = 1 << 30
    table[3, :] = 1 << 30
    cu = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    q, k, v = make_qkv_numpy(rng, int(cu[-1]), hq, hkv, 128, nb, 16, dtype)
    args = (bits_to_tensor(q, dtype), _i32(torch, cu), max(q_lens), bits_to_tensor(k, dtype), bits_to_tensor(v, dtype),
            _i32(torch, table), _i32(torch, seq))
    out16 = vtc.vtc_attn_prefill_chunk(vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE), *args,
                                       out=torch.full((int(cu[-1]), hq, 128), float("nan"), device="cuda",
                                                      dtype=torch.float16 if dtype == "f16" else torch.bfloat16))
    out32 = vtc.vtc_attn_prefill_chunk(vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE, "f32"), *args,
                                       out=torch.full((int(cu[-1]), hq, 128), float("nan"), device="cuda"))
    torch.cuda.synchronize()
    want = OA.paged_prefill_chunk(q, cu, k, v, table, seq, SCALE, dtype)
    got = check_both_outputs(out16, out32, want, dtype, "prefill, inconsistent sequences")
    for r in (1, 2, 3):
        assert (got[cu[r]:cu[r + 1]] == 0).all()
    assert np.abs(got[:40]).sum() > 0 and np.abs(got[cu[4]:]).sum() > 0


def test_prefill_chunking_is_invisible_on_the_gpu(torch):
    # a prompt prefilled in one call or in two chunks gives the same rows: a row's keys, their tiling and the order
    # of its online-softmax updates do not depend on where the chunk boundary falls, so the bits are equal
    say("prefill: one chunk vs two chunks")
    rng = np.random.default_rng(71)
    total, first = 200, 72
    hq, hkv, dtype = 8, 2, "bf16"
    table, nb = make_block_table(rng, [total], 16)
    q, k, v = make_qkv_numpy(rng, total, hq, hkv, 128, nb, 16, dtype)
    p = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE)
    kd, vd, td = bits_to_tensor(k, dtype), bits_to_tensor(v, dtype), _i32(torch, table)
    qd = bits_to_tensor(q, dtype)
    whole = vtc.vtc_attn_prefill_chunk(p, qd, _i32(torch, [0, total]), total, kd, vd, td, _i32(torch, [total]))
    part0 = vtc.vtc_attn_prefill_chunk(p, qd[:first].contiguous(), _i32(torch, [0, first]), first, kd, vd, td,
                                       _i32(torch, [first]))
    part1 = vtc.vtc_attn_prefill_chunk(p, qd[first:].contiguous(), _i32(torch, [0, total - first]), total - first, kd,
                                       vd, td, _i32(torch, [total]))
    torch.cuda.synchronize()
    assert torch.equal(whole[:first].view(torch.int16), part0.view(torch.int16))
    assert torch.equal(whole[first:].view(torch.int16), part1.view(torch.int16))
    want = OA.paged_prefill_chunk(q, [0, total], k, v, table, [total], SCALE, dtype)
    whole32 = vtc.vtc_attn_prefill_chunk(vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE, "f32"), qd,
                                         _i32(torch, [0, total]), total, kd, vd, td, _i32(torch, [total]))
    torch.cuda.synchronize()
    check_both_outputs(whole, whole32, want, dtype, "prefill in one chunk")


# ----------------------------------------------------------- extreme logits
@pytest.mark.parametrize("dtype,hq,hkv", [("f16", 4, 4), ("bf16", 8, 2)])
def test_peaked_softmax_with_large_logits(torch, dtype, hq, hkv):
    # keys six times larger: logits spread over hundreds of units (log2 domain), so almost all weights underflow
    # to zero and one or two keys carry the row; nothing may overflow, and rows past seq_len stay out of it
    say(f"large logits dtype={dtype} Hq={hq} Hkv={hkv}")
    rng = np.random.default_rng(61)
    seq = [1, 9, 64, 300, 17]
    table, nb = make_block_table(rng, seq, 16)
    q, k, v = make_qkv_numpy(rng, len(seq), hq, hkv, 128, nb, 16, dtype)
    from workloads.tensors import f32_to_storage_bits
    k = f32_to_storage_bits((6.0 * OA.widen(k, dtype)).astype(np.float32), dtype)
    poison_unused_rows(k, table, seq, NAN_BITS[dtype])
    poison_unused_rows(v, table, seq, NAN_BITS[dtype])
    p = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE)
    p32 = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE, "f32")
    kd, vd, td = bits_to_tensor(k, dtype), bits_to_tensor(v, dtype), _i32(torch, table)
    out = vtc.vtc_attn_decode(p, bits_to_tensor(q, dtype), kd, vd, td, _i32(torch, seq))
    out32 = vtc.vtc_attn_decode(p32, bits_to_tensor(q, dtype), kd, vd, td, _i32(torch, seq))
    torch.cuda.synchronize()
    want = OA.paged_decode(q, k, v, table, seq, SCALE, dtype)
    say(f"  largest weight {max(OA.softmax_weights(OA.widen(q[3, 0], dtype), OA.gather_sequence(k, table[3], 300, 0, dtype), SCALE)):.3f}")
    check_both_outputs(out, out32, want, dtype, "decode, peaked softmax")
    # the same cache as one prefill chunk per sequence (whole prompts)
    cu = np.concatenate([[0], np.cumsum(seq)]).astype(np.int32)
    rng2 = np.random.default_rng(62)
    qp = f32_to_storage_bits(rng2.standard_normal((int(cu[-1]), hq, 128), dtype=np.float32), dtype)
    outp = vtc.vtc_attn_prefill_chunk(p, bits_to_tensor(qp, dtype), _i32(torch, cu), max(seq), kd, vd, td, _i32(torch, seq))
    outp32 = vtc.vtc_attn_prefill_chunk(p32, bits_to_tensor(qp, dtype), _i32(torch, cu), max(seq), kd, vd, td, _i32(torch, seq))
    torch.cuda.synchronize()
    wantp = OA.paged_prefill_chunk(qp, cu, k, v, table, seq, SCALE, dtype)
    check_both_outputs(outp, outp32, wantp, dtype, "prefill, peaked softmax")


# ------------------------------------------------------------- random shapes
@pytest.mark.parametrize("dtype,hq,hkv", [("bf16", 8, 2), ("f16", 4, 4)])
def test_contexts_far_beyond_the_workload_lengths(torch, dtype, hq, hkv):
    # one sequence spread over every resident wave (thousands of partial results to merge) next to tiny ones,
    # and prefill chunks that sit at the end of long contexts
    say(f"long contexts dtype={dtype} Hq={hq} Hkv={hkv}")
    got, want = _decode_case(torch, [65536, 3, 40000, 1, 16], hq, hkv, dtype, seed=83)
    say(f"  decode max abs err {np.abs(got - want).max():.3e}")
    got, want = _prefill_case(torch, [100, 7, 33], [30000, 9001, 33], hq, hkv, dtype, seed=84)
    say(f"  prefill max abs err {np.abs(got - want).max():.3e}")


@pytest.mark.parametrize("seed", range(10))
def test_decode_and_prefill_on_random_small_shapes(torch, seed):
    # seeded draws over what the fixed cases do not cross: group size x dtype x batch size x length mix
    # (empty sequences, single tokens, lengths on and off block and tile boundaries) x block-table width
    rng = np.random.default_rng(9000 + seed)
    hkv = int(rng.choice([1, 2, 4, 8]))
    group = int(rng.choice([1, 2, 4, 8]))
    dtype = str(rng.choice(["f16", "bf16"]))
    n = int(rng.integers(1, 40))
    kinds = rng.integers(0, 5, size=n)
    seq = np.where(kinds == 0, 0, np.where(kinds == 1, rng.integers(1, 4, size=n),
                   np.where(kinds == 2, 16 * rng.integers(1, 9, size=n), rng.integers(1, 200, size=n)))).astype(np.int32)
    say(f"random shapes seed {seed}: Hq={hkv * group} Hkv={hkv} {dtype} n={n} lens {seq.min()}..{seq.max()}")
    got, want = _decode_case(torch, seq, hkv * group, hkv, dtype, seed=9100 + seed, poison=True,
                             min_row_len=int(rng.integers(0, 30)))
    say(f"  decode max abs err {np.abs(got - want).max():.3e}")
    assert (got[seq == 0] == 0).all()
    # prefill: chunks of random length ending anywhere in a context of random length
    m = int(rng.integers(1, 6))
    q_lens = rng.integers(1, 100, size=m).astype(np.int32)
    ctx = (q_lens + rng.integers(0, 150, size=m) * rng.integers(0, 2, size=m)).astype(np.int32)
    got, want = _prefill_case(torch, q_lens, ctx, hkv * group, hkv, dtype, seed=9200 + seed, poison=True)
    say(f"  prefill q_lens {q_lens.tolist()} ctx {ctx.tolist()} max abs err {np.abs(got - want).max():.3e}")


# ---------------------------------------------------------------- whole step
def test_mixed_step_config5_on_one_stream(torch):
    say("mixed step: prefill chunk + decode + one counter update")
    b = make_step_batch(5)
    st = make_device_step(b)
    sh = b.shape
    p = vtc.make_params(sh.num_q_heads, sh.num_kv_heads, 128, 16, st.max_blocks_per_seq, sh.dtype, SCALE)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        pf = vtc.vtc_attn_prefill_chunk(p, st.pf_q, st.pf_cu_q_lens, st.pf_max_q_len, st.k_cache, st.v_cache,
                                        st.pf_block_table, st.pf_seq_lens)
        dec = vtc.vtc_attn_decode(p, st.q, st.k_cache, st.v_cache, st.block_table, st.seq_lens)
        vtc.vtc_counter_update(st.counters, st.cu_client_ids, st.cu_n_in, st.cu_n_out, b.w_p, b.w_q)
    stream.synchronize()
    ids, n_in, n_out = b.counter_update_args()
    assert st.counters.cpu().tolist() == oracle_counter_update(b.counters_before, ids, n_in, n_out, b.w_p, b.w_q)
    assert sum(st.counters.cpu().tolist()) == 1 * 16 * 512 + 2 * 256
    from tests.helpers import check_storage_output
    check_storage_output(dec.double().cpu().numpy(), full_decode_oracle(st, SCALE), sh.dtype, "mixed step decode", flat_only=True)
    check_storage_output(pf.double().cpu().numpy(), full_prefill_oracle(st, SCALE), sh.dtype, "mixed step prefill")
