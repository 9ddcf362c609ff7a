"""Pins for the fp64 attention oracle (CPU only).

The paper prints no attention values, so the oracle is pinned to what the
mathematics fixes: closed forms, invariants, a library routine
(torch.nn.functional.scaled_dot_product_attention in float64 on a contiguous
copy) and a brute-force loop on tiny inputs.  Each pin is aimed at a
plausible slip: missing scale, wrong GQA head mapping, causal off-by-one,
wrong slot index, reading rows past seq_len, a transposed operand.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention as A
from tests.helpers import bits_to_f64_via_torch, pack_paged
from workloads.tensors import NAN_BITS, f32_to_storage_bits

DTYPES = ["f16", "bf16"]


def _decode_case(rng, seq_lens, hq, hkv, d, bs, dtype, **kw):
    keys = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    kc, vc, table, sl = pack_paged(keys, vals, bs, dtype, rng, **kw)
    q = f32_to_storage_bits(rng.standard_normal((len(seq_lens), hq, d), dtype=np.float32), dtype)
    return q, kc, vc, table, sl, keys, vals


# ----------------------------------------------------------------- widening
@pytest.mark.parametrize("dtype", DTYPES)
def test_widen_is_exact_for_every_finite_pattern(dtype):
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    ours = A.widen(bits, dtype)
    ref = bits_to_f64_via_torch(bits, dtype)
    finite = np.isfinite(ref)
    assert np.array_equal(ours[finite], ref[finite])
    assert np.array_equal(np.isnan(ours), np.isnan(ref))


# -------------------------------------------------------------- closed forms
@pytest.mark.parametrize("dtype", DTYPES)
def test_single_key_returns_its_value_exactly(dtype):
    rng = np.random.default_rng(1)
    q, kc, vc, table, sl, _, vals = _decode_case(rng, [1, 1, 1], 4, 2, 8, 4, dtype)
    out = A.paged_decode(q, kc, vc, table, sl, 0.37, dtype)
    for r in range(3):
        v0 = bits_to_f64_via_torch(f32_to_storage_bits(vals[r][0], dtype), dtype)  # [Hkv, D]
        for h in range(4):
            assert np.array_equal(out[r, h], v0[h // 2])


@pytest.mark.parametrize("dtype", DTYPES)
def test_identical_keys_give_the_mean_of_values(dtype):
    rng = np.random.default_rng(2)
    s, hkv, d = 37, 2, 16
    key = rng.standard_normal((1, hkv, d), dtype=np.float32)
    keys = [np.repeat(key, s, axis=0)]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32)]
    kc, vc, table, sl = pack_paged(keys, vals, 16, dtype, rng)
    q = f32_to_storage_bits(rng.standard_normal((1, 4, d), dtype=np.float32), dtype)
    out = A.paged_decode(q, kc, vc, table, sl, 0.25, dtype)
    mean = bits_to_f64_via_torch(f32_to_storage_bits(vals[0], dtype), dtype).mean(axis=0)  # [Hkv, D]
    for h in range(4):
        np.testing.assert_allclose(out[0, h], mean[h // 2], rtol=0, atol=1e-14)


def test_two_and_three_key_hand_arithmetic():
    # q = (1, 0), scale = 1: logits are the first key coordinate.
    q = np.array([1.0, 0.0])
    keys = np.array([[0.0, 5.0], [1.0, -3.0]])
    vals = np.array([[1.0, 0.0], [0.0, 1.0]])
    o = A.attend_one(q, keys, vals, 1.0)
    e = math.e
    np.testing.assert_allclose(o, [1 / (1 + e), e / (1 + e)], rtol=1e-15)
    # scale = 0.5, logits 0, 1, 2 -> weights 1 : e : e^2
    keys = np.array([[0.0, 1.0], [2.0, 1.0], [4.0, 1.0]])
    vals = np.array([[3.0, 0.0], [0.0, 6.0], [9.0, 9.0]])
    o = A.attend_one(q, keys, vals, 0.5)
    z = 1 + e + e * e
    np.testing.assert_allclose(o, [(3 + 9 * e * e) / z, (6 * e + 9 * e * e) / z], rtol=1e-15)


def test_weights_are_a_probability_vector():
    rng = np.random.default_rng(3)
    for s in (1, 2, 17, 300):
        w = A.softmax_weights(rng.standard_normal(32), rng.standard_normal((s, 32)) * 4, 0.7)
        assert w.shape == (s,)
        assert (w >= 0).all()
        assert abs(w.sum() - 1.0) < 1e-14


def test_scale_is_taken_as_float32():
    rng = np.random.default_rng(4)
    q, keys, vals = rng.standard_normal(8), rng.standard_normal((5, 8)), rng.standard_normal((5, 8))
    s = 1.0 / math.sqrt(128.0)
    a = A.attend_one(q, keys, vals, s)
    b = A.attend_one(q, keys, vals, float(np.float32(s)))
    assert np.array_equal(a, b)


def test_empty_context_gives_zeros():
    rng = np.random.default_rng(5)
    q, kc, vc, table, sl, _, _ = _decode_case(rng, [3, 0, 5], 2, 2, 4, 2, "f16")
    out = A.paged_decode(q, kc, vc, table, sl, 1.0, "f16")
    assert np.array_equal(out[1], np.zeros((2, 4)))
    assert np.abs(out[0]).sum() > 0 and np.abs(out[2]).sum() > 0


def test_a_chunk_longer_than_its_context_gives_zero_rows_and_reads_no_block():
    # seq_len < chunk length is a caller slip: the rows of that sequence are zero, its block-table row (here
    # ids far outside the cache) is never followed, and the sequences around it are computed as usual
    rng = np.random.default_rng(6)
    hq, hkv, d, bs = 4, 2, 8, 4
    seq_lens = [9, 3, 0, 7]
    q_lens = [4, 5, 2, 7]
    keys = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    kc, vc, table, sl = pack_paged(keys, vals, bs, "bf16", rng)
    cu = np.concatenate([[0], np.cumsum(q_lens)])
    q = f32_to_storage_bits(rng.standard_normal((int(cu[-1]), hq, d), dtype=np.float32), "bf16")
    poisoned = table.copy()
    poisoned[1, :] = 10 ** 6
    poisoned[2, :] = -7
    out = A.paged_prefill_chunk(q, cu, kc, vc, poisoned, sl, 0.3, "bf16")
    assert np.array_equal(out[cu[1]:cu[3]], np.zeros((7, hq, d)))
    good = A.paged_prefill_chunk(q, cu, kc, vc, table, [9, 5, 2, 7], 0.3, "bf16", rows=[(0, 3, 1), (3, 6, 2)])
    assert np.array_equal(out[cu[0] + 3, 1], good[cu[0] + 3, 1]) and np.array_equal(out[cu[3] + 6, 2], good[cu[3] + 6, 2])
    assert np.abs(out[cu[0] + 3, 1]).sum() > 0


# ---------------------------------------------------------------- invariances
def test_key_permutation_invariance():
    rng = np.random.default_rng(6)
    q, keys, vals = rng.standard_normal(16), rng.standard_normal((40, 16)), rng.standard_normal((40, 16))
    perm = rng.permutation(40)
    np.testing.assert_allclose(A.attend_one(q, keys, vals, 0.3), A.attend_one(q, keys[perm], vals[perm], 0.3),
                               rtol=0, atol=1e-14)


def test_logit_shift_invariance_and_dominant_key():
    rng = np.random.default_rng(7)
    d = 16
    q = rng.standard_normal(d)
    keys, vals = rng.standard_normal((25, d)), rng.standard_normal((25, d))
    shift = rng.standard_normal(d) * 3            # same vector added to every key: all logits move by <q, shift>
    np.testing.assert_allclose(A.attend_one(q, keys, vals, 0.5), A.attend_one(q, keys + shift, vals, 0.5),
                               rtol=0, atol=1e-12)
    keys2 = keys.copy()
    keys2[11] = q * 100.0                          # one key whose logit dwarfs the others
    np.testing.assert_allclose(A.attend_one(q, keys2, vals, 1.0), vals[11], rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype", DTYPES)
def test_block_table_and_block_size_invariance(dtype):
    rng = np.random.default_rng(8)
    seq_lens = [1, 5, 16, 17, 33, 64]
    hq, hkv, d = 4, 2, 8
    keys = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    q = f32_to_storage_bits(rng.standard_normal((len(seq_lens), hq, d), dtype=np.float32), dtype)
    outs = []
    for bs, seed in ((16, 1), (16, 2), (1, 3), (4, 4)):
        kc, vc, table, sl = pack_paged(keys, vals, bs, dtype, np.random.default_rng(seed))
        outs.append(A.paged_decode(q, kc, vc, table, sl, 0.35, dtype))
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])


@pytest.mark.parametrize("dtype", DTYPES)
def test_rows_past_seq_len_and_padding_entries_are_never_read(dtype):
    rng = np.random.default_rng(9)
    seq_lens = [3, 16, 21]
    hq, hkv, d, bs = 2, 1, 8, 16
    keys = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    q = f32_to_storage_bits(rng.standard_normal((3, hq, d), dtype=np.float32), dtype)
    clean = pack_paged(keys, vals, bs, dtype, np.random.default_rng(1))
    dirty = pack_paged(keys, vals, bs, dtype, np.random.default_rng(1), fill_bits=NAN_BITS[dtype])
    a = A.paged_decode(q, *clean[:3], clean[3], 0.4, dtype)
    b = A.paged_decode(q, *dirty[:3], dirty[3], 0.4, dtype)
    assert np.isfinite(b).all() and np.array_equal(a, b)
    # padding entries of the block table point at a block full of NaN
    kc, vc, table, sl = dirty
    used = {int(x) for r, s in enumerate(seq_lens) for x in table[r, : (s + bs - 1) // bs]}
    nan_block = [b_ for b_ in range(kc.shape[0]) if b_ not in used][0]
    table2 = table.copy()
    for r, s in enumerate(seq_lens):
        table2[r, (s + bs - 1) // bs:] = nan_block
    assert np.array_equal(A.paged_decode(q, kc, vc, table2, sl, 0.4, dtype), a)


def test_gqa_equals_mha_with_replicated_kv_heads():
    rng = np.random.default_rng(10)
    dtype, hq, hkv, d, bs = "bf16", 8, 2, 16, 16
    seq_lens = [7, 30]
    keys = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    q = f32_to_storage_bits(rng.standard_normal((2, hq, d), dtype=np.float32), dtype)
    g = A.paged_decode(q, *pack_paged(keys, vals, bs, dtype, np.random.default_rng(1))[:3], seq_lens, 0.3, dtype)
    keys_m = [np.repeat(k, hq // hkv, axis=1) for k in keys]     # kv head j serves q heads 4j..4j+3
    vals_m = [np.repeat(v, hq // hkv, axis=1) for v in vals]
    m = A.paged_decode(q, *pack_paged(keys_m, vals_m, bs, dtype, np.random.default_rng(2))[:3], seq_lens, 0.3, dtype)
    assert np.array_equal(g, m)


# ------------------------------------------------- library routine as a pin
def _torch_reference(q_bits, keys, vals, dtype, scale, q_pos):
    """SDPA in float64 on dense tensors; q_pos[i] = absolute position of query i (keys 0..q_pos[i] visible)."""
    q = torch.from_numpy(bits_to_f64_via_torch(q_bits, dtype))                # [Lq, Hq, D]
    k = torch.from_numpy(bits_to_f64_via_torch(f32_to_storage_bits(keys, dtype), dtype))   # [S, Hkv, D]
    v = torch.from_numpy(bits_to_f64_via_torch(f32_to_storage_bits(vals, dtype), dtype))
    group = q.shape[1] // k.shape[1]
    k = k.repeat_interleave(group, dim=1)
    v = v.repeat_interleave(group, dim=1)
    mask = torch.arange(k.shape[0])[None, :] <= torch.as_tensor(q_pos)[:, None]            # [Lq, S]
    o = torch.nn.functional.scaled_dot_product_attention(
        q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None],
        attn_mask=mask[None, None], scale=float(np.float32(scale)))
    return o[0].permute(1, 0, 2).numpy()                                      # [Lq, Hq, D]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2)])
def test_decode_matches_library_sdpa(dtype, hq, hkv):
    rng = np.random.default_rng(11)
    seq_lens = [1, 15, 16, 17, 100, 257]
    q, kc, vc, table, sl, keys, vals = _decode_case(rng, seq_lens, hq, hkv, 32, 16, dtype)
    scale = 1.0 / math.sqrt(32.0)
    out = A.paged_decode(q, kc, vc, table, sl, scale, dtype)
    for r, s in enumerate(seq_lens):
        ref = _torch_reference(q[r:r + 1], keys[r], vals[r], dtype, scale, [s - 1])
        np.testing.assert_allclose(out[r], ref[0], rtol=0, atol=1e-13)


@pytest.mark.parametrize("dtype", DTYPES)
def test_prefill_chunk_matches_library_sdpa_with_causal_mask(dtype):
    rng = np.random.default_rng(12)
    hq, hkv, d, bs = 4, 2, 16, 16
    seq_lens = [40, 64, 19]
    q_lens = [40, 24, 1]                      # first chunk, later chunk, single-token chunk
    keys = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_lens]
    kc, vc, table, sl = pack_paged(keys, vals, bs, dtype, rng)
    cu = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    q = f32_to_storage_bits(rng.standard_normal((int(cu[-1]), hq, d), dtype=np.float32), dtype)
    out = A.paged_prefill_chunk(q, cu, kc, vc, table, sl, 0.25, dtype)
    for r, (s, lq) in enumerate(zip(seq_lens, q_lens)):
        pos = [s - lq + i for i in range(lq)]
        ref = _torch_reference(q[cu[r]:cu[r + 1]], keys[r], vals[r], dtype, 0.25, pos)
        np.testing.assert_allclose(out[cu[r]:cu[r + 1]], ref, rtol=0, atol=1e-13)


# --------------------------------------------------------------- brute force
def _brute(q, keys, vals, scale):
    logits = [scale * sum(q[d] * k[d] for d in range(len(q))) for k in keys]
    m = max(logits)
    w = [math.exp(x - m) for x in logits]
    z = sum(w)
    return [sum(w[j] * vals[j][d] for j in range(len(keys))) / z for d in range(len(vals[0]))]


def test_brute_force_on_tiny_inputs():
    rng = np.random.default_rng(13)
    dtype, hq, hkv, d, bs = "f16", 2, 1, 3, 2
    seq_lens = [1, 2, 5]
    q, kc, vc, table, sl, keys, vals = _decode_case(rng, seq_lens, hq, hkv, d, bs, dtype)
    scale = float(np.float32(0.61))
    out = A.paged_decode(q, kc, vc, table, sl, scale, dtype)
    qf = bits_to_f64_via_torch(q, dtype)
    for r, s in enumerate(seq_lens):
        kf = bits_to_f64_via_torch(f32_to_storage_bits(keys[r], dtype), dtype)
        vf = bits_to_f64_via_torch(f32_to_storage_bits(vals[r], dtype), dtype)
        for h in range(hq):
            ref = _brute(qf[r, h].tolist(), kf[:, 0].tolist(), vf[:, 0].tolist(), scale)
            np.testing.assert_allclose(out[r, h], ref, rtol=0, atol=1e-14)


# ------------------------------------------- prefill / decode consistency
@pytest.mark.parametrize("dtype", DTYPES)
def test_prefill_row_equals_decode_at_that_position_and_chunking_is_invisible(dtype):
    rng = np.random.default_rng(14)
    hq, hkv, d, bs = 4, 2, 8, 4
    s = 23
    keys = [rng.standard_normal((s, hkv, d), dtype=np.float32)]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32)]
    kc, vc, table, _ = pack_paged(keys, vals, bs, dtype, rng)
    q = f32_to_storage_bits(rng.standard_normal((s, hq, d), dtype=np.float32), dtype)
    whole = A.paged_prefill_chunk(q, [0, s], kc, vc, table, [s], 0.5, dtype)
    # row i == decode with context i + 1
    for i in (0, 1, 7, 22):
        dec = A.paged_decode(q[i:i + 1], kc, vc, table, [i + 1], 0.5, dtype)
        assert np.array_equal(whole[i], dec[0])
    # two chunks (10 + 13 tokens) == one chunk of 23
    first = A.paged_prefill_chunk(q[:10], [0, 10], kc, vc, table, [10], 0.5, dtype)
    second = A.paged_prefill_chunk(q[10:], [0, 13], kc, vc, table, [23], 0.5, dtype)
    assert np.array_equal(np.concatenate([first, second]), whole)


def test_row_subset_computes_only_the_requested_rows():
    rng = np.random.default_rng(15)
    q, kc, vc, table, sl, _, _ = _decode_case(rng, [9, 4, 30], 4, 2, 8, 4, "f16")
    full = A.paged_decode(q, kc, vc, table, sl, 0.3, "f16")
    part = A.paged_decode(q, kc, vc, table, sl, 0.3, "f16", rows=[(2, 3), (0, 1)])
    assert np.array_equal(part[2, 3], full[2, 3]) and np.array_equal(part[0, 1], full[0, 1])
    assert np.isnan(part[1]).all()


# ------------------------------------------------------------------ KV append
def test_kv_append_puts_rows_where_attention_reads_them():
    rng = np.random.default_rng(16)
    dtype, hkv, d, bs = "f16", 2, 8, 4
    seq_after = [5, 9, 1, 16]
    n_new = [1, 4, 1, 0]
    keys = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_after]
    vals = [rng.standard_normal((s, hkv, d), dtype=np.float32) for s in seq_after]
    # cache filled with the old tokens only; the slots of the new tokens hold NaN
    kc, vc, table, _ = pack_paged(keys, vals, bs, dtype, rng)
    full_k, full_v = kc.copy(), vc.copy()
    for r, (s, n) in enumerate(zip(seq_after, n_new)):
        for p in range(s - n, s):
            kc[table[r, p // bs], :, p % bs, :] = NAN_BITS[dtype]
            vc[table[r, p // bs], :, p % bs, :] = NAN_BITS[dtype]
    cu = np.concatenate([[0], np.cumsum(n_new)])
    k_new = np.concatenate([f32_to_storage_bits(keys[r][s - n:s], dtype) for r, (s, n) in enumerate(zip(seq_after, n_new))])
    v_new = np.concatenate([f32_to_storage_bits(vals[r][s - n:s], dtype) for r, (s, n) in enumerate(zip(seq_after, n_new))])
    A.kv_append(kc, vc, k_new, v_new, cu, table, seq_after)
    assert np.array_equal(kc, full_k) and np.array_equal(vc, full_v)       # exactly the new slots were written
    for r, s in enumerate(seq_after):
        for g in range(hkv):
            got = A.gather_sequence(kc, table[r], s, g, dtype)
            want = bits_to_f64_via_torch(f32_to_storage_bits(keys[r][:, g], dtype), dtype)
            assert np.array_equal(got, want)
