"""Pins for the counter-charge and slot-index oracles (CPU only)."""
import numpy as np
import pytest

from oracle.counters import counter_update, gather_slots


def test_hand_example_decode_charge():
    # Algorithm 2, decode charge: c_i += w_q * |{r in B : client(r) = i}|.
    # Two clients, w_q = 2; B holds 3 requests of client 0 and 5 of client 1.
    ids = [0, 1, 1, 0, 1, 1, 0, 1]
    got = counter_update([10, 20], ids, None, [1] * 8, 1, 2)
    assert got == [10 + 6, 20 + 10]


def test_hand_example_admission_charge():
    # Algorithm 2, admission: c_k += w_p * input_length(r).
    assert counter_update([0, 0, 7], [2, 0], [300, 41], None, 1, 2) == [41, 0, 307]
    assert counter_update([0, 0, 7], [2, 0], [300, 41], None, 3, 2) == [123, 0, 907]


def test_total_charge_of_a_request_is_the_weighted_token_cost():
    # Section 3.1: W = w_p * n_p + w_q * n_q.  Charge the prompt once, then one token per step.
    rng = np.random.default_rng(0)
    for _ in range(20):
        w_p, w_q = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        n_p, n_q = int(rng.integers(1, 2000)), int(rng.integers(1, 600))
        c = counter_update([0], [0], [n_p], None, w_p, w_q)
        for _step in range(n_q):
            c = counter_update(c, [0], None, [1], w_p, w_q)
        assert c == [w_p * n_p + w_q * n_q]


def test_sum_of_increments_and_order_independence():
    rng = np.random.default_rng(1)
    n, clients = 500, 27
    ids = rng.integers(0, clients, size=n)
    n_in = rng.integers(0, 4096, size=n)
    n_out = rng.integers(0, 2, size=n)
    base = rng.integers(0, 10 ** 9, size=clients).tolist()
    got = counter_update(base, ids, n_in, n_out, 1, 2)
    assert sum(got) - sum(base) == int(n_in.sum()) + 2 * int(n_out.sum())
    perm = rng.permutation(n)
    assert counter_update(base, ids[perm], n_in[perm], n_out[perm], 1, 2) == got
    # against a vectorised library reduction
    ref = np.asarray(base, dtype=np.int64) + np.bincount(ids, weights=None, minlength=clients) * 0
    ref = ref + np.bincount(ids, weights=(n_in + 2 * n_out).astype(np.float64), minlength=clients).astype(np.int64)
    assert got == ref.tolist()


def test_out_of_range_clients_are_ignored_and_overflow_is_loud():
    assert counter_update([1, 2], [-1, 2, 1, 5], None, [1, 1, 1, 1], 1, 2) == [1, 4]
    with pytest.raises(OverflowError):
        counter_update([(1 << 63) - 2], [0], None, [1], 1, 2)


def test_negative_deltas_are_plain_integer_arithmetic():
    # a refund (negative token count) is just a signed term
    assert counter_update([100], [0, 0], None, [1, -7], 1, 2) == [100 + 2 - 14]


def test_slots_brute_force():
    table = [[7, 2, 9], [4, 0, 0]]
    assert gather_slots(table, [5, 2], 2) == [14, 15, 4, 5, 18, 8, 9]
    assert gather_slots(table, [0, 0], 16) == []
    assert gather_slots(table, [3, 1], 1) == [7, 2, 9, 4]
    rng = np.random.default_rng(2)
    bs = 16
    seq = [1, 16, 17, 250]
    tab = rng.permutation(64).reshape(4, 16)
    slots = gather_slots(tab, seq, bs)
    assert len(slots) == sum(seq)
    at = 0
    for r, s in enumerate(seq):
        for p in range(s):
            blk, row = divmod(slots[at], bs)
            assert blk == tab[r, p // bs] and row == p % bs
            at += 1
