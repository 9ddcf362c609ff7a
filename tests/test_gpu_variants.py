"""Parity of the cost-function, weighted, length-prediction counter updates and of KV append with the CPU
oracle, through the C ABI (needs an MI355X).  All of these are bit-exact."""
import math
import sys

import numpy as np
import pytest

import paper_2401_00588_amd as vtc
from oracle import attention as OA
from oracle.counters import (PROFILED_MILLI, CostPoly, counter_update, counter_update_cost,
                             counter_update_predicted)
from oracle.scheduler import VTCScheduler, simulate
from workloads import (NAN_BITS, bits_to_tensor, make_block_table, make_qkv_numpy, make_step_batch, tensor_to_bits)
from workloads.traces import fixed_lengths, poisson_trace, uniform_lengths

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


def _i64(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int64)).cuda()


def _poly(h: CostPoly) -> vtc.CostPoly:
    return vtc.CostPoly(*h.coefficients())


@pytest.mark.parametrize("n,clients,seed", [(8, 2, 0), (528, 8, 1), (5000, 27, 2), (9000, 5000, 3)])
@pytest.mark.parametrize("which", ["profiled", "linear", "full_quadratic"])
def test_cost_function_update_is_bit_exact(torch, n, clients, seed, which):
    say(f"counter_update_cost {which} n={n} clients={clients}")
    h = {"profiled": PROFILED_MILLI, "linear": CostPoly(0, 1, 2, 0, 0, 0),
         "full_quadratic": CostPoly(-7, 3, -5, 11, 13, 17)}[which]
    rng = np.random.default_rng(seed)
    ids = rng.integers(-2, clients + 2, size=n).astype(np.int32)
    po = rng.integers(0, 4097, size=n).astype(np.int32)
    qo = rng.integers(0, 2049, size=n).astype(np.int32)
    fresh = rng.random(n) < 0.2                      # requests seen for the first time
    po[fresh] = 0
    qo[fresh] = 0
    pn = (po + rng.integers(0, 513, size=n)).astype(np.int32)
    qn = (qo + rng.integers(0, 2, size=n)).astype(np.int32)
    base = rng.integers(0, 1 << 40, size=clients).astype(np.int64)
    mult = rng.integers(1, 13, size=clients).astype(np.int64)
    for use_mult in (False, True):
        c = torch.from_numpy(base.copy()).cuda()
        vtc.vtc_counter_update_cost(c, _i32(torch, ids), _i32(torch, po), _i32(torch, qo), _i32(torch, pn),
                                    _i32(torch, qn), _poly(h), _i64(torch, mult) if use_mult else None)
        want = counter_update_cost(base, ids, po, qo, pn, qn, h, mult if use_mult else None)
        assert c.cpu().tolist() == want
    if which == "linear":                            # the plain entry point computes the same thing
        c = torch.from_numpy(base.copy()).cuda()
        vtc.vtc_counter_update(c, _i32(torch, ids), _i32(torch, pn - po), _i32(torch, qn - qo), 1, 2)
        assert c.cpu().tolist() == counter_update_cost(base, ids, po, qo, pn, qn, h)


def test_profiled_cost_over_a_scheduler_run(torch):
    # replay a CPU scheduler run (Algorithm 4 with the paper's profiled cost) step by step on the device counters
    say("profiled cost replay")
    trace = poisson_trace([4.0, 1.0, 2.0], 12.0, [fixed_lengths(64, 64), fixed_lengths(256, 128), uniform_lengths(8, 300, 1, 90)], seed=8)
    sched = VTCScheduler(3, 1, 2, 10000, 256, lift=False, cost=PROFILED_MILLI)
    dev = torch.zeros(3, dtype=torch.int64).cuda()
    h = _poly(PROFILED_MILLI)
    steps = 0

    def on_step(rec):
        nonlocal steps
        if rec.admitted:
            ids = [x.client for x in rec.admitted]
            zeros = [0] * len(ids)
            vtc.vtc_counter_update_cost(dev, _i32(torch, ids), _i32(torch, zeros), _i32(torch, zeros),
                                        _i32(torch, [x.n_input for x in rec.admitted]), _i32(torch, zeros), h)
        gen = rec.decode_generated_before
        vtc.vtc_counter_update_cost(dev, _i32(torch, rec.decode_clients), _i32(torch, rec.decode_n_input),
                                    _i32(torch, gen), _i32(torch, rec.decode_n_input),
                                    _i32(torch, [g + 1 for g in gen]), h)
        steps += 1
        if steps % 50 == 0:
            assert dev.cpu().tolist() == rec.counters_after_decode_charge
        return False

    simulate(trace, sched, 0.045, 2e-4, on_step=on_step)
    assert steps > 100 and dev.cpu().tolist() == sched.c


@pytest.mark.parametrize("n,clients,seed", [(8, 2, 0), (528, 8, 1), (6000, 27, 2)])
def test_length_prediction_adjustment_is_bit_exact(torch, n, clients, seed):
    say(f"counter_update_predicted n={n} clients={clients}")
    rng = np.random.default_rng(seed)
    ids = rng.integers(-1, clients + 1, size=n).astype(np.int32)
    pred = rng.integers(0, 300, size=n).astype(np.int32)
    out = np.maximum(1, pred + rng.integers(-40, 41, size=n)).astype(np.int32)
    fin = (rng.random(n) < 0.3).astype(np.int32)
    base = rng.integers(0, 1 << 40, size=clients).astype(np.int64)
    c = torch.from_numpy(base.copy()).cuda()
    vtc.vtc_counter_update_predicted(c, _i32(torch, ids), _i32(torch, out), _i32(torch, pred), _i32(torch, fin), 2)
    assert c.cpu().tolist() == counter_update_predicted(base, ids, out, pred, fin, 2)


def test_length_prediction_life_of_a_request_on_the_device(torch):
    say("prediction telescopes on the device")
    for pred in (0, 4, 10, 25):
        c = torch.zeros(1, dtype=torch.int64).cuda()
        vtc.vtc_counter_update(c, _i32(torch, [0]), _i32(torch, [17]), _i32(torch, [pred]), 1, 2)
        for out in range(1, 11):
            vtc.vtc_counter_update_predicted(c, _i32(torch, [0]), _i32(torch, [out]), _i32(torch, [pred]),
                                             _i32(torch, [1 if out == 10 else 0]), 2)
        assert c.cpu().tolist() == [17 + 2 * 10]


@pytest.mark.parametrize("dtype,hkv", [("f16", 32), ("bf16", 8)])
def test_kv_append_is_bit_exact_and_feeds_attention(torch, dtype, hkv):
    say(f"kv_append dtype={dtype} Hkv={hkv}")
    rng = np.random.default_rng(70 + hkv)
    hq = 32
    seq_after = np.array([1, 16, 17, 40, 300, 512, 5, 64], dtype=np.int32)
    n_new = np.array([1, 1, 1, 40, 256, 0, 5, 1], dtype=np.int32)   # decode tokens, whole prompts, a chunk, nothing
    table, nb = make_block_table(rng, seq_after, 16)
    q, k_full, v_full = make_qkv_numpy(rng, len(seq_after), hq, hkv, 128, nb, 16, dtype)
    # device cache holds NaN where the new tokens go; everything else as in the full cache
    k_dev, v_dev = k_full.copy(), v_full.copy()
    new_k, new_v = [], []
    for r, (s, n) in enumerate(zip(seq_after, n_new)):
        for p in range(s - n, s):
            blk, row = table[r, p // 16], p % 16
            new_k.append(k_full[blk, :, row, :].copy())
            new_v.append(v_full[blk, :, row, :].copy())
            k_dev[blk, :, row, :] = NAN_BITS[dtype]
            v_dev[blk, :, row, :] = NAN_BITS[dtype]
    new_k, new_v = np.stack(new_k), np.stack(new_v)
    cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    p = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE)
    kc, vc = bits_to_tensor(k_dev, dtype), bits_to_tensor(v_dev, dtype)
    vtc.vtc_kv_append(p, bits_to_tensor(new_k, dtype), bits_to_tensor(new_v, dtype), _i32(torch, cu), int(n_new.max()),
                      kc, vc, _i32(torch, table), _i32(torch, seq_after))
    torch.cuda.synchronize()
    # bit-exact against the oracle's append and against the original full cache
    k_or, v_or = k_dev.copy(), v_dev.copy()
    OA.kv_append(k_or, v_or, new_k, new_v, cu, table, seq_after)
    assert np.array_equal(tensor_to_bits(kc), k_or) and np.array_equal(tensor_to_bits(vc), v_or)
    assert np.array_equal(k_or, k_full) and np.array_equal(v_or, v_full)
    # and attention over the appended cache is the attention over the full cache
    out = vtc.vtc_attn_decode(p, bits_to_tensor(q, dtype), kc, vc, _i32(torch, table), _i32(torch, seq_after))
    want = OA.paged_decode(q, k_full, v_full, table, seq_after, SCALE, dtype)
    assert np.abs(OA.widen(tensor_to_bits(out), dtype) - want).max() <= {"f16": 2e-3, "bf16": 1e-2}[dtype]


def test_weighted_vtc_on_a_config_batch(torch):
    say("weighted VTC multipliers on config 3")
    b = make_step_batch(3)
    ids, n_in, n_out = b.counter_update_args()
    zeros = np.zeros_like(n_in)
    mult = np.array([12, 6, 4, 3], dtype=np.int64)               # weights 1 : 2 : 3 : 4
    h = CostPoly(0, b.w_p, b.w_q, 0, 0, 0)
    c = torch.zeros(4, dtype=torch.int64).cuda()
    # first update of a request is marked by old counts (0, 0); later ones pass the running totals
    vtc.vtc_counter_update_cost(c, _i32(torch, ids), _i32(torch, zeros + 7), _i32(torch, zeros + 3),
                                _i32(torch, zeros + 7 + n_in), _i32(torch, zeros + 3 + n_out), _poly(h), _i64(torch, mult))
    want = counter_update_cost([0] * 4, ids, zeros + 7, zeros + 3, zeros + 7 + n_in, zeros + 3 + n_out, h, mult)
    assert c.cpu().tolist() == want
    plain = counter_update([0] * 4, ids, n_in, n_out, b.w_p, b.w_q)
    assert want == [int(m) * x for m, x in zip(mult, plain)]
