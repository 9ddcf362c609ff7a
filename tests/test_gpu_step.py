"""The fused decode step (attention + counter charge in one call) against the CPU oracle, through the
C ABI (needs an MI355X).  Attention within the floating-point tolerance, counters bit-exact."""
import math
import sys

import numpy as np
import pytest

import paper_2401_00588_amd as vtc
from oracle import attention as OA
from oracle.counters import counter_update
from tests.helpers import check_storage_output, full_decode_oracle, within_tolerance
from workloads import (bits_to_tensor, make_block_table, make_device_step, make_qkv_numpy, make_step_batch,
                       sequence_rows_to_host, tensor_to_bits)

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


def _case(torch, seq, hq, hkv, dtype, seed, clients, n_requests, with_inputs=True):
    rng = np.random.default_rng(seed)
    table, nb = make_block_table(rng, seq, 16)
    q, k, v = make_qkv_numpy(rng, len(seq), hq, hkv, 128, nb, 16, dtype)
    ids = rng.integers(-1, clients + 1, size=n_requests).astype(np.int32)      # a few ids out of range
    n_in = rng.integers(0, 2049, size=n_requests).astype(np.int32) if with_inputs else None
    n_out = rng.integers(0, 2, size=n_requests).astype(np.int32)
    before = rng.integers(-10 ** 12, 10 ** 12, size=clients).astype(np.int64)
    counters = _i64(torch, before)
    p = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE)
    out = vtc.vtc_step_decode(p, bits_to_tensor(q, dtype), bits_to_tensor(k, dtype), bits_to_tensor(v, dtype),
                              _i32(torch, table), _i32(torch, seq), counters, _i32(torch, ids),
                              None if n_in is None else _i32(torch, n_in), _i32(torch, n_out), 1, 2)
    torch.cuda.synchronize()
    got = OA.widen(tensor_to_bits(out), dtype)
    want = OA.paged_decode(q, k, v, table, seq, SCALE, dtype)
    want_c = counter_update(before.tolist(), ids.tolist(), None if n_in is None else n_in.tolist(), n_out.tolist(), 1, 2)
    return got, want, counters.cpu().tolist(), want_c


@pytest.mark.parametrize("dtype,hq,hkv,clients,extra", [("f16", 32, 32, 2, 0), ("bf16", 32, 8, 27, 16),
                                                        ("f16", 8, 4, 700, 3000)])
def test_step_decode_matches_the_oracle(torch, dtype, hq, hkv, clients, extra):
    # extra > 0: the charge covers more requests than the attention (a mixed step); 700 clients do not fit
    # the on-chip table of the fused charge, which then adds to the counters request by request
    say(f"step_decode dtype={dtype} Hq={hq} Hkv={hkv} clients={clients} extra requests={extra}")
    seq = [1, 2, 16, 17, 100, 255, 256, 257, 513, 700, 0, 33]
    got, want, c_got, c_want = _case(torch, seq, hq, hkv, dtype, 910 + clients, clients, len(seq) + extra)
    err = np.abs(got - want).max()
    say(f"  max abs err {err:.3e}")
    assert within_tolerance(got, want, dtype)
    assert c_got == c_want


@pytest.mark.parametrize("n", [1500, 1024])
def test_step_decode_large_batches_both_planning_paths(torch, n):
    say(f"step_decode {n} sequences")
    rng = np.random.default_rng(n)
    seq = rng.integers(0, 30, size=n).astype(np.int32)
    seq[rng.integers(0, n, size=3)] = 400
    got, want, c_got, c_want = _case(torch, seq, 4, 2, "bf16", 920 + n, 40, n, with_inputs=False)
    say(f"  max abs err {np.abs(got - want).max():.3e}  max |o| {np.abs(want).max():.3f}")
    assert within_tolerance(got, want, "bf16")
    assert c_got == c_want


def test_step_decode_halves_alone(torch):
    say("step_decode: charge alone, attention alone")
    rng = np.random.default_rng(930)
    ids = rng.integers(0, 5, size=300).astype(np.int32)
    n_out = np.ones(300, dtype=np.int32)
    counters = _i64(torch, np.zeros(5, dtype=np.int64))
    p = vtc.make_params(4, 4, 128, 16, 4, "f16", SCALE)
    empty = torch.empty((0, 4, 128), dtype=torch.float16, device="cuda")
    cache = torch.zeros((1, 4, 16, 128), dtype=torch.float16, device="cuda")
    vtc.vtc_step_decode(p, empty, cache, cache, torch.empty((0, 4), dtype=torch.int32, device="cuda"),
                        torch.empty((0,), dtype=torch.int32, device="cuda"), counters, _i32(torch, ids), None,
                        _i32(torch, n_out), 1, 2)
    torch.cuda.synchronize()
    assert counters.cpu().tolist() == counter_update([0] * 5, ids.tolist(), None, n_out.tolist(), 1, 2)
    # no requests to charge: the counters stay as they are, the attention still runs
    seq = [5, 40]
    table, nb = make_block_table(rng, seq, 16)
    q, k, v = make_qkv_numpy(rng, 2, 4, 4, 128, nb, 16, "f16")
    p = vtc.make_params(4, 4, 128, 16, table.shape[1], "f16", SCALE)
    before = counters.clone()
    out = vtc.vtc_step_decode(p, bits_to_tensor(q, "f16"), bits_to_tensor(k, "f16"), bits_to_tensor(v, "f16"),
                              _i32(torch, table), _i32(torch, seq), counters,
                              torch.empty((0,), dtype=torch.int32, device="cuda"), None, None, 1, 2)
    torch.cuda.synchronize()
    assert torch.equal(before, counters)
    want = OA.paged_decode(q, k, v, table, seq, SCALE, "f16")
    assert within_tolerance(OA.widen(tensor_to_bits(out), "f16"), want, "f16")


@pytest.mark.parametrize("cfg", [3, 5])
def test_step_decode_on_the_config_batches(torch, cfg):
    # the launch configuration the benchmark times: counters bit-exact against the oracle, every attention
    # output element against the oracle; repeated steps keep accumulating exactly
    say(f"step_decode on cfg{cfg}")
    b = make_step_batch(cfg)
    st = make_device_step(b)
    sh = b.shape
    p = vtc.make_params(sh.num_q_heads, sh.num_kv_heads, 128, 16, st.max_blocks_per_seq, sh.dtype, SCALE)
    ws = torch.empty(vtc.vtc_attn_workspace_bytes(p, b.num_decode, 0), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(st.q)
    for _ in range(3):
        vtc.vtc_step_decode(p, st.q, st.k_cache, st.v_cache, st.block_table, st.seq_lens, st.counters,
                            st.cu_client_ids, st.cu_n_in, st.cu_n_out, b.w_p, b.w_q, out=out, workspace=ws)
    torch.cuda.synchronize()
    ids, n_in, n_out = b.counter_update_args()
    want_c = list(b.counters_before)
    for _ in range(3):
        want_c = counter_update(want_c, ids, n_in, n_out, b.w_p, b.w_q)
    assert st.counters.cpu().tolist() == want_c
    check_storage_output(out.double().cpu().numpy(), full_decode_oracle(st, SCALE), sh.dtype,
                         f"step_decode cfg{cfg}", flat_only=True)


def test_step_decode_replays_from_a_hip_graph(torch):
    # a serving loop may capture the step once and replay it: the call must be capturable (no allocation, no
    # synchronisation, nothing that depends on state from capture time) and every replay must redo all of it
    say("step_decode captured into a graph and replayed")
    rng = np.random.default_rng(950)
    seq = [3, 40, 257, 0, 700, 16]
    hq, hkv, dtype, clients = 8, 2, "bf16", 4
    table, nb = make_block_table(rng, seq, 16)
    q, k, v = make_qkv_numpy(rng, len(seq), hq, hkv, 128, nb, 16, dtype)
    ids = rng.integers(0, clients, size=len(seq)).astype(np.int32)
    n_out = np.ones(len(seq), dtype=np.int32)
    p = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE)
    qd, kd, vd = bits_to_tensor(q, dtype), bits_to_tensor(k, dtype), bits_to_tensor(v, dtype)
    td, sd, idd, nd = _i32(torch, table), _i32(torch, seq), _i32(torch, ids), _i32(torch, n_out)
    counters = _i64(torch, np.zeros(clients, dtype=np.int64))
    out = torch.empty_like(qd)
    ws = torch.empty(vtc.vtc_attn_workspace_bytes(p, len(seq), 0), dtype=torch.uint8, device="cuda")

    def step():
        vtc.vtc_step_decode(p, qd, kd, vd, td, sd, counters, idd, None, nd, 1, 2, out=out, workspace=ws)

    step()                                   # eager once: first-call set-up happens outside the capture
    torch.cuda.synchronize()
    eager = out.clone()
    want = OA.paged_decode(q, k, v, table, seq, SCALE, dtype)
    assert within_tolerance(OA.widen(tensor_to_bits(eager), dtype), want, dtype)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    charges = 1                              # the eager call; capture itself executes nothing
    for replay in range(3):
        out.fill_(float("nan"))              # eager work between the replays
        kd_sum = float(kd.float().sum().item())
        assert np.isfinite(kd_sum)
        graph.replay()
        torch.cuda.synchronize()
        charges += 1
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {replay} differs from eager"
        want_c = [0] * clients
        for _ in range(charges):
            want_c = counter_update(want_c, ids.tolist(), None, n_out.tolist(), 1, 2)
        assert counters.cpu().tolist() == want_c


def test_whole_mixed_step_replays_from_a_hip_graph(torch):
    # One serving iteration -- append this step's K/V rows, prefill the new prompts' chunk, decode the running
    # requests and charge the counters -- captured once and replayed on fresh inputs written into the same
    # buffers: every call of the path is capturable and every replay redoes all of it.
    say("append + prefill chunk + decode step captured into one graph")
    rng = np.random.default_rng(951)
    hq, hkv, dtype, clients = 8, 2, "bf16", 3
    n_dec = 3
    seq_after = np.array([40, 257, 16, 200, 90], dtype=np.int32)     # three decoding requests, two prompts
    n_new = np.array([1, 1, 1, 72, 90], dtype=np.int32)              # a later chunk and a whole prompt
    table, nb = make_block_table(rng, seq_after, 16)
    cu_new = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    cu_pf = (cu_new[n_dec:] - cu_new[n_dec]).astype(np.int32)
    p = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE)
    ids = np.array([0, 2, 1, 1, 0], dtype=np.int32)
    n_in = np.array([0, 0, 0, 72, 90], dtype=np.int32)
    n_out = np.array([1, 1, 1, 0, 0], dtype=np.int32)

    def fresh_inputs():
        _, k_full, v_full = make_qkv_numpy(rng, 1, hq, hkv, 128, nb, 16, dtype)
        q_dec = make_qkv_numpy(rng, n_dec, hq, hkv, 128, 1, 16, dtype)[0]
        q_pf = make_qkv_numpy(rng, int(cu_pf[-1]), hq, hkv, 128, 1, 16, dtype)[0]
        k_hole, v_hole = k_full.copy(), v_full.copy()
        new_k, new_v = [], []
        for r, (s, n) in enumerate(zip(seq_after, n_new)):
            for pos in range(s - n, s):
                blk, row = table[r, pos // 16], pos % 16
                new_k.append(k_full[blk, :, row, :].copy())
                new_v.append(v_full[blk, :, row, :].copy())
                k_hole[blk, :, row, :] = 0x7FC0                      # NaN where this step's rows go
                v_hole[blk, :, row, :] = 0x7FC0
        return q_dec, q_pf, k_full, v_full, k_hole, v_hole, np.stack(new_k), np.stack(new_v)

    first = fresh_inputs()
    qd, qp = bits_to_tensor(first[0], dtype), bits_to_tensor(first[1], dtype)
    kc, vc = bits_to_tensor(first[4], dtype), bits_to_tensor(first[5], dtype)
    nk, nv = bits_to_tensor(first[6], dtype), bits_to_tensor(first[7], dtype)
    t_all, s_all, cu_d = _i32(torch, table), _i32(torch, seq_after), _i32(torch, cu_new)
    t_dec, s_dec = _i32(torch, table[:n_dec]), _i32(torch, seq_after[:n_dec])
    t_pf, s_pf, cu_pf_d = _i32(torch, table[n_dec:]), _i32(torch, seq_after[n_dec:]), _i32(torch, cu_pf)
    idd, nind, noutd = _i32(torch, ids), _i32(torch, n_in), _i32(torch, n_out)
    counters = _i64(torch, np.zeros(clients, dtype=np.int64))
    out_d, out_p = torch.empty_like(qd), torch.empty_like(qp)
    ws = torch.empty(vtc.vtc_attn_workspace_bytes(p, n_dec, 0), dtype=torch.uint8, device="cuda")

    def step():
        vtc.vtc_kv_append(p, nk, nv, cu_d, int(n_new.max()), kc, vc, t_all, s_all)
        vtc.vtc_attn_prefill_chunk(p, qp, cu_pf_d, int(n_new[n_dec:].max()), kc, vc, t_pf, s_pf, out=out_p)
        vtc.vtc_step_decode(p, qd, kc, vc, t_dec, s_dec, counters, idd, nind, noutd, 1, 2, out=out_d, workspace=ws)

    def check(inputs, charges):
        q_dec, q_pf, k_full, v_full = inputs[:4]
        assert np.array_equal(tensor_to_bits(kc), k_full) and np.array_equal(tensor_to_bits(vc), v_full)
        want_d = OA.paged_decode(q_dec, k_full, v_full, table[:n_dec], seq_after[:n_dec], SCALE, dtype)
        want_p = OA.paged_prefill_chunk(q_pf, cu_pf, k_full, v_full, table[n_dec:], seq_after[n_dec:], SCALE, dtype)
        assert within_tolerance(OA.widen(tensor_to_bits(out_d), dtype), want_d, dtype)
        assert within_tolerance(OA.widen(tensor_to_bits(out_p), dtype), want_p, dtype)
        want_c = [0] * clients
        for _ in range(charges):
            want_c = counter_update(want_c, ids.tolist(), n_in.tolist(), n_out.tolist(), 1, 2)
        assert counters.cpu().tolist() == want_c

    step()                                   # eager once: first-call set-up happens outside the capture
    torch.cuda.synchronize()
    check(first, 1)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for replay in range(3):
        inputs = fresh_inputs()              # new q, new cache contents, new rows to append: same buffers
        qd.copy_(bits_to_tensor(inputs[0], dtype))
        qp.copy_(bits_to_tensor(inputs[1], dtype))
        kc.copy_(bits_to_tensor(inputs[4], dtype))
        vc.copy_(bits_to_tensor(inputs[5], dtype))
        nk.copy_(bits_to_tensor(inputs[6], dtype))
        nv.copy_(bits_to_tensor(inputs[7], dtype))
        out_d.fill_(float("nan"))
        out_p.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        check(inputs, replay + 2)
