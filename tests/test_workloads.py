"""The seeded input generators and the stored batch snapshots (CPU only)."""
import os

import numpy as np
import pytest

from oracle import make_batch_snapshots
from oracle.counters import counter_update
from workloads import batches, make_block_table, make_step_batch, trace_for_config
from workloads.tensors import f32_to_storage_bits


def test_storage_rounding_is_round_to_nearest_even():
    import torch

    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10,
                        np.float32([1.00390625, 1.01171875, -1.00390625, 0.0, 65504.0])])
    for dtype, tdt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        ours = f32_to_storage_bits(x, dtype)
        ref = torch.from_numpy(x).to(tdt).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(ours, ref)


def test_block_table_is_a_partial_permutation():
    rng = np.random.default_rng(1)
    seq = [1, 16, 17, 0, 300]
    table, nb = make_block_table(rng, seq, 16, spare_blocks=5)
    need = [(s + 15) // 16 for s in seq]
    used = np.concatenate([table[r, :n] for r, n in enumerate(need)])
    assert len(set(used.tolist())) == len(used) == sum(need)
    assert used.min() >= 0 and used.max() < nb and nb == sum(need) + 5
    assert table.shape[1] == max(need)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_step_batches_have_the_stated_shapes(cfg):
    b = make_step_batch(cfg)
    n = {1: 8, 2: 64, 3: 256, 4: 512, 5: 256}[cfg]
    assert b.num_decode == n and b.client_ids.shape == (n,)
    assert b.num_clients == {1: 2, 2: 2, 3: 4, 4: 27, 5: 8}[cfg]
    assert b.client_ids.min() >= 0 and b.client_ids.max() < b.num_clients
    assert (b.w_p, b.w_q) == (1, 2)
    assert b.shape.dtype == ("f16" if cfg <= 3 else "bf16")
    assert b.shape.num_kv_heads == (32 if cfg <= 3 else 8)
    lo, hi = {1: (16, 256), 2: (256, 640), 3: (65, 2048 + 512), 4: (3, 8192), 5: (128, 4096)}[cfg]
    assert b.seq_lens.min() >= lo and b.seq_lens.max() <= hi
    assert b.decode_kv_bytes == int(b.seq_lens.sum()) * b.shape.kv_bytes_per_token
    if cfg == 5:
        assert b.num_prefill == 16 and b.prefill_causal_pairs == 16 * (256 * 257 // 2)
        b1 = make_step_batch(5, prefill_chunk=1)
        assert b1.prefill_causal_pairs == 16 * (256 * 256 + 256 * 257 // 2)
        assert np.array_equal(b1.seq_lens, b.seq_lens)
        ids, n_in, n_out = b.counter_update_args(first_chunk=True)
        assert len(ids) == 272 and n_in.sum() == 16 * 512 and n_out.sum() == 256
        assert b1.counter_update_args(first_chunk=False)[1].sum() == 0


@pytest.mark.parametrize("cfg", [3, 4])
def test_snapshots_are_what_the_scheduler_script_writes(cfg, tmp_path, monkeypatch):
    stored = open(os.path.join(batches.DATA_DIR, f"cfg{cfg}_batch.txt"), encoding="ascii").read()
    monkeypatch.setattr(make_batch_snapshots, "DATA_DIR", str(tmp_path))
    path = make_batch_snapshots.write(cfg)
    assert open(path, encoding="ascii").read() == stored


@pytest.mark.parametrize("cfg", [3, 4])
def test_snapshot_is_self_consistent(cfg):
    b = make_step_batch(cfg)
    trace, p = trace_for_config(cfg)
    by_rid = {r.rid: r for r in trace}
    path = os.path.join(batches.DATA_DIR, f"cfg{cfg}_batch.txt")
    rows = [list(map(int, ln.split())) for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == p["max_batch"] == b.num_decode
    for rid, cl, n_in, gen, s in rows:
        r = by_rid[rid]
        assert (r.client, r.n_input) == (cl, n_in)
        assert 0 <= gen < r.n_output and s == n_in + gen + 1
    # the recorded counters differ by exactly the decode charge of Algorithm 2
    ids, n_in, n_out = b.counter_update_args()
    assert counter_update(b.counters_before, ids, n_in, n_out, b.w_p, b.w_q) == b.counters_after.tolist()
    # VTC keeps the overloaded clients' counters close together
    assert b.counters_before.max() - b.counters_before.min() < 2 * p["w_q"] * p["M"]


def test_elementwise_tolerance_is_flat_where_the_output_format_allows_it():
    from tests.helpers import TOL, elementwise_tolerance, within_tolerance

    want = np.array([0.0, 1e-9, 0.5, 1.99, 2.0, 3.999, 4.0, 7.9, 8.0])
    bf = elementwise_tolerance(want, "bf16")
    assert (bf[:6] == TOL["bf16"]).all()                       # below 4 the flat 1e-2 holds
    assert bf[6] == bf[7] == 2.0 ** -6 + 2e-3                  # [4, 8): half the spacing 2^-5, plus a fifth of the flat bar
    assert bf[8] == 2.0 ** -5 + 2e-3
    f = elementwise_tolerance(want, "f16")
    assert (f[:6] == TOL["f16"]).all() and f[6] == 2.0 ** -9 + 4e-4
    # a correctly rounded bf16 result always passes; one more unit in the last place does not
    exact = np.array([4.0 + 2.0 ** -6 - 1e-6, 3.0 + 2.0 ** -7 - 1e-6])
    rounded = np.array([4.0, 3.0])
    assert within_tolerance(rounded, exact, "bf16")
    assert not within_tolerance(rounded - np.array([2.0 ** -5, 2.0 ** -6]), exact, "bf16")
    assert not within_tolerance(np.array([np.nan]), np.array([0.0]), "bf16")
    # the report of how the bound was used: elements the format limits, and elements that needed that allowance
    from tests.helpers import check_f32_output, check_storage_output, parity_stats
    st = parity_stats(np.array([4.0, 3.0, 1.0]), np.array([4.0 + 2.0 ** -6 - 1e-6, 3.0 + 2.0 ** -7 - 1e-6, 1.0]), "bf16")
    assert st == {"max_abs": pytest.approx(2.0 ** -6 - 1e-6), "elements": 3, "format_limited": 1, "over_flat": 1, "ok": True}
    check_storage_output(np.array([4.0, 1.0]), np.array([4.0 + 2.0 ** -6 - 1e-6, 1.0]), "bf16", "demo")
    with pytest.raises(AssertionError):            # ... which a benchmark configuration must not need
        check_storage_output(np.array([4.0, 1.0]), np.array([4.0 + 2.0 ** -6 - 1e-6, 1.0]), "bf16", "demo", flat_only=True)
    with pytest.raises(AssertionError):            # fp32 rows get the flat bar whatever their magnitude
        check_f32_output(np.array([4.0]), np.array([4.0 + 2.0 ** -6 - 1e-6]), "bf16", "demo")
    check_f32_output(np.array([4.0]), np.array([4.0 + 9e-3]), "bf16", "demo")
