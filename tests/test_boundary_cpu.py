"""The C ABI without a GPU: the library loads, exports what include/vtc.h declares,
and rejects bad host-visible arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2401_00588_amd as vtc
from paper_2401_00588_amd.binding import AttnParams

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(vtc.library_path()):
        from paper_2401_00588_amd import build
        build.build()
    return vtc.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "vtc.h"), encoding="utf-8").read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vtc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert {"vtc_attn_decode", "vtc_attn_decode_profiled", "vtc_attn_prefill_chunk", "vtc_counter_update",
            "vtc_counter_update_cost", "vtc_counter_update_predicted", "vtc_kv_append", "vtc_attn_workspace_bytes",
            "vtc_debug_gather_slots", "vtc_strerror", "vtc_version", "vtc_step_decode",
            "vtc_step_decode_profiled"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None


def test_version_and_strerror(lib):
    assert vtc.vtc_version() >= 200
    for code in (0, -1, -2, -3, -4, -99):
        assert isinstance(vtc.vtc_strerror(code), str) and vtc.vtc_strerror(code)
    assert vtc.vtc_strerror(0) == "success"


def good_params(**kw):
    base = dict(num_q_heads=32, num_kv_heads=8, head_dim=128, block_size=16, max_blocks_per_seq=256,
                dtype=vtc.VTC_BF16, scale=0.0883883461356163, out_dtype=vtc.VTC_BF16)
    base.update(kw)
    if "dtype" in kw and "out_dtype" not in kw:
        base["out_dtype"] = kw["dtype"]
    return AttnParams(**base)


def test_workspace_bytes_is_host_arithmetic(lib):
    p = good_params()
    small = vtc.vtc_attn_workspace_bytes(p, 8, 256)
    big = vtc.vtc_attn_workspace_bytes(p, 512, 4096)
    assert 0 < small < big
    # short batches cannot use many waves; from some size on the device's wave count caps the footprint
    assert vtc.vtc_attn_workspace_bytes(p, 512, 0) == big == vtc.vtc_attn_workspace_bytes(p, 512, 10 ** 9)
    assert vtc.vtc_attn_workspace_bytes(p, 4096, 0) - big <= 8 * 4096 + 256          # only the per-sequence prefix grows
    assert big % 256 == 0 and small % 256 == 0
    # room for two fp32 partials (128 floats + m, l) per q head of the group for every wave of the largest launch
    # (no device here: 256 compute units are assumed, 4 waves on each for grouped queries)
    assert big >= 2 * 1024 * 4 * (128 + 2) * 4
    assert big < 8 << 20
    # 8 sequences x 8 kv heads x (16 blocks + 1 unit for beginning a head) = 1088 cost units: 544 waves of two each
    assert 2 * 544 * 4 * (128 + 2) * 4 <= small < 2 * 544 * 4 * (128 + 2) * 4 + 16 * 544 + 4096
    mha = vtc.vtc_attn_workspace_bytes(good_params(num_q_heads=32, num_kv_heads=32), 512, 4096)
    assert mha < big                                   # twice the waves, but a quarter of the q heads per KV head
    assert vtc.vtc_attn_workspace_bytes(good_params(head_dim=64), 8, 256) == 0
    assert lib.vtc_attn_workspace_bytes(None, 8, 256) == 0
    assert vtc.vtc_attn_workspace_bytes(good_params(out_dtype=vtc.VTC_F32), 512, 4096) == big


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=64), -2), (dict(block_size=32), -2), (dict(block_size=3), -2), (dict(block_size=0), -2), (dict(dtype=7), -2),
    (dict(num_q_heads=32, num_kv_heads=5), -2), (dict(num_q_heads=48, num_kv_heads=16), -2),
    (dict(num_q_heads=0), -1), (dict(num_kv_heads=-1), -1), (dict(max_blocks_per_seq=0), -1),
    (dict(scale=float("nan")), -1),
    (dict(out_dtype=vtc.VTC_F16), -2), (dict(out_dtype=5), -2), (dict(dtype=vtc.VTC_F32, out_dtype=vtc.VTC_F32), -2),
])
def test_bad_params_are_rejected_by_every_attention_entry_point(lib, kw, code):
    p = good_params(**kw)
    one = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    assert lib.vtc_attn_decode(ctypes.byref(p), 1, one, one, one, one, one, one, one, 1 << 30, None) == code
    assert lib.vtc_attn_prefill_chunk(ctypes.byref(p), 1, one, one, 1, one, one, one, one, one, None, 0, None) == code
    assert lib.vtc_debug_gather_slots(ctypes.byref(p), 1, one, one, one, 1, one, None) == code
    assert lib.vtc_step_decode(ctypes.byref(p), 1, one, one, one, one, one, one, one, 2, one, one, one, 1, 1, 2, one,
                               1 << 30, None) == code


def test_null_pointers_sizes_alignment_and_workspace(lib):
    p = good_params()
    a = ctypes.c_void_p(4096)
    need = vtc.vtc_attn_workspace_bytes(p, 4, 0)
    assert lib.vtc_attn_decode(None, 4, a, a, a, a, a, a, a, need, None) == -1
    assert lib.vtc_attn_decode(ctypes.byref(p), -1, a, a, a, a, a, a, a, need, None) == -1
    assert lib.vtc_attn_decode(ctypes.byref(p), 0, None, None, None, None, None, None, None, 0, None) == 0
    for hole in range(7):
        args = [a] * 7
        args[hole] = None
        assert lib.vtc_attn_decode(ctypes.byref(p), 4, *args, need, None) == -1
    one_wave = vtc.vtc_attn_workspace_bytes(p, 4, 1)
    assert 0 < one_wave <= need
    assert lib.vtc_attn_decode(ctypes.byref(p), 4, a, a, a, a, a, a, a, 1024, None) == -3      # not even one wave's share
    assert lib.vtc_attn_decode(ctypes.byref(p), 4, a, a, a, a, a, a, a, 0, None) == -3
    assert lib.vtc_attn_decode(ctypes.byref(p), 4, a, a, a, a, a, a, ctypes.c_void_p(4096 + 64), need, None) == -1
    assert lib.vtc_attn_decode(ctypes.byref(p), 4, ctypes.c_void_p(4098), a, a, a, a, a, a, need, None) == -1

    assert lib.vtc_attn_prefill_chunk(ctypes.byref(p), 0, None, None, 0, None, None, None, None, None, None, 0, None) == 0
    assert lib.vtc_attn_prefill_chunk(ctypes.byref(p), 2, a, a, 0, a, a, a, a, a, None, 0, None) == 0
    assert lib.vtc_attn_prefill_chunk(ctypes.byref(p), 2, a, a, -1, a, a, a, a, a, None, 0, None) == -1
    for hole in (0, 1, 3, 4, 5, 6, 7):
        args = [a, a, 16, a, a, a, a, a]
        args[hole] = None
        assert lib.vtc_attn_prefill_chunk(ctypes.byref(p), 2, *args, None, 0, None) == -1

    assert lib.vtc_counter_update(None, 4, a, a, a, 8, 1, 2, None) == -1
    assert lib.vtc_counter_update(a, 4, None, a, a, 8, 1, 2, None) == -1
    assert lib.vtc_counter_update(a, -1, a, a, a, 8, 1, 2, None) == -1
    assert lib.vtc_counter_update(a, 4, a, a, a, -8, 1, 2, None) == -1
    assert lib.vtc_counter_update(None, 4, None, None, None, 0, 1, 2, None) == 0

    h = vtc.CostPoly(0, 1, 2, 0, 0, 0)
    assert lib.vtc_counter_update_cost(a, 4, a, a, a, a, a, 8, None, None, None) == -1
    assert lib.vtc_counter_update_cost(a, 4, a, a, a, None, a, 8, ctypes.byref(h), None, None) == -1
    assert lib.vtc_counter_update_cost(None, 4, a, a, a, a, a, 8, ctypes.byref(h), None, None) == -1
    assert lib.vtc_counter_update_cost(a, 4, a, a, a, a, a, -1, ctypes.byref(h), None, None) == -1
    assert lib.vtc_counter_update_cost(None, 4, None, None, None, None, None, 0, ctypes.byref(h), None, None) == 0
    assert lib.vtc_counter_update_predicted(a, 4, a, a, None, a, 8, 2, None) == -1
    assert lib.vtc_counter_update_predicted(a, -4, a, a, a, a, 8, 2, None) == -1
    assert lib.vtc_counter_update_predicted(None, 4, None, None, None, None, 0, 2, None) == 0
    assert lib.vtc_kv_append(ctypes.byref(p), 2, a, a, a, 1, a, a, a, None, None) == -1
    assert lib.vtc_kv_append(ctypes.byref(p), 2, a, ctypes.c_void_p(4104), a, 1, a, a, a, a, None) == -1
    assert lib.vtc_kv_append(ctypes.byref(p), 2, a, a, a, -1, a, a, a, a, None) == -1
    assert lib.vtc_kv_append(ctypes.byref(p), 0, None, None, None, 0, None, None, None, None, None) == 0
    assert lib.vtc_kv_append(ctypes.byref(good_params(head_dim=64)), 2, a, a, a, 1, a, a, a, a, None) == -2

    assert lib.vtc_debug_gather_slots(ctypes.byref(p), 2, a, a, a, -1, a, None) == -1
    assert lib.vtc_debug_gather_slots(ctypes.byref(p), 2, None, a, a, 5, a, None) == -1
    assert lib.vtc_debug_gather_slots(ctypes.byref(p), 0, None, None, None, 0, None, None) == 0


def test_wrappers_refuse_cpu_tensors(lib):
    import torch

    p = good_params()
    q = torch.zeros(1, 32, 128, dtype=torch.bfloat16)
    kc = torch.zeros(2, 8, 16, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        vtc.vtc_attn_decode(p, q, kc, kc, torch.zeros(1, 256, dtype=torch.int32), torch.ones(1, dtype=torch.int32))
    with pytest.raises(ValueError):
        vtc.vtc_counter_update(torch.zeros(2, dtype=torch.int64), torch.zeros(3, dtype=torch.int32), None, None, 1, 2)


def test_missing_library_is_a_loud_error(monkeypatch):
    from paper_2401_00588_amd import binding

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_NAME", "libvtc_not_built.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library()


def test_fused_step_validates_both_halves_before_enqueueing(lib):
    p = good_params()
    a = ctypes.c_void_p(4096)
    need = vtc.vtc_attn_workspace_bytes(p, 4, 0)

    def call(num_seqs=4, attn=None, counters=a, num_clients=3, ids=a, n_in=a, n_out=a, n=4, ws=a, ws_bytes=need):
        attn = [a] * 6 if attn is None else attn
        return lib.vtc_step_decode(ctypes.byref(p), num_seqs, *attn, counters, num_clients, ids, n_in, n_out, n, 1, 2,
                                   ws, ws_bytes, None)

    assert call(num_seqs=-1) == -1
    assert call(n=-1) == -1
    assert call(num_clients=-1) == -1
    assert call(counters=None) == -1                       # a charge was asked for: its arrays must be there
    assert call(ids=None) == -1
    for hole in range(6):                                  # the attention half's pointers
        attn = [a] * 6
        attn[hole] = None
        assert call(attn=attn) == -1
    assert call(ws=None) == -1
    assert call(ws_bytes=512) == -3
    assert call(ws=ctypes.c_void_p(4096 + 64)) == -1
    # nothing to do at all is a successful no-op, whatever the pointers are
    assert lib.vtc_step_decode(ctypes.byref(p), 0, None, None, None, None, None, None, None, 3, None, None, None, 0,
                               1, 2, None, 0, None) == 0
    assert lib.vtc_step_decode(ctypes.byref(p), 0, None, None, None, None, None, None, None, 0, a, a, a, 5,
                               1, 2, None, 0, None) == 0   # no clients: every id is out of range


def test_static_decode_validates_on_the_host(lib):
    # the entry point without a workspace argument: same host-side checks, plus its own size limit, all before
    # any HIP call
    p = good_params()
    a = ctypes.c_void_p(4096)
    call = lambda n, args: lib.vtc_attn_decode_static(ctypes.byref(p), n, *args, None)
    assert call(0, [None] * 6) == 0
    assert call(-1, [a] * 6) == -1
    assert call(65537, [a] * 6) == -5
    assert vtc.vtc_strerror(-5) and "65536" in vtc.vtc_strerror(-5)
    for hole in range(6):
        args = [a] * 6
        args[hole] = None
        assert call(4, args) == -1
    assert call(4, [ctypes.c_void_p(4098)] + [a] * 5) == -1
    bad = good_params(head_dim=64)
    assert lib.vtc_attn_decode_static(ctypes.byref(bad), 4, a, a, a, a, a, a, None) == -2
