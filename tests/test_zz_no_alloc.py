"""vtc_attn_decode_static (the entry point that allocates nothing and takes no workspace) against
vtc_attn_decode and the CPU oracle, through the C ABI (needs an MI355X).  Two calls in a row share the
library's built-in scratch array, the second on a smaller batch."""
import math
import sys

import numpy as np
import pytest

import paper_2401_00588_amd as vtc
from oracle import attention as OA
from tests.helpers import check_storage_output
from workloads import bits_to_tensor, make_block_table, make_qkv_numpy, tensor_to_bits

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


def _one_call(torch, seq, hq, hkv, dtype, seed, out_dtype=None):
    rng = np.random.default_rng(seed)
    table, nb = make_block_table(rng, seq, 16)
    q, k, v = make_qkv_numpy(rng, len(seq), hq, hkv, 128, nb, 16, dtype)
    p = vtc.make_params(hq, hkv, 128, 16, table.shape[1], dtype, SCALE, out_dtype)
    args = (bits_to_tensor(q, dtype), bits_to_tensor(k, dtype), bits_to_tensor(v, dtype), _i32(torch, table),
            _i32(torch, seq))
    t_out = torch.float32 if out_dtype == "f32" else args[0].dtype
    out = torch.full((len(seq), hq, 128), float("nan"), dtype=t_out, device="cuda")
    vtc.vtc_attn_decode_static(p, *args, out)
    torch.cuda.synchronize()
    ref = vtc.vtc_attn_decode(p, *args)                 # the existing entry point, caller-side workspace
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32 if out_dtype == "f32" else torch.int16),
                       ref.view(torch.int32 if out_dtype == "f32" else torch.int16))
    want = OA.paged_decode(q, k, v, table, seq, SCALE, dtype)
    if out_dtype is None:
        check_storage_output(OA.widen(tensor_to_bits(out), dtype), want, dtype, f"static decode, {len(seq)} sequences")
    else:
        assert np.abs(out.double().cpu().numpy() - want).max() <= {"f16": 2e-3, "bf16": 1e-2}[dtype]
    return out


@pytest.mark.parametrize("dtype,hq,hkv", [("bf16", 32, 8), ("f16", 8, 8), ("bf16", 16, 2)])
def test_two_calls_in_a_row_the_second_smaller(torch, dtype, hq, hkv):
    say(f"static decode dtype={dtype} Hq={hq} Hkv={hkv}: a large call, then a smaller one")
    rng = np.random.default_rng(4242)
    big = [int(x) for x in rng.integers(0, 900, size=300)] + [5000, 1, 0, 17]      # thousands of ranges, many cut
    _one_call(torch, big, hq, hkv, dtype, seed=1)
    small = [1, 40, 0, 513, 16]                                                     # fewer waves than before: stale
    _one_call(torch, small, hq, hkv, dtype, seed=2)                                 # partials must not be picked up
    _one_call(torch, [3], hq, hkv, dtype, seed=3, out_dtype="f32")


def test_more_sequences_than_the_scratch_array_is_laid_out_for(torch):
    say("static decode: size limit")
    p = vtc.make_params(8, 2, 128, 16, 4, "bf16", SCALE)
    n = 65537
    z = torch.zeros((n, 8, 128), dtype=torch.bfloat16, device="cuda")
    cache = torch.zeros((1, 2, 16, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(vtc.VtcError) as err:
        vtc.vtc_attn_decode_static(p, z, cache, cache, torch.zeros((n, 4), dtype=torch.int32, device="cuda"),
                                   torch.zeros(n, dtype=torch.int32, device="cuda"), torch.empty_like(z))
    assert err.value.code == -5
