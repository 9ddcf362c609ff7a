"""ctypes binding of libvtc_mi355x.so (see include/vtc.h for the contract).

The wrappers take torch tensors that already live on the GPU, check dtype,
shape, contiguity and device, and pass raw device pointers plus the current
HIP stream to the library.  PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

VTC_F16 = 0
VTC_BF16 = 1
VTC_F32 = 2          # output rows only

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libvtc_mi355x.so"
_lib: Optional[ctypes.CDLL] = None


class VtcError(RuntimeError):
    def __init__(self, code: int, where: str) -> None:
        self.code = code
        super().__init__(f"{where} failed with code {code}: {vtc_strerror(code)}")


class AttnParams(ctypes.Structure):
    """Mirror of ``vtc_attn_params``."""

    _fields_ = [
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("max_blocks_per_seq", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("out_dtype", ctypes.c_int32),
    ]


class CostPoly(ctypes.Structure):
    """Mirror of ``vtc_cost_poly``: h = c0 + cp*n_p + cq*n_q + cpp*n_p^2 + cpq*n_p*n_q + cqq*n_q^2."""

    _fields_ = [(name, ctypes.c_int64) for name in ("c0", "cp", "cq", "cpp", "cpq", "cqq")]


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library() -> ctypes.CDLL:
    """Load the built HIP library; fail loudly if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build the HIP extension first (python -m paper_2401_00588_amd.build). "
            "There is no CPU fallback."
        )
    lib = ctypes.CDLL(path)
    P = ctypes.POINTER(AttnParams)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.vtc_version.restype = ctypes.c_int
    lib.vtc_version.argtypes = []
    lib.vtc_strerror.restype = ctypes.c_char_p
    lib.vtc_strerror.argtypes = [ctypes.c_int]
    lib.vtc_attn_workspace_bytes.restype = sz
    lib.vtc_attn_workspace_bytes.argtypes = [P, i32, i32]
    lib.vtc_attn_decode.restype = ctypes.c_int
    lib.vtc_attn_decode.argtypes = [P, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.vtc_attn_decode_static.restype = ctypes.c_int
    lib.vtc_attn_decode_static.argtypes = [P, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.vtc_attn_decode_profiled.restype = ctypes.c_int
    lib.vtc_attn_decode_profiled.argtypes = [P, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp]
    lib.vtc_step_decode.restype = ctypes.c_int
    lib.vtc_step_decode.argtypes = [P, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, i32, i64, i64, vp, sz, vp]
    lib.vtc_step_decode_profiled.restype = ctypes.c_int
    lib.vtc_step_decode_profiled.argtypes = [P, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, i32, i64, i64, vp,
                                             sz, vp, vp, vp]
    lib.vtc_attn_prefill_chunk.restype = ctypes.c_int
    lib.vtc_attn_prefill_chunk.argtypes = [P, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.vtc_counter_update.restype = ctypes.c_int
    lib.vtc_counter_update.argtypes = [vp, i32, vp, vp, vp, i32, i64, i64, vp]
    lib.vtc_counter_update_cost.restype = ctypes.c_int
    lib.vtc_counter_update_cost.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, ctypes.POINTER(CostPoly), vp, vp]
    lib.vtc_counter_update_predicted.restype = ctypes.c_int
    lib.vtc_counter_update_predicted.argtypes = [vp, i32, vp, vp, vp, vp, i32, i64, vp]
    lib.vtc_kv_append.restype = ctypes.c_int
    lib.vtc_kv_append.argtypes = [P, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.vtc_debug_gather_slots.restype = ctypes.c_int
    lib.vtc_debug_gather_slots.argtypes = [P, i32, vp, vp, vp, i32, vp, vp]
    _lib = lib
    return lib


def vtc_version() -> int:
    return int(load_library().vtc_version())


def vtc_strerror(code: int) -> str:
    return load_library().vtc_strerror(int(code)).decode("ascii")


def _dtype_code(dtype) -> int:
    if isinstance(dtype, str):
        return {"f16": VTC_F16, "bf16": VTC_BF16, "f32": VTC_F32}[dtype]
    if isinstance(dtype, int):
        return dtype
    import torch

    return {torch.float16: VTC_F16, torch.bfloat16: VTC_BF16, torch.float32: VTC_F32}[dtype]


def make_params(num_q_heads: int, num_kv_heads: int, head_dim: int, block_size: int,
                max_blocks_per_seq: int, dtype, scale: float, out_dtype=None) -> AttnParams:
    """``dtype`` is VTC_F16 / VTC_BF16, "f16" / "bf16", or a torch dtype; ``out_dtype`` (default: the same)
    may also be VTC_F32 / "f32" / torch.float32 for unrounded fp32 output rows."""
    code = _dtype_code(dtype)
    out_code = code if out_dtype is None else _dtype_code(out_dtype)
    return AttnParams(num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, code, scale, out_code)


def vtc_attn_workspace_bytes(params: AttnParams, max_num_seqs: int, max_seq_len: int = 0) -> int:
    return int(load_library().vtc_attn_workspace_bytes(ctypes.byref(params), max_num_seqs, max_seq_len))


# ------------------------------------------------------------------ marshalling
def _torch():
    import torch

    return torch


def _elt_dtype(params: AttnParams):
    torch = _torch()
    return torch.float16 if params.dtype == VTC_F16 else torch.bfloat16


def _out_dtype(params: AttnParams):
    return _torch().float32 if params.out_dtype == VTC_F32 else _elt_dtype(params)


def _check(t, name: str, dtype, ndim: Optional[int] = None) -> None:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if ndim is not None and t.dim() != ndim:
        raise ValueError(f"{name} must have {ndim} dimensions")


def _stream() -> int:
    return int(_torch().cuda.current_stream().cuda_stream)


class HipEvent:
    """A timing-enabled hipEvent_t owned by Python (created through the HIP runtime, not torch)."""

    _hip = None

    @classmethod
    def _rt(cls):
        if cls._hip is None:
            hip = ctypes.CDLL("libamdhip64.so")
            hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
            hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
            hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
            hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
            cls._hip = hip
        return cls._hip

    def __init__(self) -> None:
        self.handle = ctypes.c_void_p()
        rc = self._rt().hipEventCreate(ctypes.byref(self.handle))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed with {rc}")

    def synchronize(self) -> None:
        rc = self._rt().hipEventSynchronize(self.handle)
        if rc != 0:
            raise RuntimeError(f"hipEventSynchronize failed with {rc}")

    def elapsed_ms(self, end: "HipEvent") -> float:
        ms = ctypes.c_float()
        rc = self._rt().hipEventElapsedTime(ctypes.byref(ms), self.handle, end.handle)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed with {rc}")
        return float(ms.value)

    def __del__(self) -> None:
        try:
            if self.handle:
                self._rt().hipEventDestroy(self.handle)
        except Exception:
            pass


def vtc_attn_decode(params: AttnParams, q, k_cache, v_cache, block_table, seq_lens, out=None, workspace=None,
                    ev_begin: Optional[HipEvent] = None, ev_end: Optional[HipEvent] = None):
    """out[N, Hq, D] = decode attention; allocates ``out`` / ``workspace`` with torch when not given.

    With ``ev_begin`` / ``ev_end`` the call goes through ``vtc_attn_decode_profiled`` and the events
    bracket the attention kernel on the current stream.
    """
    torch = _torch()
    lib = load_library()
    elt = _elt_dtype(params)
    _check(q, "q", elt, 3)
    _check(k_cache, "k_cache", elt, 4)
    _check(v_cache, "v_cache", elt, 4)
    _check(block_table, "block_table", torch.int32, 2)
    _check(seq_lens, "seq_lens", torch.int32, 1)
    n = int(seq_lens.shape[0])
    if tuple(q.shape) != (n, params.num_q_heads, params.head_dim):
        raise ValueError("q must be [num_seqs, num_q_heads, head_dim]")
    if tuple(k_cache.shape[1:]) != (params.num_kv_heads, params.block_size, params.head_dim) or k_cache.shape != v_cache.shape:
        raise ValueError("k_cache / v_cache must be [num_blocks, num_kv_heads, block_size, head_dim]")
    if tuple(block_table.shape) != (n, params.max_blocks_per_seq):
        raise ValueError("block_table must be [num_seqs, max_blocks_per_seq]")
    if out is None:
        out = torch.empty_like(q, dtype=_out_dtype(params))
    _check(out, "out", _out_dtype(params), 3)
    if out.shape != q.shape:
        raise ValueError("out must have the shape of q")
    need = vtc_attn_workspace_bytes(params, n, 0)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(workspace, "workspace", torch.uint8, 1)
    if ev_begin is None and ev_end is None:
        rc = lib.vtc_attn_decode(ctypes.byref(params), n, q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(),
                                 block_table.data_ptr(), seq_lens.data_ptr(), out.data_ptr(),
                                 workspace.data_ptr(), workspace.numel(), _stream())
    else:
        rc = lib.vtc_attn_decode_profiled(ctypes.byref(params), n, q.data_ptr(), k_cache.data_ptr(),
                                          v_cache.data_ptr(), block_table.data_ptr(), seq_lens.data_ptr(),
                                          out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(),
                                          ev_begin.handle if ev_begin else None,
                                          ev_end.handle if ev_end else None)
    if rc != 0:
        raise VtcError(rc, "vtc_attn_decode")
    return out


def vtc_attn_decode_static(params: AttnParams, q, k_cache, v_cache, block_table, seq_lens, out):
    """``vtc_attn_decode`` on the library's built-in scratch array: no workspace argument, and nothing is
    allocated here either (``out`` must be given)."""
    torch = _torch()
    lib = load_library()
    elt = _elt_dtype(params)
    _check(q, "q", elt, 3)
    _check(k_cache, "k_cache", elt, 4)
    _check(v_cache, "v_cache", elt, 4)
    _check(block_table, "block_table", torch.int32, 2)
    _check(seq_lens, "seq_lens", torch.int32, 1)
    n = int(seq_lens.shape[0])
    if tuple(q.shape) != (n, params.num_q_heads, params.head_dim):
        raise ValueError("q must be [num_seqs, num_q_heads, head_dim]")
    if tuple(k_cache.shape[1:]) != (params.num_kv_heads, params.block_size, params.head_dim) or k_cache.shape != v_cache.shape:
        raise ValueError("k_cache / v_cache must be [num_blocks, num_kv_heads, block_size, head_dim]")
    if tuple(block_table.shape) != (n, params.max_blocks_per_seq):
        raise ValueError("block_table must be [num_seqs, max_blocks_per_seq]")
    _check(out, "out", _out_dtype(params), 3)
    if out.shape != q.shape:
        raise ValueError("out must have the shape of q")
    rc = lib.vtc_attn_decode_static(ctypes.byref(params), n, q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(),
                                    block_table.data_ptr(), seq_lens.data_ptr(), out.data_ptr(), _stream())
    if rc != 0:
        raise VtcError(rc, "vtc_attn_decode_static")
    return out


def vtc_step_decode(params: AttnParams, q, k_cache, v_cache, block_table, seq_lens, counters, client_ids,
                    n_input_tokens, n_output_tokens, w_p: int, w_q: int, out=None, workspace=None,
                    ev_begin: Optional[HipEvent] = None, ev_end: Optional[HipEvent] = None):
    """Decode attention plus the step's counter charge in one call (``counters`` is updated in place).

    The attention arguments are those of ``vtc_attn_decode``, the charge arguments those of
    ``vtc_counter_update``; ``client_ids`` may list more requests than ``seq_lens`` (a mixed step).
    """
    torch = _torch()
    lib = load_library()
    elt = _elt_dtype(params)
    _check(q, "q", elt, 3)
    _check(k_cache, "k_cache", elt, 4)
    _check(v_cache, "v_cache", elt, 4)
    _check(block_table, "block_table", torch.int32, 2)
    _check(seq_lens, "seq_lens", torch.int32, 1)
    n = int(seq_lens.shape[0])
    if tuple(q.shape) != (n, params.num_q_heads, params.head_dim):
        raise ValueError("q must be [num_seqs, num_q_heads, head_dim]")
    if tuple(k_cache.shape[1:]) != (params.num_kv_heads, params.block_size, params.head_dim) or k_cache.shape != v_cache.shape:
        raise ValueError("k_cache / v_cache must be [num_blocks, num_kv_heads, block_size, head_dim]")
    if tuple(block_table.shape) != (n, params.max_blocks_per_seq):
        raise ValueError("block_table must be [num_seqs, max_blocks_per_seq]")
    if out is None:
        out = torch.empty_like(q, dtype=_out_dtype(params))
    _check(out, "out", _out_dtype(params), 3)
    if out.shape != q.shape:
        raise ValueError("out must have the shape of q")
    _check(counters, "counters", torch.int64, 1)
    _check(client_ids, "client_ids", torch.int32, 1)
    n_req = int(client_ids.shape[0])
    for name, t in (("n_input_tokens", n_input_tokens), ("n_output_tokens", n_output_tokens)):
        if t is not None:
            _check(t, name, torch.int32, 1)
            if t.shape[0] != n_req:
                raise ValueError(f"{name} must have one entry per request")
    need = vtc_attn_workspace_bytes(params, n, 0)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(workspace, "workspace", torch.uint8, 1)
    args = [ctypes.byref(params), n, q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), block_table.data_ptr(),
            seq_lens.data_ptr(), out.data_ptr(), counters.data_ptr(), int(counters.shape[0]), client_ids.data_ptr(),
            None if n_input_tokens is None else n_input_tokens.data_ptr(),
            None if n_output_tokens is None else n_output_tokens.data_ptr(), n_req, int(w_p), int(w_q),
            workspace.data_ptr(), workspace.numel(), _stream()]
    if ev_begin is None and ev_end is None:
        rc = lib.vtc_step_decode(*args)
    else:
        rc = lib.vtc_step_decode_profiled(*args, ev_begin.handle if ev_begin else None,
                                          ev_end.handle if ev_end else None)
    if rc != 0:
        raise VtcError(rc, "vtc_step_decode")
    return out


def vtc_attn_prefill_chunk(params: AttnParams, q, cu_q_lens, max_q_len: int, k_cache, v_cache, block_table,
                           seq_lens, out=None):
    """out[T, Hq, D] = causal prefill-chunk attention over the paged cache."""
    torch = _torch()
    lib = load_library()
    elt = _elt_dtype(params)
    _check(q, "q", elt, 3)
    _check(cu_q_lens, "cu_q_lens", torch.int32, 1)
    _check(k_cache, "k_cache", elt, 4)
    _check(v_cache, "v_cache", elt, 4)
    _check(block_table, "block_table", torch.int32, 2)
    _check(seq_lens, "seq_lens", torch.int32, 1)
    n = int(seq_lens.shape[0])
    if cu_q_lens.shape[0] != n + 1:
        raise ValueError("cu_q_lens must be [num_seqs + 1]")
    if tuple(q.shape[1:]) != (params.num_q_heads, params.head_dim):
        raise ValueError("q must be [total_q_tokens, num_q_heads, head_dim]")
    if tuple(k_cache.shape[1:]) != (params.num_kv_heads, params.block_size, params.head_dim) or k_cache.shape != v_cache.shape:
        raise ValueError("k_cache / v_cache must be [num_blocks, num_kv_heads, block_size, head_dim]")
    if tuple(block_table.shape) != (n, params.max_blocks_per_seq):
        raise ValueError("block_table must be [num_seqs, max_blocks_per_seq]")
    if out is None:
        out = torch.empty_like(q, dtype=_out_dtype(params))
    _check(out, "out", _out_dtype(params), 3)
    if out.shape != q.shape:
        raise ValueError("out must have the shape of q")
    rc = lib.vtc_attn_prefill_chunk(ctypes.byref(params), n, q.data_ptr(), cu_q_lens.data_ptr(), int(max_q_len),
                                    k_cache.data_ptr(), v_cache.data_ptr(), block_table.data_ptr(),
                                    seq_lens.data_ptr(), out.data_ptr(), None, 0, _stream())
    if rc != 0:
        raise VtcError(rc, "vtc_attn_prefill_chunk")
    return out


def vtc_counter_update(counters, client_ids, n_input_tokens, n_output_tokens, w_p: int, w_q: int):
    """counters[client_ids[r]] += w_p * n_input_tokens[r] + w_q * n_output_tokens[r], in place."""
    torch = _torch()
    lib = load_library()
    _check(counters, "counters", torch.int64, 1)
    _check(client_ids, "client_ids", torch.int32, 1)
    n = int(client_ids.shape[0])
    for name, t in (("n_input_tokens", n_input_tokens), ("n_output_tokens", n_output_tokens)):
        if t is not None:
            _check(t, name, torch.int32, 1)
            if t.shape[0] != n:
                raise ValueError(f"{name} must have one entry per request")
    rc = lib.vtc_counter_update(counters.data_ptr(), int(counters.shape[0]), client_ids.data_ptr(),
                                None if n_input_tokens is None else n_input_tokens.data_ptr(),
                                None if n_output_tokens is None else n_output_tokens.data_ptr(),
                                n, int(w_p), int(w_q), _stream())
    if rc != 0:
        raise VtcError(rc, "vtc_counter_update")
    return counters


def vtc_counter_update_cost(counters, client_ids, n_p_old, n_q_old, n_p_new, n_q_new, h: CostPoly,
                            client_multiplier=None):
    """counters[client] += (h(new) - h(old)) * multiplier[client], in place (general / weighted VTC)."""
    torch = _torch()
    lib = load_library()
    _check(counters, "counters", torch.int64, 1)
    _check(client_ids, "client_ids", torch.int32, 1)
    n = int(client_ids.shape[0])
    for name, t in (("n_p_old", n_p_old), ("n_q_old", n_q_old), ("n_p_new", n_p_new), ("n_q_new", n_q_new)):
        _check(t, name, torch.int32, 1)
        if t.shape[0] != n:
            raise ValueError(f"{name} must have one entry per request")
    if client_multiplier is not None:
        _check(client_multiplier, "client_multiplier", torch.int64, 1)
        if client_multiplier.shape[0] != counters.shape[0]:
            raise ValueError("client_multiplier must have one entry per client")
    rc = lib.vtc_counter_update_cost(counters.data_ptr(), int(counters.shape[0]), client_ids.data_ptr(),
                                     n_p_old.data_ptr(), n_q_old.data_ptr(), n_p_new.data_ptr(), n_q_new.data_ptr(),
                                     n, ctypes.byref(h),
                                     None if client_multiplier is None else client_multiplier.data_ptr(), _stream())
    if rc != 0:
        raise VtcError(rc, "vtc_counter_update_cost")
    return counters


def vtc_counter_update_predicted(counters, client_ids, n_output, n_predicted, finished, w_q: int):
    """Per-step adjustment of VTC with length prediction, in place."""
    torch = _torch()
    lib = load_library()
    _check(counters, "counters", torch.int64, 1)
    _check(client_ids, "client_ids", torch.int32, 1)
    n = int(client_ids.shape[0])
    for name, t in (("n_output", n_output), ("n_predicted", n_predicted), ("finished", finished)):
        _check(t, name, torch.int32, 1)
        if t.shape[0] != n:
            raise ValueError(f"{name} must have one entry per request")
    rc = lib.vtc_counter_update_predicted(counters.data_ptr(), int(counters.shape[0]), client_ids.data_ptr(),
                                          n_output.data_ptr(), n_predicted.data_ptr(), finished.data_ptr(), n,
                                          int(w_q), _stream())
    if rc != 0:
        raise VtcError(rc, "vtc_counter_update_predicted")
    return counters


def vtc_kv_append(params: AttnParams, k_new, v_new, cu_new_lens, max_new_len: int, k_cache, v_cache, block_table,
                  seq_lens):
    """Write the new tokens' K/V rows into the paged cache (in place)."""
    torch = _torch()
    lib = load_library()
    elt = _elt_dtype(params)
    _check(k_new, "k_new", elt, 3)
    _check(v_new, "v_new", elt, 3)
    _check(cu_new_lens, "cu_new_lens", torch.int32, 1)
    _check(k_cache, "k_cache", elt, 4)
    _check(v_cache, "v_cache", elt, 4)
    _check(block_table, "block_table", torch.int32, 2)
    _check(seq_lens, "seq_lens", torch.int32, 1)
    n = int(seq_lens.shape[0])
    if cu_new_lens.shape[0] != n + 1:
        raise ValueError("cu_new_lens must be [num_seqs + 1]")
    if tuple(k_new.shape[1:]) != (params.num_kv_heads, params.head_dim) or k_new.shape != v_new.shape:
        raise ValueError("k_new / v_new must be [total_new_tokens, num_kv_heads, head_dim]")
    if tuple(k_cache.shape[1:]) != (params.num_kv_heads, params.block_size, params.head_dim) or k_cache.shape != v_cache.shape:
        raise ValueError("k_cache / v_cache must be [num_blocks, num_kv_heads, block_size, head_dim]")
    if tuple(block_table.shape) != (n, params.max_blocks_per_seq):
        raise ValueError("block_table must be [num_seqs, max_blocks_per_seq]")
    rc = lib.vtc_kv_append(ctypes.byref(params), n, k_new.data_ptr(), v_new.data_ptr(), cu_new_lens.data_ptr(),
                           int(max_new_len), k_cache.data_ptr(), v_cache.data_ptr(), block_table.data_ptr(),
                           seq_lens.data_ptr(), _stream())
    if rc != 0:
        raise VtcError(rc, "vtc_kv_append")


def vtc_debug_gather_slots(params: AttnParams, block_table, seq_lens, cu_out, max_seq_len: int, slots_out):
    torch = _torch()
    lib = load_library()
    _check(block_table, "block_table", torch.int32, 2)
    _check(seq_lens, "seq_lens", torch.int32, 1)
    _check(cu_out, "cu_out", torch.int32, 1)
    _check(slots_out, "slots_out", torch.int32, 1)
    n = int(seq_lens.shape[0])
    rc = lib.vtc_debug_gather_slots(ctypes.byref(params), n, block_table.data_ptr(), seq_lens.data_ptr(),
                                    cu_out.data_ptr(), int(max_seq_len), slots_out.data_ptr(), _stream())
    if rc != 0:
        raise VtcError(rc, "vtc_debug_gather_slots")
    return slots_out
