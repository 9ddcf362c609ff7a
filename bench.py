#!/usr/bin/env python3
"""Benchmark of one VTC serving step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg3|cfg4|cfg5] [--no-cpu-baseline]
                    [--no-other-configs]

A step is one pass of the hot path over one synthetic batch that is already
resident in HBM: decode attention over the paged KV cache of every running
request, the prefill-chunk attention of newly admitted prompts when the
workload has any (cfg5), and one virtual-token-counter update for the whole
batch (carried by the decode call's last launch: ``vtc_step_decode``).  Prints ONE JSON line: whole-step KV GB/s as ``value``, plus the
roofline of the dominant kernel (decode attention, HBM-bound; its duration is
measured with HIP events recorded on the launch stream right around that
kernel) and the CPU oracle timed on a bounded sample of the same workload.
Unless --no-other-configs is given, the line also carries, under
"other_configs", the decode kernel on the other configurations and the
prefill-chunk kernel on both chunks of cfg5 (a second or two in all).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0      # dense bf16 / fp16
EVENT_EVERY = 5                # steps between two kernel-level HIP event pairs

# HBM bytes per launch of decode_attend_kernel on cfg3 from rocprofv3 FETCH_SIZE / WRITE_SIZE counters, scaled
# by the copy-kernel calibration (profiles/decode_attend_cfg3_hbm_bytes.md).  Valid only for the kernel
# source the counters were taken with: keyed by the SHA-256 of the two files that define that kernel.
DECODE_TRAFFIC_CFG3 = {
    "c4da850657273659": 4060144550,
}
# The same counters for the decode kernel on cfg4 / cfg5 and for the prefill kernel on the two cfg5 chunks
# (profiles/decode_attend_cfg4_kernel_trace.md, profiles/mixed_step_cfg5_kernel_trace.md).
DECODE_TRAFFIC_OTHER = {
    4: {"c4da850657273659": 1169578684},
    5: {"c4da850657273659": 2108728181},
}
PREFILL_TRAFFIC_CFG5 = {
    0: {"20a71fd2a92a36be": 84122384},
    1: {"20a71fd2a92a36be": 100899308},
}


def decode_kernel_fingerprint() -> str:
    import hashlib

    h = hashlib.sha256()
    for name in ("attn_decode.hip", "vtc_internal.h"):
        with open(os.path.join(ROOT, "paper_2401_00588_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def prefill_kernel_fingerprint() -> str:
    import hashlib

    h = hashlib.sha256()
    for name in ("attn_prefill.hip", "vtc_internal.h"):
        with open(os.path.join(ROOT, "paper_2401_00588_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def decode_traffic(cfg):
    """Measured HBM bytes per launch of the decode kernel on ``cfg``, or None (not measured, or the kernel changed)."""
    table = DECODE_TRAFFIC_CFG3 if cfg == 3 else DECODE_TRAFFIC_OTHER.get(cfg, {})
    return table.get(decode_kernel_fingerprint())


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--prefill-chunk", type=int, default=1, choices=[0, 1], help="cfg5: which 256-token chunk")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other configurations (key other_configs)")
    ap.add_argument("--cpu-sample-requests", type=int, default=256,
                    help="decode requests handed to the CPU oracle (default: the whole cfg3 batch, ~20 core-seconds)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the benchmark, run a plain 1 GiB device copy a few times "
                         "(reference dispatch of known size for scaling rocprofv3 byte counters)")
    return ap.parse_args()


def cpu_baseline(st, scale, sample_requests):
    """Time the fp64 oracle on a bounded sample of the decode batch, on the host cores."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor

    from oracle import attention as OA          # the only use of the oracle here: the reported CPU baseline
    from workloads import tensor_to_bits

    try:
        from threadpoolctl import threadpool_limits
    except Exception:                            # pragma: no cover
        threadpool_limits = None
    b = st.batch
    sh = b.shape
    rng = np.random.default_rng(7)
    picks = sorted(int(x) for x in rng.choice(b.num_decode, size=min(sample_requests, b.num_decode), replace=False))
    # compact copy of the sampled requests' blocks (host), with a remapped block table
    bs = sh.block_size
    tables, blocks, at = [], [], 0
    width = max((int(b.seq_lens[r]) + bs - 1) // bs for r in picks)
    for r in picks:
        nb = (int(b.seq_lens[r]) + bs - 1) // bs
        blocks.append(st.block_table[r, :nb].long())
        row = np.zeros(width, dtype=np.int32)
        row[:nb] = np.arange(at, at + nb)
        tables.append(row)
        at += nb
    import torch

    idx = torch.cat(blocks)
    k_bits = tensor_to_bits(st.k_cache[idx])
    v_bits = tensor_to_bits(st.v_cache[idx])
    q_bits = tensor_to_bits(st.q[torch.as_tensor(picks, device=st.q.device)])
    table = np.stack(tables)
    seq = [int(b.seq_lens[r]) for r in picks]
    cores = max(1, min(16, os.cpu_count() or 1, len(picks)))

    def one(i):
        return OA.paged_decode(q_bits[i:i + 1], k_bits, v_bits, table[i:i + 1], seq[i:i + 1], scale, sh.dtype)

    def run():
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as pool:
            list(pool.map(one, range(len(picks))))
        return time.perf_counter() - t0

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            secs = run()
    else:
        secs = run()
    kv_bytes = sum(seq) * sh.kv_bytes_per_token
    # the small correctness configuration on one core, for scale (8 requests, ~18 MB of KV, host-generated inputs)
    from workloads import make_qkv_numpy, make_block_table, make_step_batch
    b1 = make_step_batch(1)
    rng1 = np.random.default_rng(1)
    table1, nb1 = make_block_table(rng1, b1.seq_lens, b1.shape.block_size)
    q1, k1, v1 = make_qkv_numpy(rng1, b1.num_decode, b1.shape.num_q_heads, b1.shape.num_kv_heads, b1.shape.head_dim,
                                nb1, b1.shape.block_size, b1.shape.dtype)
    t0 = time.perf_counter()
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            OA.paged_decode(q1, k1, v1, table1, b1.seq_lens, scale, b1.shape.dtype)
    else:
        OA.paged_decode(q1, k1, v1, table1, b1.seq_lens, scale, b1.shape.dtype)
    secs1 = time.perf_counter() - t0
    kv1 = int(sum(int(x) for x in b1.seq_lens)) * b1.shape.kv_bytes_per_token
    return {
        "value": kv_bytes / secs / 1e9,
        "unit": "GB/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"{len(picks)} of {b.num_decode} decode requests x all {sh.num_q_heads} q heads "
                  f"({sum(seq)} context tokens, {kv_bytes / 1e6:.1f} MB of KV), fp64 numpy, {secs:.2f} s",
        "seconds": secs,
        "one_core_cfg1": {"seconds": round(secs1, 4), "value": round(kv1 / secs1 / 1e9, 4), "unit": "GB/s",
                          "sample": f"cfg1: {b1.num_decode} requests, {kv1 / 1e6:.1f} MB of KV, 1 thread"},
    }


def aux_kernel_times(torch, vtc, st, params, stream, reps: int = 50):
    """Average GPU time (us) of the small kernels around attention, on this batch: appending the batch's
    current tokens to the cache, and the three counter updates.  Latency-bound; reported, not rooflined."""
    b = st.batch
    sh = b.shape
    n = b.num_decode
    dev = st.q.device
    k_new = torch.randn((n, sh.num_kv_heads, sh.head_dim), device=dev).to(st.k_cache.dtype)
    v_new = torch.randn((n, sh.num_kv_heads, sh.head_dim), device=dev).to(st.k_cache.dtype)
    cu = torch.arange(n + 1, dtype=torch.int32, device=dev)
    ids = st.cu_client_ids[:n].contiguous()
    zeros = torch.zeros(n, dtype=torch.int32, device=dev)
    ones = torch.ones(n, dtype=torch.int32, device=dev)
    n_in = (st.seq_lens - 1).clamp(min=0).to(torch.int32)
    h = vtc.CostPoly(11460, 2100, 1000, 0, 40, 32)
    scratch = st.counters.clone()

    def timed(fn):
        with torch.cuda.stream(stream):
            for _ in range(5):
                fn()
            a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(reps):
                fn()
            e.record(stream)
            e.synchronize()
        return round(a.elapsed_time(e) * 1e3 / reps, 2)

    # the append rewrites the rows of the current tokens with fresh values; it runs after all attention timing
    return {
        "kv_append_current_tokens": timed(lambda: vtc.vtc_kv_append(params, k_new, v_new, cu, 1, st.k_cache,
                                                                    st.v_cache, st.block_table, st.seq_lens)),
        "counter_update": timed(lambda: vtc.vtc_counter_update(scratch, ids, None, ones, b.w_p, b.w_q)),
        "counter_update_cost_profiled": timed(lambda: vtc.vtc_counter_update_cost(scratch, ids, n_in, zeros, n_in,
                                                                                  ones, h)),
        "counter_update_predicted": timed(lambda: vtc.vtc_counter_update_predicted(scratch, ids, ones, zeros, zeros,
                                                                                   b.w_q)),
        "note": "back-to-back launches on one stream, average per launch",
    }


def decode_kernel_on(torch, vtc, cfg, steps=20, warmup=5):
    """Decode kernel time on configuration ``cfg``: a short run of whole decode steps with a HIP event pair around
    the attention kernel on every 4th step (rotating over copies of a small cache, as in the main run)."""
    from workloads import make_device_step, make_step_batch

    batch = make_step_batch(cfg)
    st = make_device_step(batch)
    sh = batch.shape
    params = vtc.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.block_size, st.max_blocks_per_seq,
                             sh.dtype, 1.0 / math.sqrt(sh.head_dim))
    ws = torch.empty(vtc.vtc_attn_workspace_bytes(params, batch.num_decode, 0), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(st.q)
    cache_bytes = 2 * st.k_cache.numel() * st.k_cache.element_size()
    n_copies = 1 if cache_bytes >= (1 << 30) else min(16, -(-(2 << 30) // cache_bytes))
    ks = [st.k_cache] + [st.k_cache.clone() for _ in range(n_copies - 1)]
    vs = [st.v_cache] + [st.v_cache.clone() for _ in range(n_copies - 1)]
    stream = torch.cuda.Stream()
    timed = [i for i in range(steps) if i % 4 == 0]
    evs = {i: (vtc.HipEvent(), vtc.HipEvent()) for i in timed}
    with torch.cuda.stream(stream):
        for i in range(-warmup, steps):
            eb, ee = evs.get(i, (None, None))
            vtc.vtc_step_decode(params, st.q, ks[i % n_copies], vs[i % n_copies], st.block_table, st.seq_lens,
                                st.counters, st.cu_client_ids[:batch.num_decode].contiguous(), None,
                                st.cu_n_out[:batch.num_decode].contiguous(), batch.w_p, batch.w_q, out=out,
                                workspace=ws, ev_begin=eb, ev_end=ee)
            if i == -1:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
        torch.cuda.synchronize()
        step_ms = (time.perf_counter() - t0) * 1e3 / steps
    ms = sorted(a.elapsed_ms(b) for a, b in evs.values())
    avg = sum(ms) / len(ms)
    kv = batch.decode_kv_bytes
    return {"kernel": "decode_attend_kernel", "requests": batch.num_decode, "kv_bytes": kv, "dtype": sh.dtype,
            "kernel_avg_ms": round(avg, 5), "kernel_min_ms": round(ms[0], 5), "achieved": round(kv / avg / 1e6, 1),
            "unit": "GB/s", "frac": round(kv / avg / 1e6 / HBM_PEAK_GBS, 4), "traffic": decode_traffic(cfg),
            "step_ms": round(step_ms, 5),
            "kv_cache_copies": n_copies}


def prefill_kernel_on_cfg5(torch, vtc, chunk, launches=24, reps=5, rotate=6):
    """Prefill-chunk kernel time on chunk ``chunk`` of cfg5 (16 prompts x 256 chunk tokens, GQA 32/8 bf16): ``launches``
    back-to-back launches between one event pair, over ``rotate`` distinct sets of inputs and outputs (q, out and
    the paged cache: ~100 MB each, more than the last-level cache in all), so that every launch streams from HBM and
    no event sits between two kernels.  Average time per launch, median over ``reps`` such runs."""
    import numpy as np

    from workloads import make_block_table, make_step_batch

    batch = make_step_batch(5, prefill_chunk=chunk)
    sh = batch.shape
    n, lq, s_len = batch.num_prefill, int(batch.pf_q_lens[0]), int(batch.pf_seq_lens[0])
    sets = []
    for i in range(rotate):
        table, nb = make_block_table(np.random.default_rng(500 + 10 * chunk + i), [s_len] * n, sh.block_size)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(500 + 10 * chunk + i)
        mk = lambda *shape: torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        sets.append((mk(n * lq, sh.num_q_heads, sh.head_dim), mk(nb, sh.num_kv_heads, sh.block_size, sh.head_dim),
                     mk(nb, sh.num_kv_heads, sh.block_size, sh.head_dim), torch.from_numpy(table).cuda(),
                     torch.empty((n * lq, sh.num_q_heads, sh.head_dim), dtype=torch.bfloat16, device="cuda")))
    cu = torch.arange(0, n * lq + 1, lq, dtype=torch.int32, device="cuda")
    seq = torch.full((n,), s_len, dtype=torch.int32, device="cuda")
    params = vtc.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.block_size, sets[0][3].shape[1], sh.dtype,
                             1.0 / math.sqrt(sh.head_dim))

    def launch(i):
        q, k, v, table, out = sets[i % rotate]
        vtc.vtc_attn_prefill_chunk(params, q, cu, lq, k, v, table, seq, out=out)

    for i in range(2 * launches):                    # warm-up: clocks, TLBs, instruction cache
        launch(i)
    torch.cuda.synchronize()
    per_launch = []
    for _ in range(reps):
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(launches):
            launch(i)
        e.record()
        e.synchronize()
        per_launch.append(a.elapsed_time(e) / launches)
    per_launch.sort()
    ms = per_launch[len(per_launch) // 2]
    tf = batch.prefill_flops / ms / 1e9
    # the bytes that must cross HBM at least once: q rows in, output rows out, K and V of every sequence's context
    esz = 2
    hbm_bytes = (2 * n * lq * sh.num_q_heads + 2 * n * s_len * sh.num_kv_heads) * sh.head_dim * esz
    return {"kernel": "prefill_chunk_kernel", "chunk": chunk, "flops": batch.prefill_flops, "dtype": sh.dtype,
            "ms_per_launch": round(ms, 5), "ms_per_launch_min": round(per_launch[0], 5), "achieved": round(tf, 1),
            "unit": "TFLOP/s", "frac": round(tf / MFMA_PEAK_TFLOPS, 4),
            "hbm_bytes": hbm_bytes, "traffic": PREFILL_TRAFFIC_CFG5[chunk].get(prefill_kernel_fingerprint()),
            "hbm_gbs": round(hbm_bytes / ms / 1e6, 1),
            "hbm_frac": round(hbm_bytes / ms / 1e6 / HBM_PEAK_GBS, 4),
            "flop_per_byte": round(batch.prefill_flops / hbm_bytes, 1),
            "method": f"{launches} back-to-back launches over {rotate} distinct input sets per event pair"}


def main() -> int:
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "the serving step has no multi-GPU path.", file=sys.stderr)
        return 2

    import torch

    import paper_2401_00588_amd as vtc
    from workloads import make_device_step, make_step_batch

    vtc.load_library()                           # fail loudly if the HIP extension is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 256)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "device copy", "bytes_read": n, "bytes_written": n, "dispatches": 4}))
        return 0
    cfg = int(args.workload[3:])
    batch = make_step_batch(cfg, prefill_chunk=args.prefill_chunk) if cfg == 5 else make_step_batch(cfg)
    st = make_device_step(batch)
    sh = batch.shape
    scale = 1.0 / math.sqrt(sh.head_dim)
    params = vtc.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.block_size, st.max_blocks_per_seq,
                             sh.dtype, scale)
    ws = torch.empty(vtc.vtc_attn_workspace_bytes(params, batch.num_decode, 0), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(st.q)
    pf_out = torch.empty_like(st.pf_q) if batch.num_prefill else None
    stream = torch.cuda.Stream()
    # A cache smaller than 1 GiB would be served, in part, from the 256 MB last-level cache when every step reads the
    # same copy: such workloads rotate over enough identical copies of the paged cache (2 GiB worth, 16 at most) that
    # every timed step streams its K/V from HBM.
    cache_bytes = 2 * st.k_cache.numel() * st.k_cache.element_size()
    n_copies = 1 if cache_bytes >= (1 << 30) else min(16, -(-(2 << 30) // cache_bytes))
    k_copies = [st.k_cache] + [st.k_cache.clone() for _ in range(n_copies - 1)]
    v_copies = [st.v_cache] + [st.v_cache.clone() for _ in range(n_copies - 1)]
    calls = [0]

    def step(ev_b=None, ev_e=None, pf_ev=None):
        k_cache, v_cache = k_copies[calls[0] % n_copies], v_copies[calls[0] % n_copies]
        calls[0] += 1
        if batch.num_prefill:
            if pf_ev is not None:
                pf_ev[0].record(stream)
            vtc.vtc_attn_prefill_chunk(params, st.pf_q, st.pf_cu_q_lens, st.pf_max_q_len, k_cache, v_cache,
                                       st.pf_block_table, st.pf_seq_lens, out=pf_out)
            if pf_ev is not None:
                pf_ev[1].record(stream)
        # decode attention and the step's counter charge (decoding and newly prefilled requests) in one call
        vtc.vtc_step_decode(params, st.q, k_cache, v_cache, st.block_table, st.seq_lens, st.counters,
                            st.cu_client_ids, st.cu_n_in, st.cu_n_out, batch.w_p, batch.w_q, out=out, workspace=ws,
                            ev_begin=ev_b, ev_end=ev_e)

    # The kernel-level events sit inside the timed region, on the launch stream, but only on every
    # EVENT_EVERY-th step: an event between two kernels costs a few microseconds of queue drain.
    timed = [i for i in range(args.steps) if i % EVENT_EVERY == 0]
    begins = {i: vtc.HipEvent() for i in timed}
    ends = {i: vtc.HipEvent() for i in timed}
    pf_events = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                 for i in timed} if batch.num_prefill else None
    with torch.cuda.stream(stream):
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(begins.get(i), ends.get(i), pf_events.get(i) if pf_events else None)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernel_ms = sorted(begins[i].elapsed_ms(ends[i]) for i in timed)
    kernel_avg_ms = sum(kernel_ms) / len(kernel_ms)

    kv_bytes = batch.decode_kv_bytes
    value = kv_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = kv_bytes / (kernel_avg_ms * 1e-3) / 1e9
    line = {
        "metric": "decode attention KV GB/s (% of HBM peak) + batch tokens/s per step, 1 GPU",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": sh.dtype,
        "data": "synthetic",
        "config": {
            "workload": {2: "cfg2: 64-request Llama-2-7B-shaped decode", 3: "cfg3: 4-client mixed decode, 256 requests, "
                         "MHA 32 heads, head_dim 128, fp16, block 16, batch admitted by the CPU VTC scheduler",
                         4: "cfg4: 27-client GQA 32/8 bf16 decode, 512 requests",
                         5: f"cfg5: mixed step, 16 prompts x 256-token prefill chunk {args.prefill_chunk} + 256 decodes, GQA 32/8 bf16"}[cfg],
            "requests": batch.num_decode,
            "context_tokens": int(batch.seq_lens.sum()),
            "kv_bytes": kv_bytes,
            "clients": batch.num_clients,
            "prefill_tokens": int(batch.pf_q_lens.sum()) if batch.num_prefill else 0,
            "kv_cache_copies": n_copies,
        },
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "tokens_per_s": round(batch.tokens_advanced / (ms_per_step * 1e-3), 1),
        "roofline": {
            "kernel": "decode_attend_kernel",
            "bound": "hbm",
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": decode_traffic(cfg),
            "kernel_avg_ms": round(kernel_avg_ms, 5),
            "kernel_min_ms": round(kernel_ms[0], 5),
            "kernel_median_ms": round(kernel_ms[len(kernel_ms) // 2], 5),
            "kernel_samples": len(kernel_ms),
            "algorithmic_bytes_per_launch": kv_bytes,
        },
    }
    if pf_events:
        pf_ms = sorted(a.elapsed_time(b) for a, b in pf_events.values())
        pf_avg = sum(pf_ms) / len(pf_ms)
        line["prefill"] = {
            "kernel": "prefill_chunk_kernel",
            "bound": "mfma",
            "flops": batch.prefill_flops,
            "avg_ms": round(pf_avg, 5),
            "achieved": round(batch.prefill_flops / (pf_avg * 1e-3) / 1e12, 2),
            "peak": MFMA_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(batch.prefill_flops / (pf_avg * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4),
            "note": "one launch between two events inside the mixed step (the events add a few us); "
                    "other_configs holds the back-to-back figure",
        }
    line["aux_kernels_us"] = aux_kernel_times(torch, vtc, st, params, stream)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(st, scale, args.cpu_sample_requests)
        line["cpu_baseline"]["value"] = round(line["cpu_baseline"]["value"], 4)
        line["cpu_baseline"]["seconds"] = round(line["cpu_baseline"]["seconds"], 3)
    if not args.no_other_configs:
        st = k_copies = v_copies = out = pf_out = ws = None            # free the main workload's memory first
        torch.cuda.empty_cache()
        others = {}
        for c in (2, 3, 4, 5):
            if c != cfg:
                others[f"cfg{c}_decode"] = decode_kernel_on(torch, vtc, c)
                torch.cuda.empty_cache()
        for chunk in (0, 1):
            others[f"cfg5_prefill_chunk{chunk}"] = prefill_kernel_on_cfg5(torch, vtc, chunk)
            torch.cuda.empty_cache()
        line["other_configs"] = others
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
