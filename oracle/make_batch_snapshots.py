"""Write the running-batch snapshots of configurations 3 and 4.

Runs the CPU VTC scheduler (``oracle.scheduler``, Algorithm 2 of the paper)
over the seeded Poisson traces of ``workloads.traces`` and stores the first
execution-stream iteration, after a warm-up, whose decode batch is full
(|B| == max_batch).  The stored file lists, per decoding request, its client,
prompt length, tokens generated so far and context length for this step
(prompt + generated + the current token), and the counters before and after
the step's decode charge.  Calls only ``oracle`` and the input generators.

    python -m oracle.make_batch_snapshots          # rewrites workloads/data/cfg{3,4}_batch.txt

TEST INFRASTRUCTURE ONLY.
"""
from __future__ import annotations

import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from oracle.scheduler import VTCScheduler, simulate  # noqa: E402
from workloads.batches import DATA_DIR  # noqa: E402
from workloads.traces import trace_for_config  # noqa: E402

WARMUP_ITERATIONS = 600
MODEL = {3: "mha_f16", 4: "gqa_bf16"}


def snapshot(config_id: int):
    trace, p = trace_for_config(config_id)
    sched = VTCScheduler(p["num_clients"], p["w_p"], p["w_q"], p["M"], p["L_output"], p["max_batch"])
    hit = []

    def on_step(rec) -> bool:
        if rec.iteration >= WARMUP_ITERATIONS and len(rec.decode_rids) == p["max_batch"]:
            hit.append(rec)
            return True
        return False

    simulate(trace, sched, p["t_decode_s"], p["t_prefill_token_s"], on_step=on_step)
    if not hit:
        raise RuntimeError(f"config {config_id}: the batch never filled after warm-up")
    return hit[0], p, len(trace)


def write(config_id: int) -> str:
    rec, p, n_trace = snapshot(config_id)
    path = os.path.join(DATA_DIR, f"cfg{config_id}_batch.txt")
    seq = [a + b + 1 for a, b in zip(rec.decode_n_input, rec.decode_generated_before)]
    with open(path, "w", encoding="ascii") as fh:
        fh.write(f"# config: {config_id}\n")
        fh.write(f"# model: {MODEL[config_id]}\n")
        fh.write(f"# num_clients: {p['num_clients']}\n")
        fh.write(f"# w_p: {p['w_p']}\n# w_q: {p['w_q']}\n")
        fh.write(f"# M: {p['M']}\n# L_output: {p['L_output']}\n# max_batch: {p['max_batch']}\n")
        fh.write(f"# trace_requests: {n_trace}\n")
        fh.write(f"# iteration: {rec.iteration}\n")
        fh.write(f"# virtual_time_s: {rec.time_s:.6f}\n")
        fh.write(f"# admitted_this_iteration: {len(rec.admitted)}\n")
        fh.write(f"# total_context_tokens: {sum(seq)}\n")
        fh.write("# counters_before_decode_charge: " + " ".join(map(str, rec.counters_before_decode_charge)) + "\n")
        fh.write("# counters_after_decode_charge: " + " ".join(map(str, rec.counters_after_decode_charge)) + "\n")
        fh.write("# columns = rid client n_input n_generated seq_len\n")
        for rid, cl, n_in, gen, s in zip(rec.decode_rids, rec.decode_clients, rec.decode_n_input,
                                         rec.decode_generated_before, seq):
            fh.write(f"{rid} {cl} {n_in} {gen} {s}\n")
    return path


if __name__ == "__main__":
    for cfg in (3, 4):
        print(write(cfg))
