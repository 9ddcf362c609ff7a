"""Batch shapes of one serving step for the five benchmark configurations.

A *step batch* says, for one iteration of the execution stream (Algorithm 2 of
the paper), which requests decode (context length and client of each) and
which newly admitted prompts are prefilled (chunk length, context length after
the chunk, client).  Configurations 1, 2 and 5 are drawn directly from a
seeded generator; configurations 3 and 4 are snapshots of a running batch that
a CPU VTC scheduler produced from a seeded Poisson trace -- those snapshots
are small text files under ``workloads/data`` and are only *read* here.
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field
from typing import Dict, List

import numpy as np

from .traces import SEED_BASE

CONFIG_IDS = (1, 2, 3, 4, 5)
DATA_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "data")


@dataclass(frozen=True)
class ModelShape:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    dtype: str  # "f16" | "bf16"

    @property
    def elt_bytes(self) -> int:
        return 2

    @property
    def kv_bytes_per_token(self) -> int:
        """K and V bytes of one context token over all KV heads (one layer)."""
        return 2 * self.num_kv_heads * self.head_dim * self.elt_bytes


MHA_F16 = ModelShape(32, 32, 128, 16, "f16")
GQA_BF16 = ModelShape(32, 8, 128, 16, "bf16")


@dataclass
class StepBatch:
    config_id: int
    shape: ModelShape
    num_clients: int
    w_p: int
    w_q: int
    # decoding requests: one query token each
    seq_lens: np.ndarray            # int32 [Nd], context length including the current token
    client_ids: np.ndarray          # int32 [Nd]
    # prompts prefilled in this step (possibly one chunk of a longer prompt)
    pf_client_ids: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    pf_q_lens: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))      # chunk length
    pf_seq_lens: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))    # context after the chunk
    pf_prompt_lens: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))  # whole prompt
    counters_before: np.ndarray | None = None   # int64 [num_clients]
    counters_after: np.ndarray | None = None    # as recorded by the scheduler that made the snapshot
    meta: Dict[str, str] = field(default_factory=dict)

    def __post_init__(self) -> None:
        if self.counters_before is None:
            self.counters_before = np.zeros(self.num_clients, dtype=np.int64)

    @property
    def num_decode(self) -> int:
        return int(self.seq_lens.shape[0])

    @property
    def num_prefill(self) -> int:
        return int(self.pf_q_lens.shape[0])

    @property
    def decode_kv_bytes(self) -> int:
        """Algorithmic K/V bytes one decode step reads: valid tokens only."""
        return int(self.seq_lens.astype(np.int64).sum()) * self.shape.kv_bytes_per_token

    @property
    def prefill_causal_pairs(self) -> int:
        """Unmasked (query, key) pairs per q-head over all prefill chunks."""
        total = 0
        for lq, s in zip(self.pf_q_lens.tolist(), self.pf_seq_lens.tolist()):
            first = s - lq  # keys visible to the first chunk token, minus one
            total += lq * first + lq * (lq + 1) // 2
        return total

    @property
    def prefill_flops(self) -> int:
        return 4 * self.shape.head_dim * self.shape.num_q_heads * self.prefill_causal_pairs

    @property
    def tokens_advanced(self) -> int:
        """Tokens the step processes: one per decoding request plus the chunk tokens."""
        return self.num_decode + int(self.pf_q_lens.astype(np.int64).sum())

    def counter_update_args(self, first_chunk: bool = True):
        """Arrays for one counter update covering the whole step.

        Decoding requests contribute one output token each.  Prefilling
        requests contribute their whole prompt on the step that admits them
        (``first_chunk``) and nothing on later chunks, which is when
        Algorithm 2 charges input tokens.
        """
        ids = np.concatenate([self.client_ids, self.pf_client_ids]).astype(np.int32)
        n_out = np.concatenate([np.ones(self.num_decode, np.int32), np.zeros(self.num_prefill, np.int32)])
        charged = self.pf_prompt_lens if first_chunk else np.zeros(self.num_prefill, np.int32)
        n_in = np.concatenate([np.zeros(self.num_decode, np.int32), charged.astype(np.int32)])
        return ids, n_in, n_out


def load_snapshot(config_id: int) -> StepBatch:
    """Read ``workloads/data/cfg<N>_batch.txt`` (see ``oracle/make_batch_snapshots.py``)."""
    path = os.path.join(DATA_DIR, f"cfg{config_id}_batch.txt")
    meta: Dict[str, str] = {}
    rows: List[List[int]] = []
    with open(path, "r", encoding="ascii") as fh:
        for line in fh:
            line = line.strip()
            if not line:
                continue
            if line.startswith("#"):
                if ":" in line:
                    key, val = line[1:].split(":", 1)
                    meta[key.strip()] = val.strip()
                continue
            rows.append([int(tok) for tok in line.split()])
    arr = np.asarray(rows, dtype=np.int64)  # rid client n_input n_generated seq_len
    shape = MHA_F16 if meta["model"] == "mha_f16" else GQA_BF16
    ints = lambda key: np.asarray([int(t) for t in meta[key].split()], dtype=np.int64)
    return StepBatch(
        config_id=config_id,
        shape=shape,
        num_clients=int(meta["num_clients"]),
        w_p=int(meta["w_p"]),
        w_q=int(meta["w_q"]),
        seq_lens=arr[:, 4].astype(np.int32),
        client_ids=arr[:, 1].astype(np.int32),
        counters_before=ints("counters_before_decode_charge"),
        counters_after=ints("counters_after_decode_charge"),
        meta=meta,
    )


def make_step_batch(config_id: int, prefill_chunk: int = 0) -> StepBatch:
    """The step batch of configuration 1..5 (``prefill_chunk`` selects chunk 0 or 1 of config 5)."""
    rng = np.random.default_rng(SEED_BASE + config_id)
    if config_id == 1:
        seq = rng.integers(16, 257, size=8).astype(np.int32)
        cid = np.asarray([0, 0, 0, 0, 1, 1, 1, 1], dtype=np.int32)
        return StepBatch(1, MHA_F16, 2, 1, 2, seq, cid)
    if config_id == 2:
        # client A (prompt 256, up to 256 generated) arrives twice as often as
        # client B (prompt 512, up to 128 generated): 43 + 21 requests.
        seq_a = rng.integers(256, 513, size=43)
        seq_b = rng.integers(512, 641, size=21)
        seq = np.concatenate([seq_a, seq_b]).astype(np.int32)
        cid = np.concatenate([np.zeros(43, np.int32), np.ones(21, np.int32)])
        order = rng.permutation(64)
        return StepBatch(2, MHA_F16, 2, 1, 2, seq[order], cid[order])
    if config_id in (3, 4):
        return load_snapshot(config_id)
    if config_id == 5:
        seq = rng.integers(128, 4097, size=256).astype(np.int32)
        cid = rng.integers(0, 8, size=256).astype(np.int32)
        pf_cid = rng.integers(0, 8, size=16).astype(np.int32)
        if prefill_chunk not in (0, 1):
            raise ValueError("config 5 has prefill chunks 0 and 1")
        pf_q = np.full(16, 256, np.int32)
        pf_s = np.full(16, 256 * (prefill_chunk + 1), np.int32)
        pf_p = np.full(16, 512, np.int32)
        return StepBatch(5, GQA_BF16, 8, 1, 2, seq, cid, pf_cid, pf_q, pf_s, pf_p,
                         meta={"prefill_chunk": str(prefill_chunk)})
    raise ValueError(f"unknown config {config_id}")
