"""Baseline schedulers of the paper's evaluation (Section 5.1) and its fairness metrics, CPU only.

* FCFS  -- requests are admitted strictly in arrival order, whoever sent them.
* RPM(k) -- at most k requests per client are accepted per one-minute window; a request over the
            limit is held back until the next window starts (then queued FCFS).
* LCF   -- ``oracle.scheduler.VTCScheduler(lift=False)``.
The memory-fit rule and the virtual clock are those of ``oracle.scheduler`` so that runs are comparable.

Metrics (Section 5.1): accumulated service W_i(0, t) with the weighted-token cost, the maximal pairwise
difference max_{i,j} |W_i - W_j|, and the "service difference" between two clients,
min(s_2 - s_1, |r_1 - s_1|) for s_1 <= s_2, where r_1 is the service the less-served client asked for.

TEST INFRASTRUCTURE ONLY.
"""
from __future__ import annotations

from collections import deque
from typing import Callable, List, Optional, Sequence

from .scheduler import Running, StepRecord


class FCFSScheduler:
    """Continuous batching (Algorithm 1) with first-come-first-serve selection."""

    def __init__(self, num_clients: int, w_p: int, w_q: int, M: int, L_output: int,
                 max_batch: Optional[int] = None, rpm_limit: Optional[int] = None) -> None:
        self.num_clients = num_clients
        self.w_p, self.w_q, self.M, self.L_output = int(w_p), int(w_q), int(M), int(L_output)
        self.max_batch = max_batch
        self.rpm_limit = rpm_limit
        self.queue = deque()                      # admitted to the waiting queue, in arrival order
        self.held: List[deque] = [deque() for _ in range(num_clients)]   # over the RPM limit, per client
        self.window_start = 0.0
        self.window_count = [0] * num_clients
        self.B: List[Running] = []
        self.reserved = 0
        self.service = [0] * num_clients
        self.requested = [0] * num_clients        # service asked for so far: sum of w_p*n_p + w_q*n_q of arrivals
        self.iteration = 0
        self.now = 0.0

    # -- monitoring stream
    def _roll_window(self, t: float) -> None:
        while t >= self.window_start + 60.0:
            self.window_start += 60.0
            self.window_count = [0] * self.num_clients
            for c in range(self.num_clients):     # blocked requests enter at the start of the new window
                while self.held[c] and (self.rpm_limit is None or self.window_count[c] < self.rpm_limit):
                    self.queue.append(self.held[c].popleft())
                    self.window_count[c] += 1

    def on_arrival(self, req) -> None:
        self._roll_window(req.arrival)
        self.requested[req.client] += self.w_p * req.n_input + self.w_q * req.n_output
        if self.rpm_limit is not None and self.window_count[req.client] >= self.rpm_limit:
            self.held[req.client].append(req)
            return
        self.window_count[req.client] += 1
        self.queue.append(req)

    # -- execution stream
    def step(self, time_s: float = 0.0, admit: bool = True) -> StepRecord:
        self._roll_window(time_s)
        new: List[Running] = []
        while admit and self.queue:
            r = self.queue[0]
            if self.max_batch is not None and len(self.B) + len(new) >= self.max_batch:
                break
            if self.reserved + r.n_input + self.L_output > self.M:
                break
            self.queue.popleft()
            self.reserved += r.n_input + self.L_output
            self.service[r.client] += self.w_p * r.n_input
            new.append(Running(r.rid, r.client, r.n_input, r.n_output))
        self.B.extend(new)
        rec = StepRecord(self.iteration, time_s, new, [x.rid for x in self.B], [x.client for x in self.B],
                         [x.n_input for x in self.B], [x.generated for x in self.B], [], [], [])
        for x in self.B:
            x.generated += 1
            self.service[x.client] += self.w_q
        rec.finished = [x for x in self.B if x.generated >= x.n_output]
        self.B = [x for x in self.B if x.generated < x.n_output]
        for x in rec.finished:
            self.reserved -= x.n_input + self.L_output
        self.iteration += 1
        return rec

    def idle(self) -> bool:
        return not self.B and not self.queue

    def has_held(self) -> bool:
        return any(self.held)


def simulate_baseline(trace: Sequence, sched: FCFSScheduler, t_decode_s: float, t_prefill_token_s: float,
                      on_step: Optional[Callable[[StepRecord], bool]] = None) -> List[StepRecord]:
    records: List[StepRecord] = []
    t, nxt, n = 0.0, 0, len(trace)
    while nxt < n or not sched.idle() or sched.has_held():
        while nxt < n and trace[nxt].arrival <= t:
            sched.on_arrival(trace[nxt])
            nxt += 1
        if sched.idle():
            if nxt < n:
                t_next = trace[nxt].arrival
                if sched.has_held():
                    t_next = min(t_next, sched.window_start + 60.0)
            elif sched.has_held():
                t_next = sched.window_start + 60.0
            else:
                break
            t = max(t, t_next)
            sched._roll_window(t)
            continue
        rec = sched.step(time_s=t)
        t += t_decode_s + t_prefill_token_s * sum(x.n_input for x in rec.admitted)
        records.append(rec)
        if on_step is not None and on_step(rec):
            break
    return records


def max_pairwise_difference(service: Sequence[int]) -> int:
    """max_{i,j} |W_i - W_j| (Section 5.1, absolute difference in accumulated service)."""
    return max(service) - min(service)


def service_difference(s1: float, s2: float, r1: float, r2: float) -> float:
    """Section 5.1: min(s_hi - s_lo, |r_lo - s_lo|) where lo is the client that received less service."""
    if s1 <= s2:
        return min(s2 - s1, abs(r1 - s1))
    return min(s1 - s2, abs(r2 - s2))
