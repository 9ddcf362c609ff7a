"""Virtual Token Counter scheduler (Algorithm 2 of the paper) on a virtual clock.

State follows the paper's notation: counters c_i (one per client, start at 0),
the waiting queue Q (here one FIFO per client, since the algorithm only ever
takes "the earliest request in Q from client k"), the running batch B, and the
weights w_p, w_q.

Monitoring stream  -> ``on_arrival``:   counter lift, then enqueue.
Execution stream   -> ``step``:         select a minibatch by repeatedly taking
    the waiting client with the smallest counter, charge w_p * input_length at
    admission, "prefill" it, merge it into B, "decode" B (one token per
    request), charge w_q per request of B, then drop finished requests.

Points the paper leaves open, and the reading taken here:
  * argmin ties: smallest client id.
  * "the last client left Q": the client whose queue most recently became
    empty because its request was moved into the minibatch; before any client
    ever left, no lift happens on an empty queue.
  * lift value: exactly max(c_u, min over waiting clients), as printed.
  * can_add_new_request(): every ``admit_every``-th iteration (default: all).
  * "r cannot fit in the memory": no preemption exists, so every admitted
    request reserves input_length + L_output tokens of the pool M; r fits iff
    the reservations of B, of the minibatch so far and of r are <= M, and the
    batch has fewer than ``max_batch`` requests (a harness cap, not in the
    paper).  The scheduler never looks at a request's hidden output length.
  * when the smallest-counter client's head request does not fit: stop
    filling the minibatch (break), as printed; no skipping to another client.
  * the decode charge precedes the removal of finished requests, so a request
    is charged for the step in which it finishes.
  * a request with output length n_q takes part in exactly n_q decode steps;
    prefill itself charges no w_q.  Its total charge is w_p*n_p + w_q*n_q,
    the weighted-token cost of Section 3.1.
  * simultaneous arrivals are ordered by request id.
  * time: a fixed cost per decode iteration plus a cost per prefilled token;
    this only decides *which* arrivals land before which iteration.

``lift=False`` gives the Least Counter First baseline of Section 5.1.

Two variants of the paper are switched on by constructor arguments:
  * ``cost=h`` (Section 4.2 / Algorithm 4): admission charges h(n_p, 0) and a decode step charges
    h(n_p, n_q) - h(n_p, n_q - 1) per running request; ``h`` is any callable on integers.  With
    h = w_p*n_p + w_q*n_q this is Algorithm 2 again.
  * ``predictor`` (Section 4.4 / Algorithm 3): admission also charges w_q * predicted_output_len(r);
    after a decode step a request is charged w_q only once its output exceeds the prediction, and
    when it finishes short of the prediction the unused part w_q * (output - predicted) is refunded.
    ``predictor(client, request)`` returns the predicted length; ``LastFivePredictor`` is the paper's
    "average output length of the last five requests of the client" (integer floor, 0 without history).

TEST INFRASTRUCTURE ONLY.
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field
from typing import Callable, Deque, List, Optional, Sequence


@dataclass
class Running:
    rid: int
    client: int
    n_input: int
    n_output: int      # hidden: only compared with ``generated`` to detect the end
    generated: int = 0
    predicted: int = 0  # predicted output length (Algorithm 3); unused otherwise


class LastFivePredictor:
    """Mean output length of the client's last five finished requests (Section 5.1, "VTC (predict)")."""

    def __init__(self, num_clients: int) -> None:
        self.history = [deque(maxlen=5) for _ in range(num_clients)]

    def __call__(self, client: int, request) -> int:
        h = self.history[client]
        return sum(h) // len(h) if h else 0

    def observe(self, client: int, n_output: int) -> None:
        self.history[client].append(int(n_output))


@dataclass
class StepRecord:
    iteration: int
    time_s: float
    admitted: List[Running]                 # the minibatch of this iteration (generated == 0 at admission)
    decode_rids: List[int]
    decode_clients: List[int]
    decode_n_input: List[int]
    decode_generated_before: List[int]      # tokens generated before this decode step
    counters_before_decode_charge: List[int]
    counters_after_decode_charge: List[int]
    finished: List[Running]


Observer = Callable[[str, "VTCScheduler"], None]


class VTCScheduler:
    def __init__(
        self,
        num_clients: int,
        w_p: int,
        w_q: int,
        M: int,
        L_output: int,
        max_batch: Optional[int] = None,
        lift: bool = True,
        observer: Optional[Observer] = None,
        cost: Optional[Callable[[int, int], int]] = None,
        predictor: Optional[Callable] = None,
    ) -> None:
        self.num_clients = num_clients
        self.w_p, self.w_q = int(w_p), int(w_q)
        self.M, self.L_output = int(M), int(L_output)
        self.max_batch = max_batch
        self.lift = lift
        self.observer = observer
        self.cost = cost
        self.predictor = predictor
        if cost is not None and predictor is not None:
            raise ValueError("the paper defines length prediction for the weighted-token cost only")
        self.c: List[int] = [0] * num_clients                      # virtual token counters
        self.Q: List[Deque] = [deque() for _ in range(num_clients)]  # waiting queue, per client
        self.B: List[Running] = []                                  # running batch
        self.last_left: Optional[int] = None
        self.reserved = 0                                           # tokens of M promised to B
        self.service: List[int] = [0] * num_clients                 # W_i(0, now)
        self.iteration = 0

    # ------------------------------------------------------------ helpers
    def waiting_clients(self) -> List[int]:
        return [i for i in range(self.num_clients) if self.Q[i]]

    def _notify(self, event: str) -> None:
        if self.observer is not None:
            self.observer(event, self)

    def _fits(self, req, minibatch: List[Running], minibatch_reserved: int) -> bool:
        if self.max_batch is not None and len(self.B) + len(minibatch) >= self.max_batch:
            return False
        return self.reserved + minibatch_reserved + req.n_input + self.L_output <= self.M

    # ---------------------------------------------------- monitoring stream
    def _lifted_counter(self, client: int) -> int:
        """Counter a client gets when a request of it arrives while none of its requests is waiting: not below
        the smallest counter among the clients that are waiting, or -- nobody waiting at all -- not below the
        counter of the client whose queue emptied last (Algorithm 2, monitoring stream)."""
        waiting = self.waiting_clients()
        if waiting:
            floor = min(self.c[i] for i in waiting)
        elif self.last_left is not None:
            floor = self.c[self.last_left]
        else:
            return self.c[client]                       # nobody has ever left the queue: nothing to catch up with
        return max(self.c[client], floor)

    def on_arrival(self, req) -> None:
        if self.lift and not self.Q[req.client]:
            self.c[req.client] = self._lifted_counter(req.client)
        self.Q[req.client].append(req)
        self._notify("arrival")

    # ----------------------------------------------------- execution stream
    def _admission_charge(self, run: Running, req) -> None:
        """What a client pays when its request enters the minibatch (Algorithm 2; Section 4.2; Algorithm 3)."""
        client = req.client
        if self.cost is not None:
            self.c[client] += self.cost(req.n_input, 0)
            self.service[client] += self.cost(req.n_input, 0)
            return
        self.c[client] += self.w_p * req.n_input
        self.service[client] += self.w_p * req.n_input
        if self.predictor is not None:
            run.predicted = int(self.predictor(client, req))
            self.c[client] += self.w_q * run.predicted      # pre-payment; not service received yet

    def select_new_requests(self) -> List[Running]:
        admitted: List[Running] = []
        admitted_reserved = 0
        # keep taking the oldest request of the waiting client with the smallest counter until it does not fit
        while self.waiting_clients():
            lowest = min(self.waiting_clients(), key=lambda i: (self.c[i], i))
            head = self.Q[lowest][0]
            if not self._fits(head, admitted, admitted_reserved):
                break
            run = Running(head.rid, head.client, head.n_input, head.n_output)
            self._admission_charge(run, head)
            admitted.append(run)
            admitted_reserved += head.n_input + self.L_output
            self.Q[lowest].popleft()
            if not self.Q[lowest]:
                self.last_left = lowest
            self._notify("admit")
        self.reserved += admitted_reserved
        if not self.B and not admitted and self.waiting_clients():
            raise ValueError("the head request can never fit: input_length + L_output exceeds M")
        return admitted

    def step(self, time_s: float = 0.0, admit: bool = True) -> StepRecord:
        admitted = self.select_new_requests() if admit else []
        # a real server prefills the admitted requests here
        self.B.extend(admitted)
        # forward_decode(B): every running request produces one token
        before = list(self.c)
        rec = StepRecord(
            iteration=self.iteration,
            time_s=time_s,
            admitted=admitted,
            decode_rids=[x.rid for x in self.B],
            decode_clients=[x.client for x in self.B],
            decode_n_input=[x.n_input for x in self.B],
            decode_generated_before=[x.generated for x in self.B],
            counters_before_decode_charge=before,
            counters_after_decode_charge=[],
            finished=[],
        )
        for x in self.B:
            x.generated += 1
        if self.cost is not None:
            for x in self.B:
                d = self.cost(x.n_input, x.generated) - self.cost(x.n_input, x.generated - 1)
                self.c[x.client] += d
                self.service[x.client] += d
        elif self.predictor is not None:
            for x in self.B:
                self.service[x.client] += self.w_q
                delta = x.generated - x.predicted
                if delta > 0:
                    self.c[x.client] += self.w_q
                if x.generated >= x.n_output and delta < 0:
                    self.c[x.client] += self.w_q * delta
        else:
            for i in range(self.num_clients):
                n_i = sum(1 for x in self.B if x.client == i)
                self.c[i] += self.w_q * n_i
                self.service[i] += self.w_q * n_i
        rec.counters_after_decode_charge = list(self.c)
        self._notify("decode")
        # filter_finished_requests(B)
        rec.finished = [x for x in self.B if x.generated >= x.n_output]
        self.B = [x for x in self.B if x.generated < x.n_output]
        for x in rec.finished:
            self.reserved -= x.n_input + self.L_output
            if self.predictor is not None and hasattr(self.predictor, "observe"):
                self.predictor.observe(x.client, x.generated)
        self.iteration += 1
        return rec

    def idle(self) -> bool:
        return not self.B and not self.waiting_clients()


def simulate(
    trace: Sequence,
    sched: VTCScheduler,
    t_decode_s: float,
    t_prefill_token_s: float,
    admit_every: int = 1,
    max_iterations: Optional[int] = None,
    on_step: Optional[Callable[[StepRecord], bool]] = None,
) -> List[StepRecord]:
    """Run the two streams over an arrival trace on a virtual clock.

    Arrivals whose time has come are handed to the monitoring stream before
    each execution-stream iteration.  ``on_step`` may return True to stop.
    Returns the step records (all of them, so keep traces modest).
    """
    records: List[StepRecord] = []
    t = 0.0
    nxt = 0
    n = len(trace)
    while nxt < n or not sched.idle():
        while nxt < n and trace[nxt].arrival <= t:
            sched.on_arrival(trace[nxt])
            nxt += 1
        if sched.idle():
            t = trace[nxt].arrival                      # server idle: wait for the next request
            continue
        rec = sched.step(time_s=t, admit=(sched.iteration % admit_every == 0))
        t += t_decode_s + t_prefill_token_s * sum(x.n_input for x in rec.admitted)
        records.append(rec)
        if on_step is not None and on_step(rec):
            break
        if max_iterations is not None and len(records) >= max_iterations:
            break
    return records
