"""Virtual-token-counter charge and paged-cache slot index -- the definitions.

Counter charge.  Algorithm 2 of the paper adds ``w_p * input_length(r)`` to
client k's counter when request r is admitted, and after every decode step
adds ``w_q * |{r in B : client(r) = i}|`` to every client i.  The general
framework (Algorithm 4) states the same thing as "when new tokens have been
processed, c_i += sum over the client's requests of the increase of h", and
with the weighted-token cost of Section 3.1, h = w_p*n_p + w_q*n_q, that
increase is ``w_p * (new input tokens) + w_q * (new output tokens)``.
``counter_update`` is that sentence as a sequential loop in Python integers
(arbitrary precision, so no overflow can hide), checked to fit int64.

Slot index.  Token p of sequence r lives in physical block
``block_table[r][p // Bs]`` at row ``p % Bs`` (the paper only names a paged
cache, Section 5.1; the index formula is the usual one).

TEST INFRASTRUCTURE ONLY.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

INT64_MIN = -(1 << 63)
INT64_MAX = (1 << 63) - 1


def counter_update(
    counters: Sequence[int],
    client_ids: Sequence[int],
    n_input_tokens: Optional[Sequence[int]],
    n_output_tokens: Optional[Sequence[int]],
    w_p: int,
    w_q: int,
) -> List[int]:
    """Return the counters after charging every request of one step.

    ``None`` for either token array means "all zero".  Requests whose client id
    is outside [0, len(counters)) are ignored.
    """
    c = [int(x) for x in counters]
    for r, client in enumerate(client_ids):
        client = int(client)
        if client < 0 or client >= len(c):
            continue
        n_p = int(n_input_tokens[r]) if n_input_tokens is not None else 0
        n_q = int(n_output_tokens[r]) if n_output_tokens is not None else 0
        c[client] += int(w_p) * n_p + int(w_q) * n_q
    for x in c:
        if not INT64_MIN <= x <= INT64_MAX:
            raise OverflowError("counter does not fit int64")
    return c


def gather_slots(block_table, seq_lens: Sequence[int], block_size: int) -> List[int]:
    """slot(r, p) for every valid (r, p), sequences concatenated in order."""
    slots: List[int] = []
    for r, s in enumerate(seq_lens):
        for p in range(int(s)):
            slots.append(int(block_table[r][p // block_size]) * block_size + p % block_size)
    return slots


# ---------------------------------------------------------------------------
# General cost function (Section 4.2 and Algorithm 4 of the paper)
# ---------------------------------------------------------------------------
class CostPoly:
    """h(n_p, n_q) = c0 + cp*n_p + cq*n_q + cpp*n_p^2 + cpq*n_p*n_q + cqq*n_q^2 with integer coefficients.

    Integer (fixed-point) coefficients keep the counters exact.  The paper's profiled cost of Appendix B.2,
    h = 2.1 n_p + n_q + 0.04 n_p n_q + 0.032 n_q^2 + 11.46, is ``PROFILED_MILLI`` in units of 1/1000.
    The weighted-token cost of Section 3.1 is ``CostPoly(0, w_p, w_q, 0, 0, 0)``.
    """

    def __init__(self, c0: int, cp: int, cq: int, cpp: int, cpq: int, cqq: int) -> None:
        self.c0, self.cp, self.cq, self.cpp, self.cpq, self.cqq = (int(x) for x in (c0, cp, cq, cpp, cpq, cqq))

    def __call__(self, n_p: int, n_q: int) -> int:
        n_p, n_q = int(n_p), int(n_q)
        return (self.c0 + self.cp * n_p + self.cq * n_q + self.cpp * n_p * n_p + self.cpq * n_p * n_q
                + self.cqq * n_q * n_q)

    def coefficients(self):
        return (self.c0, self.cp, self.cq, self.cpp, self.cpq, self.cqq)


PROFILED_MILLI = CostPoly(11460, 2100, 1000, 0, 40, 32)


def counter_update_cost(
    counters: Sequence[int],
    client_ids: Sequence[int],
    n_p_old: Sequence[int],
    n_q_old: Sequence[int],
    n_p_new: Sequence[int],
    n_q_new: Sequence[int],
    h,
    client_multiplier: Optional[Sequence[int]] = None,
) -> List[int]:
    """Algorithm 4: "when new tokens have been processed", c_i += sum_r h(new_r) - h(old_r).

    A request none of whose tokens has been processed yet (old counts both 0) has cost 0, so its first
    update charges h(n_p, 0) in full -- what Section 4.2 states for the admission line of Algorithm 2.
    ``client_multiplier[i]`` (weighted VTC, Section 4.3) scales client i's increment: dividing by the
    client's weight w_i is expressed exactly as multiplying by W / w_i for a common multiple W.
    """
    c = [int(x) for x in counters]
    for r, client in enumerate(client_ids):
        client = int(client)
        if client < 0 or client >= len(c):
            continue
        po, qo, pn, qn = int(n_p_old[r]), int(n_q_old[r]), int(n_p_new[r]), int(n_q_new[r])
        old_cost = 0 if (po == 0 and qo == 0) else h(po, qo)
        delta = h(pn, qn) - old_cost
        if client_multiplier is not None:
            delta *= int(client_multiplier[client])
        c[client] += delta
    for x in c:
        if not INT64_MIN <= x <= INT64_MAX:
            raise OverflowError("counter does not fit int64")
    return c


# ---------------------------------------------------------------------------
# VTC with length prediction (Algorithm 3 of the paper), the per-step adjustment
# ---------------------------------------------------------------------------
def counter_update_predicted(
    counters: Sequence[int],
    client_ids: Sequence[int],
    n_output: Sequence[int],
    n_predicted: Sequence[int],
    finished: Sequence[int],
    w_q: int,
) -> List[int]:
    """After a decode step, for each running request r (Algorithm 3, "adjust the cost of output tokens"):

        delta = output_len(r) - predicted_output_len(r)        (output_len counts the token just made)
        if delta > 0:                 c[client(r)] += w_q       (the prediction is used up: pay as you go)
        if r finished and delta < 0:  c[client(r)] += w_q * delta   (refund what was pre-paid and not used)

    The pre-payment itself, w_p*input_len + w_q*predicted_len at admission, is an ordinary counter charge.
    """
    c = [int(x) for x in counters]
    for r, client in enumerate(client_ids):
        client = int(client)
        if client < 0 or client >= len(c):
            continue
        delta = int(n_output[r]) - int(n_predicted[r])
        if delta > 0:
            c[client] += int(w_q)
        if int(finished[r]) != 0 and delta < 0:
            c[client] += int(w_q) * delta
    for x in c:
        if not INT64_MIN <= x <= INT64_MAX:
            raise OverflowError("counter does not fit int64")
    return c
