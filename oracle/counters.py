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
