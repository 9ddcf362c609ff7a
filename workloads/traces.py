"""Seeded request arrival traces.

A request is the paper's three-tuple (arrival time a, input tokens x, client u)
of Section 2.1; only the *length* of x matters here.  The output length is
carried along but is hidden from any scheduler until the request finishes.

The shapes follow the paper's synthetic workloads (Section 5.2: evenly spaced
and Poisson arrivals, fixed or per-client lengths) and, for the 27-client case,
stand in for the real trace of Section 5.3, which is not available: log-normal
lengths and per-client Poisson rates spread log-uniformly over a factor of ten.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class Request:
    rid: int          # unique id, also the tie-break for equal arrival times
    client: int       # u
    arrival: float    # a, seconds on the virtual clock
    n_input: int      # len(x)
    n_output: int     # number of tokens the request will generate (hidden)


LengthSampler = Callable[[np.random.Generator], Tuple[int, int]]


def _finalise(rows: List[Tuple[float, int, int, int]]) -> List[Request]:
    """Sort by arrival time (stable in generation order) and assign ids."""
    order = sorted(range(len(rows)), key=lambda i: (rows[i][0], i))
    return [
        Request(rid=n, client=rows[i][1], arrival=rows[i][0], n_input=rows[i][2], n_output=rows[i][3])
        for n, i in enumerate(order)
    ]


def fixed_lengths(n_input: int, n_output: int) -> LengthSampler:
    return lambda rng: (n_input, n_output)


def uniform_lengths(in_lo: int, in_hi: int, out_lo: int, out_hi: int) -> LengthSampler:
    """Inclusive integer ranges."""
    def sample(rng: np.random.Generator) -> Tuple[int, int]:
        return int(rng.integers(in_lo, in_hi + 1)), int(rng.integers(out_lo, out_hi + 1))
    return sample


def lognormal_lengths(median_in: float, median_out: float, sigma: float, lo: int, hi: int) -> LengthSampler:
    def sample(rng: np.random.Generator) -> Tuple[int, int]:
        a = int(round(float(rng.lognormal(np.log(median_in), sigma))))
        b = int(round(float(rng.lognormal(np.log(median_out), sigma))))
        return min(max(a, lo), hi), min(max(b, lo), hi)
    return sample


def uniform_trace(
    rates_per_min: Sequence[float],
    duration_s: float,
    lengths: Sequence[LengthSampler],
    seed: int = 0,
    on_off_period_s: Sequence[float] | None = None,
) -> List[Request]:
    """Evenly spaced arrivals (Section 5.2, constant request rates).

    ``on_off_period_s[c] = p > 0`` makes client c alternate between sending for
    p seconds and being silent for p seconds (the ON/OFF pattern).
    """
    rng = np.random.default_rng(seed)
    rows: List[Tuple[float, int, int, int]] = []
    for c, rate in enumerate(rates_per_min):
        if rate <= 0:
            continue
        gap = 60.0 / rate
        k = 0
        while True:
            t = k * gap
            if t >= duration_s:
                break
            k += 1
            if on_off_period_s is not None and on_off_period_s[c] > 0:
                if int(t // on_off_period_s[c]) % 2 == 1:
                    continue
            n_in, n_out = lengths[c](rng)
            rows.append((t, c, n_in, n_out))
    return _finalise(rows)


def poisson_trace(
    rates_per_s: Sequence[float],
    duration_s: float,
    lengths: Sequence[LengthSampler],
    seed: int = 0,
) -> List[Request]:
    """Independent Poisson arrivals per client (exponential gaps, CV = 1)."""
    rng = np.random.default_rng(seed)
    rows: List[Tuple[float, int, int, int]] = []
    for c, rate in enumerate(rates_per_s):
        if rate <= 0:
            continue
        t = 0.0
        while True:
            t += float(rng.exponential(1.0 / rate))
            if t >= duration_s:
                break
            n_in, n_out = lengths[c](rng)
            rows.append((t, c, n_in, n_out))
    return _finalise(rows)


# ----------------------------------------------------------------------------
# The two scheduler-driven configurations.  Everything below is a harness
# constant, not something the paper fixes.
# ----------------------------------------------------------------------------

SEED_BASE = 0x5EED0000


def trace_for_config(config_id: int, duration_s: float | None = None) -> Tuple[List[Request], dict]:
    """Arrival trace plus simulator parameters for configs 3 and 4.

    Returns (trace, params) where params holds the number of clients, the
    memory pool M in tokens, the output-length cap, the batch cap and the
    virtual-clock constants used to turn the trace into a running batch.
    """
    seed = SEED_BASE + config_id
    if config_id == 3:
        # 4 overloaded clients, Poisson, rates 8:4:2:1; short-prompt clients 0,1
        # and long-prompt clients 2,3; hidden output length uniform in [64,512].
        base = 4.0
        rates = [8 * base, 4 * base, 2 * base, 1 * base]
        lengths = [
            uniform_lengths(64, 1024, 64, 512),
            uniform_lengths(64, 1024, 64, 512),
            uniform_lengths(512, 2048, 64, 512),
            uniform_lengths(512, 2048, 64, 512),
        ]
        params = dict(num_clients=4, M=1 << 20, L_input=2048, L_output=512, max_batch=256,
                      t_decode_s=0.030, t_prefill_token_s=1.0e-4, w_p=1, w_q=2)
        dur = 40.0 if duration_s is None else duration_s
        return poisson_trace(rates, dur, lengths, seed), params
    if config_id == 4:
        # 27 clients, rates log-uniform over one decade, log-normal lengths.
        rng = np.random.default_rng(seed ^ 0xC11E)
        u = rng.uniform(0.0, 1.0, size=27)
        lam_min = 1.4
        rates = [lam_min * 10.0 ** float(x) for x in u]
        lengths = [lognormal_lengths(200.0, 150.0, 1.0, 2, 4096)] * 27
        params = dict(num_clients=27, M=8 << 20, L_input=4096, L_output=4096, max_batch=512,
                      t_decode_s=0.030, t_prefill_token_s=1.0e-4, w_p=1, w_q=2)
        dur = 40.0 if duration_s is None else duration_s
        return poisson_trace(rates, dur, lengths, seed), params
    raise ValueError(f"config {config_id} is not scheduler-driven")
