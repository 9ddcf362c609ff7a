"""Pins for the oracle's general-cost, weighted and length-prediction counter updates (CPU only)."""
import os
from collections import defaultdict
from fractions import Fraction

import numpy as np
import pytest

from oracle.counters import (PROFILED_MILLI, CostPoly, counter_update, counter_update_cost,
                             counter_update_predicted)
from oracle.scheduler import LastFivePredictor, VTCScheduler, simulate
from workloads.traces import Request, fixed_lengths, poisson_trace, uniform_lengths, uniform_trace

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "profiled_cost_values.txt")


# ------------------------------------------------------------ cost function
def test_profiled_cost_matches_the_formula_printed_in_the_paper():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 5
    for n_p, n_q, h in rows:
        assert Fraction(PROFILED_MILLI(int(n_p), int(n_q)), 1000) == Fraction(h)
    # monotone in both arguments, as Section 3.1 requires of a cost function
    for n_p in (0, 7, 300):
        for n_q in (0, 5, 400):
            assert PROFILED_MILLI(n_p + 1, n_q) > PROFILED_MILLI(n_p, n_q)
            assert PROFILED_MILLI(n_p, n_q + 1) > PROFILED_MILLI(n_p, n_q)


def test_linear_cost_reduces_to_the_weighted_token_charge():
    rng = np.random.default_rng(0)
    n, clients = 300, 9
    ids = rng.integers(-1, clients + 1, size=n)
    po, qo = rng.integers(0, 500, size=n), rng.integers(0, 200, size=n)
    dp, dq = rng.integers(0, 300, size=n), rng.integers(0, 2, size=n)
    base = rng.integers(0, 10 ** 6, size=clients).tolist()
    h = CostPoly(0, 3, 5, 0, 0, 0)
    got = counter_update_cost(base, ids, po, qo, po + dp, qo + dq, h)
    assert got == counter_update(base, ids, dp, dq, 3, 5)


def test_cost_updates_telescope_to_h_of_the_finished_request():
    # Section 4.2: admission charges h(n_p, 0), each decode step h(n_p, n_q) - h(n_p, n_q - 1).
    rng = np.random.default_rng(1)
    for _ in range(10):
        n_p, n_q = int(rng.integers(1, 1500)), int(rng.integers(1, 300))
        c = counter_update_cost([0], [0], [0], [0], [n_p], [0], PROFILED_MILLI)
        assert c == [PROFILED_MILLI(n_p, 0)]                     # includes the constant term, once
        for q in range(1, n_q + 1):
            c = counter_update_cost(c, [0], [n_p], [q - 1], [n_p], [q], PROFILED_MILLI)
        assert c == [PROFILED_MILLI(n_p, n_q)]
    # chunked prefill: per-processed-token accounting ends at the same total
    c = counter_update_cost([0], [0], [0], [0], [256], [0], PROFILED_MILLI)
    c = counter_update_cost(c, [0], [256], [0], [512], [0], PROFILED_MILLI)
    assert c == [PROFILED_MILLI(512, 0)]


def test_weighted_vtc_multipliers():
    # Section 4.3: the increment of client i is divided by its weight w_i; with weights 1:2:3:4 and W = 12
    # that is a multiplication by 12, 6, 4, 3.
    ids = [0, 1, 2, 3, 3]
    h = CostPoly(0, 1, 2, 0, 0, 0)
    got = counter_update_cost([0, 0, 0, 0], ids, [0] * 5, [0] * 5, [10] * 5, [0] * 5, h, client_multiplier=[12, 6, 4, 3])
    assert got == [120, 60, 40, 60]
    assert [Fraction(x, 12) for x in got] == [Fraction(10, 1), Fraction(10, 2), Fraction(10, 3), Fraction(20, 4)]


# --------------------------------------------------------- length prediction
def test_prediction_adjustment_hand_cases():
    # w_q = 2.  r0: predicted 5, now at 3 tokens, running        -> nothing
    #           r1: predicted 5, now at 6 tokens                  -> +2 (pay as you go past the prediction)
    #           r2: predicted 5, finished at 3                    -> 2 * (3 - 5) = -4 refund
    #           r3: predicted 5, finished at 5                    -> nothing
    #           r4: predicted 5, finished at 7                    -> +2 only (delta > 0), no refund
    got = counter_update_predicted([100, 100], [0, 0, 1, 1, 1], [3, 6, 3, 5, 7], [5, 5, 5, 5, 5], [0, 0, 1, 1, 1], 2)
    assert got == [102, 100 - 4 + 2]


@pytest.mark.parametrize("pred", [0, 3, 10, 11, 40])
def test_prediction_charges_telescope_to_the_true_cost(pred):
    # whatever the prediction, a finished request has paid exactly w_p*n_p + w_q*n_q  (Algorithm 3)
    w_p, w_q, n_p, n_q = 1, 2, 17, 10
    c = counter_update([0], [0], [n_p], [pred], w_p, w_q)                       # admission: prompt + prediction
    for out in range(1, n_q + 1):
        c = counter_update_predicted(c, [0], [out], [pred], [1 if out == n_q else 0], w_q)
    assert c == [w_p * n_p + w_q * n_q]


def _finish_all(trace, **kw):
    sched = VTCScheduler(kw.pop("clients"), 1, 2, kw.pop("M"), kw.pop("L_out"), lift=kw.pop("lift", True), **kw)
    log = []
    simulate(trace, sched, 0.045, 2e-4, on_step=lambda rec: log.append(list(sched.service)) and False)
    return sched, log


def test_scheduler_with_linear_cost_function_is_algorithm_2():
    trace = poisson_trace([5.0, 2.0, 1.0], 40.0, [uniform_lengths(8, 300, 1, 150)] * 3, seed=4)
    a = VTCScheduler(3, 1, 2, 6000, 150)
    b = VTCScheduler(3, 1, 2, 6000, 150, cost=CostPoly(0, 1, 2, 0, 0, 0))
    ra = simulate(trace, a, 0.03, 1e-4)
    rb = simulate(trace, b, 0.03, 1e-4)
    assert len(ra) == len(rb)
    for x, y in zip(ra, rb):
        assert x.decode_rids == y.decode_rids and x.counters_after_decode_charge == y.counters_after_decode_charge


def test_scheduler_with_profiled_cost_charges_h_per_finished_request():
    trace = poisson_trace([4.0, 1.0], 30.0, [fixed_lengths(64, 64), fixed_lengths(256, 256)], seed=5)
    sched = VTCScheduler(2, 1, 2, 10000, 256, lift=False, cost=PROFILED_MILLI)
    simulate(trace, sched, 0.045, 2e-4)
    want = defaultdict(int)
    for r in trace:
        want[r.client] += PROFILED_MILLI(r.n_input, r.n_output)
    assert sched.c == [want[0], want[1]] == sched.service


@pytest.mark.parametrize("kind", ["oracle", "zero", "half", "double", "last5"])
def test_scheduler_with_length_prediction_ends_at_the_true_cost(kind):
    trace = poisson_trace([3.0, 2.0], 40.0, [uniform_lengths(16, 300, 1, 200)] * 2, seed=6)
    predictor = {"oracle": lambda c, r: r.n_output, "zero": lambda c, r: 0, "half": lambda c, r: r.n_output // 2,
                 "double": lambda c, r: 2 * r.n_output, "last5": LastFivePredictor(2)}[kind]
    sched = VTCScheduler(2, 1, 2, 8000, 200, lift=False, predictor=predictor)
    simulate(trace, sched, 0.045, 2e-4)
    want = defaultdict(int)
    for r in trace:
        want[r.client] += r.n_input + 2 * r.n_output
    assert sched.c == [want[0], want[1]]          # every pre-payment was either used up or refunded
    assert sched.service == [want[0], want[1]]


def test_last_five_predictor():
    p = LastFivePredictor(2)
    assert p(0, None) == 0
    for n in (10, 20, 30, 40, 50, 60):
        p.observe(0, n)
    assert p(0, None) == (20 + 30 + 40 + 50 + 60) // 5 and p(1, None) == 0


def test_exact_length_prediction_bounds_the_counter_spread_by_one_request():
    # Section 4.4: with a perfect predictor the whole cost of a request is on the counter when it is admitted
    # and nothing is added or refunded later, so the counters of waiting clients never drift further apart than
    # the cost of one request, w_p*L_input + w_q*L_output -- far below the bound w_q*M of plain VTC, which learns
    # the output cost token by token and over-admits the client with the smallest counter.
    trace = uniform_trace([90, 180], 240.0, [fixed_lengths(256, 256)] * 2)

    def max_spread(**kw):
        worst = 0

        def observer(event, s):
            nonlocal worst
            P = s.waiting_clients()
            if len(P) == 2:
                worst = max(worst, abs(s.c[0] - s.c[1]))

        sched = VTCScheduler(2, 1, 2, 10000, 256, observer=observer, **kw)
        simulate(trace, sched, 0.045, 2e-4)
        return worst

    one_request = 1 * 256 + 2 * 256
    exact = max_spread(predictor=lambda c, r: r.n_output)
    plain = max_spread()
    assert 0 < exact <= one_request
    assert plain > 2 * one_request
