"""The paper's baseline schedulers in the CPU simulator: FCFS, RPM, LCF versus VTC (CPU only).

These reproduce, qualitatively and on the paper's synthetic workload shapes (Section 5.2), what the
evaluation shows: FCFS serves clients in proportion to what they send, VTC equalises backlogged
clients and keeps an under-share client unaffected, RPM is not work-conserving.
"""
import pytest

from oracle.baselines import (FCFSScheduler, max_pairwise_difference, service_difference,
                              simulate_baseline)
from oracle.scheduler import VTCScheduler, simulate
from workloads.traces import Request, fixed_lengths, uniform_trace

T_DEC, T_PF = 0.045, 2e-4


def _overloaded_pair():
    # Section 5.2: 90 and 180 requests per minute, 256 in / 256 out, both beyond capacity
    return uniform_trace([90, 180], 300.0, [fixed_lengths(256, 256)] * 2)


def test_fcfs_is_arrival_order_and_unfair_under_overload():
    trace = _overloaded_pair()
    f = FCFSScheduler(2, 1, 2, 10000, 256)
    order = []
    simulate_baseline(trace, f, T_DEC, T_PF, on_step=lambda rec: order.extend(x.rid for x in rec.admitted) and False)
    assert order == sorted(order)                                   # request ids are assigned in arrival order
    # while both clients are backlogged FCFS serves them 1 : 2, like their request rates
    f2 = FCFSScheduler(2, 1, 2, 10000, 256)
    snap = {}

    def at(rec):
        if rec.time_s >= 200 and "s" not in snap:
            snap["s"] = list(f2.service)
        return False

    simulate_baseline(trace, f2, T_DEC, T_PF, on_step=at)
    assert 1.8 < snap["s"][1] / snap["s"][0] < 2.2


def test_vtc_equalises_where_fcfs_does_not():
    trace = _overloaded_pair()
    v = VTCScheduler(2, 1, 2, 10000, 256)
    snap = {}

    def at(rec):
        if rec.time_s >= 200 and "s" not in snap:
            snap["s"] = list(v.service)
        return False

    simulate(trace, v, T_DEC, T_PF, on_step=at)
    s = snap["s"]
    assert max_pairwise_difference(s) <= 2 * max(256, 2 * 10000)     # the fairness theorem's bound
    assert abs(s[0] - s[1]) < 0.05 * max(s)                          # and in practice nearly equal
    f = FCFSScheduler(2, 1, 2, 10000, 256)
    snapf = {}
    simulate_baseline(trace, f, T_DEC, T_PF,
                      on_step=lambda rec: snapf.setdefault("s", list(f.service)) and False if rec.time_s >= 200 else False)
    assert max_pairwise_difference(snapf["s"]) > 10 * max_pairwise_difference(s)


def test_rpm_limit_blocks_until_the_next_minute_and_wastes_capacity():
    # one client, 120 requests per minute of 64/64 tokens: far below capacity, but RPM(30) admits 30 per minute
    trace = uniform_trace([120], 120.0, [fixed_lengths(64, 64)])
    free = FCFSScheduler(1, 1, 2, 10000, 64)
    simulate_baseline(trace, free, T_DEC, T_PF)
    limited = FCFSScheduler(1, 1, 2, 10000, 64, rpm_limit=30)
    first_minute = []
    recs = simulate_baseline(trace, limited, T_DEC, T_PF,
                             on_step=lambda rec: first_minute.extend(x.rid for x in rec.admitted if rec.time_s < 60.0) and False)
    assert len(first_minute) == 30                                   # the rest waits for the window to roll
    assert limited.service == free.service                           # everything is served in the end ...
    assert recs[-1].time_s > 7 * 60                                  # ... 240 requests at 30 per minute take 8 windows
    # no window ever admits more than the limit
    per_window = {}
    limited2 = FCFSScheduler(1, 1, 2, 10000, 64, rpm_limit=30)
    simulate_baseline(trace, limited2, T_DEC, T_PF,
                      on_step=lambda rec: [per_window.__setitem__(int(rec.time_s // 60), per_window.get(int(rec.time_s // 60), 0) + len(rec.admitted))] and False)
    assert max(per_window.values()) <= 30


def test_isolation_of_an_under_share_client():
    # Section 5.2, isolation: client 0 sends 30 requests/min (under its share), client 1 floods.  Under VTC client 0's
    # requests are admitted almost at once; under FCFS they queue behind the flood.
    trace = uniform_trace([30, 240], 240.0, [fixed_lengths(256, 256)] * 2)
    arrival = {r.rid: r.arrival for r in trace}

    def waits(run, sched_factory):
        sched = sched_factory()
        w = []

        def on_step(rec):
            w.extend(rec.time_s - arrival[x.rid] for x in rec.admitted if x.client == 0 and arrival[x.rid] > 60)
            return False

        run(trace, sched, T_DEC, T_PF, on_step=on_step)
        return sum(w) / len(w)

    vtc_wait = waits(simulate, lambda: VTCScheduler(2, 1, 2, 10000, 256))
    fcfs_wait = waits(simulate_baseline, lambda: FCFSScheduler(2, 1, 2, 10000, 256))
    assert vtc_wait < 15.0 and fcfs_wait > 5 * vtc_wait


def test_service_difference_metric():
    # s1 <= s2: min(s2 - s1, |r1 - s1|)
    assert service_difference(100, 300, 100, 1000) == 0          # the low client got all it asked for
    assert service_difference(100, 300, 500, 1000) == 200
    assert service_difference(100, 300, 150, 1000) == 50
    assert service_difference(300, 100, 1000, 150) == 50         # symmetric in the arguments
