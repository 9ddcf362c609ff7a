"""Planted mistakes for the CPU oracle (test infrastructure of the test infrastructure).

Each mutant replaces one function of ``oracle`` by a copy with one plausible slip -- a dropped term, a
wrong sign or index, a transposed operand.  ``tests/test_oracle_mutations.py`` runs the pin tests with a
mutant switched on (in a child process, through the environment variable read by ``tests/conftest.py``)
and demands that at least one pin fails: a pin set that lets a mutant through does not pin the oracle.
Nothing here runs on a GPU and nothing here is used unless the variable is set.
"""
from __future__ import annotations

import numpy as np

ENV = "VTC_ORACLE_MUTANT"


def _attention():
    from oracle import attention as A
    return A


def _counters():
    from oracle import counters as C
    return C


# ---------------------------------------------------------------- attention
def m_scale_dropped():
    A = _attention()
    def softmax_weights(q, keys, scale):
        s = keys @ q                                   # slip: logits not scaled
        w = np.exp(s - s.max())
        return w / w.sum()
    A.softmax_weights = softmax_weights


def m_scale_in_float64():
    A = _attention()
    def softmax_weights(q, keys, scale):
        s = np.float64(scale) * (keys @ q)             # slip: scale not taken as the float32 that was passed
        w = np.exp(s - s.max())
        return w / w.sum()
    A.softmax_weights = softmax_weights


def m_not_normalised():
    A = _attention()
    def softmax_weights(q, keys, scale):
        s = np.float64(np.float32(scale)) * (keys @ q)
        return np.exp(s - s.max())                     # slip: division by the sum forgotten
    A.softmax_weights = softmax_weights


def m_gqa_modulo_mapping():
    A = _attention()
    def paged_decode(q_bits, k_bits, v_bits, block_table, seq_lens, scale, dtype, rows=None):
        n, hq, d = q_bits.shape
        hkv = k_bits.shape[1]
        out = np.zeros((n, hq, d))
        for r in range(n):
            s = int(seq_lens[r])
            for h in range(hq):
                g = h % hkv                            # slip: interleaved instead of contiguous head groups
                keys = A.gather_sequence(k_bits, block_table[r], s, g, dtype)
                vals = A.gather_sequence(v_bits, block_table[r], s, g, dtype)
                out[r, h] = A.attend_one(A.widen(q_bits[r, h], dtype), keys, vals, scale)
        return out
    A.paged_decode = paged_decode


def m_cache_row_off_by_one():
    A = _attention()
    def gather_sequence(cache_bits, block_row, seq_len, kv_head, dtype):
        bs = cache_bits.shape[2]
        pos = np.arange(seq_len)
        blocks = np.asarray(block_row)[pos // bs]
        return A.widen(cache_bits[blocks, kv_head, (pos + 1) % bs, :], dtype)   # slip: row index off by one
    A.gather_sequence = gather_sequence


def m_causal_excludes_own_position():
    A = _attention()
    def paged_prefill_chunk(q_bits, cu_q_lens, k_bits, v_bits, block_table, seq_lens, scale, dtype, rows=None):
        t, hq, d = q_bits.shape
        group = hq // k_bits.shape[1]
        out = np.zeros((t, hq, d))
        for r in range(len(cu_q_lens) - 1):
            s = int(seq_lens[r]); lq = int(cu_q_lens[r + 1]) - int(cu_q_lens[r])
            for h in range(hq):
                keys = A.gather_sequence(k_bits, block_table[r], s, h // group, dtype)
                vals = A.gather_sequence(v_bits, block_table[r], s, h // group, dtype)
                for i in range(lq):
                    p = s - lq + i
                    row = int(cu_q_lens[r]) + i
                    out[row, h] = A.attend_one(A.widen(q_bits[row, h], dtype), keys[:p], vals[:p], scale)  # slip: keys 0..p-1
        return out
    A.paged_prefill_chunk = paged_prefill_chunk


def m_chunk_position_from_zero():
    A = _attention()
    def paged_prefill_chunk(q_bits, cu_q_lens, k_bits, v_bits, block_table, seq_lens, scale, dtype, rows=None):
        t, hq, d = q_bits.shape
        group = hq // k_bits.shape[1]
        out = np.zeros((t, hq, d))
        for r in range(len(cu_q_lens) - 1):
            s = int(seq_lens[r]); lq = int(cu_q_lens[r + 1]) - int(cu_q_lens[r])
            for h in range(hq):
                keys = A.gather_sequence(k_bits, block_table[r], s, h // group, dtype)
                vals = A.gather_sequence(v_bits, block_table[r], s, h // group, dtype)
                for i in range(lq):
                    row = int(cu_q_lens[r]) + i
                    out[row, h] = A.attend_one(A.widen(q_bits[row, h], dtype), keys[: i + 1], vals[: i + 1], scale)  # slip: earlier chunks invisible
        return out
    A.paged_prefill_chunk = paged_prefill_chunk


def m_values_weighted_by_keys():
    A = _attention()
    def attend_one(q, keys, values, scale):
        if keys.shape[0] == 0:
            return np.zeros(values.shape[1])
        return A.softmax_weights(q, keys, scale) @ keys          # slip: K used where V belongs
    A.attend_one = attend_one


def m_bf16_widened_as_fp16():
    A = _attention()
    orig = A.widen
    def widen(bits, dtype):
        return orig(bits, "f16")                                  # slip: storage dtype ignored
    A.widen = widen


def m_kv_append_position_before_append():
    A = _attention()
    def kv_append(k_cache, v_cache, k_new, v_new, cu_new_lens, block_table, seq_lens):
        bs = k_cache.shape[2]
        for r in range(len(cu_new_lens) - 1):
            n_r = int(cu_new_lens[r + 1]) - int(cu_new_lens[r])
            for i in range(n_r):
                p = int(seq_lens[r]) + i                          # slip: seq_lens read as the length before the append
                blk = int(block_table[r][min(p // bs, len(block_table[r]) - 1)])
                t = int(cu_new_lens[r]) + i
                k_cache[blk, :, p % bs, :] = k_new[t]
                v_cache[blk, :, p % bs, :] = v_new[t]
    A.kv_append = kv_append


# ----------------------------------------------------------------- counters
def m_weights_swapped():
    C = _counters()
    orig = C.counter_update
    def counter_update(counters, client_ids, n_in, n_out, w_p, w_q):
        return orig(counters, client_ids, n_in, n_out, w_q, w_p)  # slip: w_p and w_q exchanged
    C.counter_update = counter_update


def m_out_of_range_client_wraps():
    C = _counters()
    def counter_update(counters, client_ids, n_in, n_out, w_p, w_q):
        c = [int(x) for x in counters]
        for r, client in enumerate(client_ids):
            n_p = int(n_in[r]) if n_in is not None else 0
            n_q = int(n_out[r]) if n_out is not None else 0
            c[int(client) % len(c)] += int(w_p) * n_p + int(w_q) * n_q   # slip: bad ids wrap instead of being ignored
        return c
    C.counter_update = counter_update


def m_slot_uses_wrong_block_size():
    C = _counters()
    def gather_slots(block_table, seq_lens, block_size):
        out = []
        for r, s in enumerate(seq_lens):
            for p in range(int(s)):
                out.append(int(block_table[r][p // block_size]) * block_size + p // block_size)   # slip: p // Bs for p % Bs
        return out
    C.gather_slots = gather_slots


def m_cost_constant_dropped():
    C = _counters()
    def call(self, n_p, n_q):
        n_p, n_q = int(n_p), int(n_q)
        return (self.cp * n_p + self.cq * n_q + self.cpp * n_p * n_p + self.cpq * n_p * n_q + self.cqq * n_q * n_q)  # slip: c0
    C.CostPoly.__call__ = call


def m_cost_cross_term_squared():
    C = _counters()
    def call(self, n_p, n_q):
        n_p, n_q = int(n_p), int(n_q)
        return (self.c0 + self.cp * n_p + self.cq * n_q + self.cpp * n_p * n_p + self.cpq * n_q * n_q + self.cqq * n_q * n_q)  # slip
    C.CostPoly.__call__ = call


def m_first_update_charges_h00():
    C = _counters()
    def counter_update_cost(counters, client_ids, n_p_old, n_q_old, n_p_new, n_q_new, h, client_multiplier=None):
        c = [int(x) for x in counters]
        for r, client in enumerate(client_ids):
            client = int(client)
            if client < 0 or client >= len(c):
                continue
            delta = h(int(n_p_new[r]), int(n_q_new[r])) - h(int(n_p_old[r]), int(n_q_old[r]))   # slip: old cost of a fresh request
            if client_multiplier is not None:
                delta *= int(client_multiplier[client])
            c[client] += delta
        return c
    C.counter_update_cost = counter_update_cost


def m_refund_sign():
    C = _counters()
    def counter_update_predicted(counters, client_ids, n_output, n_predicted, finished, w_q):
        c = [int(x) for x in counters]
        for r, client in enumerate(client_ids):
            client = int(client)
            if client < 0 or client >= len(c):
                continue
            delta = int(n_output[r]) - int(n_predicted[r])
            if delta > 0:
                c[client] += int(w_q)
            if int(finished[r]) != 0 and delta < 0:
                c[client] -= int(w_q) * delta                      # slip: the refund is added instead of subtracted
        return c
    C.counter_update_predicted = counter_update_predicted


def m_pay_as_you_go_off_by_one():
    C = _counters()
    def counter_update_predicted(counters, client_ids, n_output, n_predicted, finished, w_q):
        c = [int(x) for x in counters]
        for r, client in enumerate(client_ids):
            client = int(client)
            if client < 0 or client >= len(c):
                continue
            delta = int(n_output[r]) - int(n_predicted[r])
            if delta >= 0:                                         # slip: the last pre-paid token is paid twice
                c[client] += int(w_q)
            if int(finished[r]) != 0 and delta < 0:
                c[client] += int(w_q) * delta
        return c
    C.counter_update_predicted = counter_update_predicted


# ---------------------------------------------------------------- scheduler
def m_no_counter_lift():
    from oracle import scheduler as S
    orig_init = S.VTCScheduler.__init__
    def init(self, *a, **kw):
        orig_init(self, *a, **kw)
        self.lift = False                                          # slip: the lift of Algorithm 2 never happens (= LCF)
    S.VTCScheduler.__init__ = init


def m_lift_to_max_instead_of_min():
    import builtins
    from oracle import scheduler as S
    src_min = builtins.min
    # slip: a returning client is lifted to the largest waiting counter instead of the smallest
    orig = S.VTCScheduler.on_arrival
    def on_arrival(self, req):
        S.min = builtins.max
        try:
            return orig(self, req)
        finally:
            S.min = src_min
    S.VTCScheduler.on_arrival = on_arrival


def m_ties_go_to_the_largest_id():
    import builtins
    from oracle import scheduler as S
    orig = S.VTCScheduler.select_new_requests
    def select_new_requests(self):
        # slip: among equal counters the largest client id is picked
        S.min = lambda P, key=None: builtins.min(P, key=(lambda i: (self.c[i], -i))) if key is not None else builtins.min(P)
        try:
            return orig(self)
        finally:
            S.min = builtins.min
    S.VTCScheduler.select_new_requests = select_new_requests


def m_skip_instead_of_break_when_the_head_request_does_not_fit():
    from oracle import scheduler as S
    def select_new_requests(self):
        B_new, new_reserved = [], 0
        skipped = set()
        while True:
            P = [i for i in self.waiting_clients() if i not in skipped]
            if not P:
                break
            k = min(P, key=lambda i: (self.c[i], i))
            r = self.Q[k][0]
            if not self._fits(r, B_new, new_reserved):
                skipped.add(k)                                     # slip: tries the next client instead of stopping
                continue
            run = S.Running(r.rid, r.client, r.n_input, r.n_output)
            self.c[k] += self.w_p * r.n_input
            self.service[k] += self.w_p * r.n_input
            B_new.append(run)
            new_reserved += r.n_input + self.L_output
            self.Q[k].popleft()
            if not self.Q[k]:
                self.last_left = k
            self._notify("admit")
        self.reserved += new_reserved
        return B_new
    S.VTCScheduler.select_new_requests = select_new_requests


def m_finishing_step_is_not_charged():
    from oracle import scheduler as S
    orig = S.VTCScheduler.step
    def step(self, time_s=0.0, admit=True):
        rec = orig(self, time_s, admit)
        for x in rec.finished:                                     # slip: filter before the charge
            self.c[x.client] -= self.w_q
            self.service[x.client] -= self.w_q
        return rec
    S.VTCScheduler.step = step


def m_fcfs_serves_the_newest_first():
    from oracle import baselines as B
    orig = B.FCFSScheduler.on_arrival
    def on_arrival(self, req):
        orig(self, req)
        if self.queue and self.queue[-1] is req:
            self.queue.rotate(1)                                   # slip: last come, first served
    B.FCFSScheduler.on_arrival = on_arrival


def m_rpm_limit_off_by_one():
    from oracle import baselines as B
    orig = B.FCFSScheduler.on_arrival
    def on_arrival(self, req):
        if self.rpm_limit is not None:
            self.rpm_limit += 1                                    # slip: "<=" for "<" in the per-window test
            try:
                return orig(self, req)
            finally:
                self.rpm_limit -= 1
        return orig(self, req)
    B.FCFSScheduler.on_arrival = on_arrival


def m_service_difference_ignores_the_demand():
    from oracle import baselines as B
    B.service_difference = lambda s1, s2, r1, r2: abs(s1 - s2)    # slip: the min with |r - s| is dropped


MUTANTS = {name[2:]: fn for name, fn in list(globals().items()) if name.startswith("m_") and callable(fn)}

# which pin files must catch which mutant
TARGETS = {
    "scale_dropped": "tests/test_oracle_attention.py",
    "scale_in_float64": "tests/test_oracle_attention.py",
    "not_normalised": "tests/test_oracle_attention.py",
    "gqa_modulo_mapping": "tests/test_oracle_attention.py",
    "cache_row_off_by_one": "tests/test_oracle_attention.py",
    "causal_excludes_own_position": "tests/test_oracle_attention.py",
    "chunk_position_from_zero": "tests/test_oracle_attention.py",
    "values_weighted_by_keys": "tests/test_oracle_attention.py",
    "bf16_widened_as_fp16": "tests/test_oracle_attention.py",
    "kv_append_position_before_append": "tests/test_oracle_attention.py",
    "weights_swapped": "tests/test_oracle_counters.py",
    "out_of_range_client_wraps": "tests/test_oracle_counters.py",
    "slot_uses_wrong_block_size": "tests/test_oracle_counters.py",
    "cost_constant_dropped": "tests/test_oracle_variants.py",
    "cost_cross_term_squared": "tests/test_oracle_variants.py",
    "first_update_charges_h00": "tests/test_oracle_variants.py",
    "refund_sign": "tests/test_oracle_variants.py",
    "pay_as_you_go_off_by_one": "tests/test_oracle_variants.py",
    "no_counter_lift": "tests/test_oracle_scheduler.py",
    "lift_to_max_instead_of_min": "tests/test_oracle_scheduler.py",
    "ties_go_to_the_largest_id": "tests/test_oracle_scheduler.py",
    "skip_instead_of_break_when_the_head_request_does_not_fit": "tests/test_oracle_scheduler.py",
    "finishing_step_is_not_charged": "tests/test_oracle_scheduler.py",
    "fcfs_serves_the_newest_first": "tests/test_oracle_baselines.py",
    "rpm_limit_off_by_one": "tests/test_oracle_baselines.py",
    "service_difference_ignores_the_demand": "tests/test_oracle_baselines.py",
}


def apply(name: str) -> None:
    MUTANTS[name]()
