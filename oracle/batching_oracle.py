"""Plain, slow reference of the adaptive batching scheduler (paper section 4.2, equations 2-5).
TEST INFRASTRUCTURE ONLY; shares no code with the C++ scheduler behind include/lora_sched.h.

Per function i (equation 2):  T_i(b) = t0_i + alpha_i * (b - 1)  -- time to first token of a batch of b.
B_i = the largest b with T_i(b) <= SLO_i (at least 1)            -- "maximum batch size within the SLO".
N_i = the function's current batch size setting, 1 <= N_i <= B_i; its batch delay (equation 3) is
    d_i = SLO_i - T_i(N_i).
Fill or expire: the forming batch of i = its oldest min(queued, N_i) requests; it is READY when it holds N_i requests
or when its oldest request has waited d_i.  (A batch of n <= N_i requests dispatched then produces its first
token after at most d_i + T_i(n) <= SLO_i.)  With M batches sharing the GPU a batch takes M * T_i(b) (equation 4)
and its deadline margin is
    margin = SLO_i - (w + M * T_i(b)),  w = time its oldest request has waited, b = its size          (equation 5)
Ready batches are dispatched in order of increasing margin (ties: lower function index).

Readings taken where the text is open (each also listed in the design document):
  * N_i in equation 3 is the function's batch size setting (the same N_i that closes the batch), not the number
    collected so far; the text leaves its choice to an adjustment loop it does not describe, so it is a parameter
    here (default: half of B_i, at least 1) that the caller may change at any time;
  * M counts the batch under decision: M = batches already running + 1; it orders ready batches and is
    reported, it does not enter the batch delay (equation 3 is printed without it).
"""
from __future__ import annotations

import math

MAX_BATCH_LIMIT = 65536  # requests one lora_plan accepts


class BatchingOracle:
    def __init__(self, profiles):
        self.p = [dict(t0=float(q["t0_ms"]), alpha=float(q["alpha_ms"]), slo=float(q["slo_ms"]),
                       adapter=int(q.get("adapter", -1)), cap=int(q.get("max_batch", 0))) for q in profiles]
        self.q = [[] for _ in self.p]  # per function: list of (id, arrival, ntok), oldest first
        self.n_set = [max(1, self.max_batch(i) // 2) for i in range(len(self.p))]
        self.next_id = 0

    def T(self, i, b):
        return self.p[i]["t0"] + self.p[i]["alpha"] * (b - 1)

    def max_batch(self, i):
        b = 1
        while b < MAX_BATCH_LIMIT and self.T(i, b + 1) <= self.p[i]["slo"]:
            b += 1
        if self.p[i]["cap"] > 0:
            b = min(b, self.p[i]["cap"])
        return b

    def set_batch_size(self, i, n):
        assert 1 <= n <= self.max_batch(i)
        self.n_set[i] = n

    def delay(self, i):
        return self.p[i]["slo"] - self.T(i, self.n_set[i])

    def submit(self, i, ntok, now):
        rid = self.next_id
        self.next_id += 1
        self.q[i].append((rid, float(now), int(ntok)))
        return rid

    def _state(self, i, now, running):
        """(n, expiry time, margin, T(n), w) of function i's forming batch, or None if its queue is empty."""
        if not self.q[i]:
            return None
        M = running + 1
        n = min(len(self.q[i]), self.n_set[i])
        tb = self.T(i, n)
        t_old = self.q[i][0][1]
        t_exp = t_old + self.delay(i)
        w = now - t_old
        margin = self.p[i]["slo"] - (w + M * tb)
        return n, t_exp, margin, tb, w

    def poll(self, now, running, max_batches=1 << 30, max_requests=1 << 30):
        ready = []
        for i in range(len(self.p)):
            st = self._state(i, now, running)
            if st is None:
                continue
            n, t_exp, margin, tb, w = st
            if n == self.n_set[i] or now >= t_exp:
                ready.append((margin, i, n, tb, w))
        ready.sort(key=lambda r: (r[0], r[1]))
        out, used = [], 0
        for margin, i, n, tb, w in ready:
            if len(out) >= max_batches or used + n > max_requests:
                break
            reqs, self.q[i] = self.q[i][:n], self.q[i][n:]
            out.append(dict(function=i, adapter=self.p[i]["adapter"], n=n, first=used, wait_ms=w, margin_ms=margin,
                            t_batch_ms=tb, request_ids=[r[0] for r in reqs], ntok=[r[2] for r in reqs]))
            used += n
        return out

    def next_event(self, now, running):
        t = math.inf
        for i in range(len(self.p)):
            st = self._state(i, now, running)
            if st is None:
                continue
            n, t_exp, _, _, _ = st
            t = min(t, now if n == self.n_set[i] else max(now, t_exp))
        return t

    def queued(self, i):
        return len(self.q[i])
