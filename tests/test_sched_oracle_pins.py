"""Pins of the scheduling oracles (oracle/batching_oracle.py, oracle/residency_oracle.py) against what the paper and
the mathematics fix: closed forms of equations 2-5, hand-derived worked examples (tests/golden/
scheduling_examples.json), invariants (every request meets its SLO when the GPU is uncontended; capacity and
precedence hold), and exhaustive optima on tiny instances."""
import json
import math
import os

import numpy as np
import pytest

from oracle.batching_oracle import BatchingOracle
from oracle import residency_oracle as R

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "scheduling_examples.json")))


# ---- batching (section 4.2) ------------------------------------------------------------------------------------
def test_max_batch_closed_form():
    for t0 in (100, 500, 800, 3000):
        for alpha in (1, 7, 100, 250):
            for slo in (2500, 4000, 90):
                o = BatchingOracle([dict(t0_ms=t0, alpha_ms=alpha, slo_ms=slo)])
                want = 1 if t0 > slo else (slo - t0) // alpha + 1  # integers: exact
                assert o.max_batch(0) == want, (t0, alpha, slo)
    assert BatchingOracle([dict(t0_ms=500, alpha_ms=100, slo_ms=2500, max_batch=8)]).max_batch(0) == 8
    assert BatchingOracle([dict(t0_ms=500, alpha_ms=0, slo_ms=2500)]).max_batch(0) == 65536  # no marginal cost: the plan's limit


def test_lone_request_waits_exactly_the_batch_delay():
    g = GOLD["batching"]
    o = BatchingOracle(g["profiles"])
    assert [o.n_set[i] for i in range(2)] == g["batch_size_default"] and [o.delay(i) for i in range(2)] == g["delay_ms"]
    o.submit(1, 10, 50.0)
    d = 4000.0 - (800.0 + 200.0 * 7)  # equation 3 with N = 8
    assert o.next_event(50.0, 0) == 50.0 + d
    assert o.poll(50.0 + d - 1e-6, 0) == []
    (b,) = o.poll(50.0 + d, 0)
    assert (b["function"], b["n"], b["request_ids"], b["ntok"]) == (1, 1, [0], [10])
    assert b["wait_ms"] == d and b["t_batch_ms"] == 800.0 and b["margin_ms"] == 4000.0 - (d + 800.0)
    # with the batch size set to 1 the delay is SLO - T(1) and the first token arrives exactly at the SLO
    o.set_batch_size(1, 1)
    o.submit(1, 4, 5000.0)
    assert o.poll(5000.0, 0)[0]["margin_ms"] == 4000.0 - 800.0  # N = 1: full at once


def test_delay_grows_as_the_batch_size_setting_shrinks():
    """Equation 3: d = SLO - T(N); the scheduler waits longer when the batch size is small."""
    o = BatchingOracle(GOLD["batching"]["profiles"])
    prev = None
    for n in range(21, 0, -1):
        o.set_batch_size(0, n)
        assert o.delay(0) == 2500.0 - (500.0 + 100.0 * (n - 1))
        assert prev is None or o.delay(0) - prev == 100.0
        prev = o.delay(0)
    assert BatchingOracle(GOLD["batching"]["profiles"]).delay(0) == 1100.0


def test_worked_example_margins_and_order():
    g = GOLD["batching"]
    assert [BatchingOracle(g["profiles"]).max_batch(i) for i in range(2)] == g["max_batch"]
    for chk in g["checks"]:
        o = BatchingOracle(g["profiles"])
        for f, t, ntok in sorted(g["arrivals"], key=lambda a: a[1]):
            o.submit(f, ntok, t)
        margins = [o._state(i, chk["now"], g["running"])[2] for i in range(2)]
        assert margins == chk["margins"]
        out = o.poll(chk["now"], g["running"])
        assert [b["function"] for b in out] == chk["ready"]
        assert [b["margin_ms"] for b in out] == sorted(b["margin_ms"] for b in out)


def test_burst_fills_batches_at_once():
    o = BatchingOracle([dict(t0_ms=500, alpha_ms=100, slo_ms=2500, adapter=4)])
    for _ in range(50):
        o.submit(0, 3, 10.0)
    sizes = []
    while True:
        out = o.poll(10.0, 0)
        if not out:
            break
        sizes += [b["n"] for b in out]
    assert sizes == [10] * 5 and o.queued(0) == 0  # full batches (N = 10) leave immediately
    for _ in range(7):
        o.submit(0, 3, 20.0)
    assert o.poll(20.0, 0) == [] and o.next_event(20.0, 0) == 20.0 + 1100.0  # a partial batch waits for its delay


def _simulate(o, arrivals, running=0):
    """Event-driven run: polls at every arrival and at every time the scheduler announces.  Returns
    [(dispatch time, batch)] ."""
    arrivals = sorted(arrivals, key=lambda a: a[1])
    out, now, k = [], 0.0, 0
    while True:
        t_next = arrivals[k][1] if k < len(arrivals) else math.inf
        t_ev = o.next_event(now, running)
        t = min(t_next, t_ev)
        if t == math.inf:
            return out
        now = t
        while k < len(arrivals) and arrivals[k][1] <= now:
            o.submit(arrivals[k][0], arrivals[k][2], arrivals[k][1])
            k += 1
        while True:
            got = o.poll(now, running)
            if not got:
                break
            out += [(now, b) for b in got]


@pytest.mark.parametrize("seed", range(5))
def test_every_request_meets_its_slo_on_an_uncontended_gpu(seed):
    rng = np.random.default_rng(seed)
    prof = [dict(t0_ms=float(rng.integers(100, 900)), alpha_ms=float(rng.integers(5, 200)), slo_ms=float(rng.integers(1000, 5000)),
                 adapter=i) for i in range(4)]
    arrivals = [(int(rng.integers(0, 4)), float(t), int(rng.integers(1, 50))) for t in np.cumsum(rng.exponential(60.0, size=300))]
    o = BatchingOracle(prof)
    arrive = {}
    for rid, a in enumerate(sorted(arrivals, key=lambda a: a[1])):
        arrive[rid] = a
    done = set()
    for t, b in _simulate(o, arrivals):
        p = prof[b["function"]]
        full = b["n"] == o.n_set[b["function"]]
        oldest = arrive[b["request_ids"][0]][1]
        if not full:  # expired: dispatched exactly when its delay ran out, not earlier
            assert abs(t - (oldest + o.delay(b["function"]))) < 1e-6
        for rid in b["request_ids"]:
            assert arrive[rid][0] == b["function"] and rid not in done
            done.add(rid)
            assert t - arrive[rid][1] + b["t_batch_ms"] <= p["slo_ms"] + 1e-6  # time to first token within the SLO
        assert b["request_ids"] == sorted(b["request_ids"])  # first come, first served inside a function
    assert len(done) == len(arrivals)


# ---- residency (sections 4.1, 4.3) -----------------------------------------------------------------------------
def test_preload_worked_example():
    g = GOLD["preload"]
    mask, value = R.preload_greedy(g["artifacts"], g["container_bytes"], g["gpu_bytes"])
    assert mask == g["place"] and value == g["value"]


def test_offload_worked_example():
    g, o = GOLD["preload"], GOLD["offload"]
    evict, freed, lost, enough = R.offload_greedy(g["artifacts"], o["on_gpu"], o["need_bytes"])
    assert (evict, freed, lost, enough) == (o["evict"], o["freed"], o["value_lost"], True)


def _random_artifacts(rng, n_fn, with_deps, equal_bytes):
    arts = []
    for f in range(n_fn):
        kinds = [R.ADAPTER]
        if with_deps:
            kinds = [k for k in (R.LIB, R.BACKBONE, R.ADAPTER, R.KERNEL) if rng.random() < 0.8] or [R.ADAPTER]
        for k in kinds:
            arts.append(dict(function=f, kind=k, share_id=int(rng.integers(0, 2)), pinned=0,
                             bytes=1.0 if equal_bytes else float(rng.integers(1, 6)), value=float(rng.integers(0, 20))))
    # members of one shared backbone have one size
    size = {}
    for a in arts:
        if a["kind"] == R.BACKBONE:
            a["bytes"] = size.setdefault(a["share_id"], a["bytes"])
    return arts


@pytest.mark.parametrize("seed", range(8))
def test_preload_greedy_is_optimal_for_equal_sizes_without_precedence(seed):
    rng = np.random.default_rng(seed)
    arts = _random_artifacts(rng, 5, with_deps=False, equal_bytes=True)
    cb, gb = float(rng.integers(0, 4)), float(rng.integers(0, 4))
    mask, value = R.preload_greedy(arts, cb, gb)
    assert value == R.preload_optimal(arts, cb, gb)


@pytest.mark.parametrize("seed", range(8))
def test_preload_greedy_respects_constraints_and_never_beats_the_optimum(seed):
    rng = np.random.default_rng(100 + seed)
    arts = _random_artifacts(rng, 3, with_deps=True, equal_bytes=False)
    cb, gb = float(rng.integers(2, 10)), float(rng.integers(2, 14))
    mask, value = R.preload_greedy(arts, cb, gb)
    objs = R._objects(arts)
    of, fn = R._obj_of(objs, len(arts)), R._fn_index(arts)
    placed = {(of[i], pl) for i, m in enumerate(mask) for pl, bit in ((R.CONTAINER, 1), (R.GPU, 2)) if m & bit}
    for pl, cap in ((R.CONTAINER, cb), (R.GPU, gb)):
        assert sum(objs[k]["bytes"] for k, p in placed if p == pl) <= cap
    for c in placed:  # every placement is supported by the others
        assert R._feasible(arts, objs, of, fn, placed - {c}, c[0], c[1])
    assert value <= R.preload_optimal(arts, cb, gb) + 1e-9
    # maximal: nothing that still fits was left out
    for k, o in enumerate(objs):
        for pl, cap in ((R.CONTAINER, cb), (R.GPU, gb)):
            fits = sum(objs[q]["bytes"] for q, p in placed if p == pl) + o["bytes"] <= cap
            assert not (fits and R._feasible(arts, objs, of, fn, placed, k, pl))


def test_density_order_is_scale_invariant():
    rng = np.random.default_rng(5)
    arts = _random_artifacts(rng, 4, with_deps=True, equal_bytes=False)
    m1, _ = R.preload_greedy(arts, 6.0, 9.0)
    scaled = [dict(a, bytes=a["bytes"] * 4.0, value=a["value"] * 4.0) for a in arts]
    m2, _ = R.preload_greedy(scaled, 24.0, 36.0)
    assert m1 == m2


@pytest.mark.parametrize("seed", range(10))
def test_offload_frees_enough_in_dependency_order_and_loses_the_least_for_equal_sizes(seed):
    rng = np.random.default_rng(200 + seed)
    equal = seed % 2 == 0
    arts = _random_artifacts(rng, 4, with_deps=not equal, equal_bytes=equal)
    for a in arts:
        a["pinned"] = int(rng.random() < 0.2)
    on_gpu = [int(a["kind"] != R.LIB and rng.random() < 0.8) for a in arts]
    need = float(rng.integers(1, 8))
    evict, freed, lost, enough = R.offload_greedy(arts, on_gpu, need)
    best = R.offload_optimal(arts, on_gpu, need)
    assert enough == (best is not None)
    for i, e in enumerate(evict):
        assert not (e and (arts[i]["pinned"] or not on_gpu[i] or arts[i]["kind"] == R.LIB))
    objs, here, pinned, dependents = R._gpu_state(arts, on_gpu)
    of = R._obj_of(objs, len(arts))
    chosen = {of[i] for i, e in enumerate(evict) if e}
    assert all(dependents[k] <= chosen for k in chosen)  # nothing is removed from under a dependent
    if enough:
        assert freed >= need and lost >= best - 1e-9
        if equal:
            assert lost == best
