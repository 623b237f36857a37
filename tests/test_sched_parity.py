"""The native schedulers behind include/lora_sched.h against their oracles: the same random request traces and
artifact sets through both, every decision compared exactly (ids, order, sizes; times and margins to the last bit --
both sides evaluate the paper's formulas in the same order in IEEE doubles).  Host code: no GPU needed."""
import json
import math
import os
import re

import numpy as np
import pytest

from oracle.batching_oracle import BatchingOracle
from oracle import residency_oracle as R
from paper_2505_14468_amd import sched as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = json.load(open(os.path.join(ROOT, "tests", "golden", "scheduling_examples.json")))


def test_library_exports_every_symbol_of_the_scheduling_header():
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "lora_sched.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(lora_[a-z_]+)\s*\(", text)))
    assert sorted(S.EXPORTS) == names
    for n in names:
        assert hasattr(S.lib(), n), n


def _same_batches(got, want):
    assert len(got) == len(want)
    for g, w in zip(got, want):
        for k in ("function", "adapter", "n", "first", "request_ids", "ntok", "wait_ms", "margin_ms", "t_batch_ms"):
            assert g[k] == w[k], (k, g[k], w[k])


@pytest.mark.parametrize("seed", range(8))
def test_batcher_matches_the_oracle_on_random_traces(seed):
    rng = np.random.default_rng(seed)
    nf = int(rng.integers(1, 7))
    prof = [dict(t0_ms=float(rng.integers(50, 900)) + 0.125 * float(rng.integers(0, 8)), alpha_ms=float(rng.integers(0, 200)) / 4.0,
                 slo_ms=float(rng.integers(300, 5000)), adapter=int(rng.integers(-1, 40)),
                 max_batch=int(rng.choice([0, 0, 3, 12]))) for _ in range(nf)]
    nat, ora = S.Batcher(prof), BatchingOracle(prof)
    for i in range(nf):
        assert nat.max_batch(i) == ora.max_batch(i) and nat.batch_size(i) == ora.n_set[i] and nat.delay(i) == ora.delay(i)
        if rng.random() < 0.5:
            n = int(rng.integers(1, ora.max_batch(i) + 1))
            nat.set_batch_size(i, n)
            ora.set_batch_size(i, n)
    arrivals = [(int(rng.integers(0, nf)), float(t), int(rng.integers(0, 40))) for t in np.cumsum(rng.exponential(40.0, size=400))]
    now, k, running, dispatched = 0.0, 0, 0, 0
    while True:
        running = int(rng.integers(0, 4))
        t_ev_n, t_ev_o = nat.next_event(now, running), ora.next_event(now, running)
        assert t_ev_n == t_ev_o
        t = min(arrivals[k][1] if k < len(arrivals) else math.inf, t_ev_o)
        if t == math.inf:
            break
        now = t
        while k < len(arrivals) and arrivals[k][1] <= now:
            f, ta, ntok = arrivals[k]
            assert nat.submit(f, ntok, ta) == ora.submit(f, ntok, ta)
            k += 1
        limits = dict(max_batches=int(rng.integers(1, 4)), max_requests=int(rng.integers(40, 200)))
        got, ra, rn, ids = nat.poll(now, running, **limits)
        want = ora.poll(now, running, **limits)
        _same_batches(got, want)
        # the flat arrays are the multi-LoRA batch lora_plan takes
        assert ra.tolist() == [b["adapter"] for b in want for _ in range(b["n"])]
        assert rn.tolist() == [x for b in want for x in b["ntok"]] and ids.tolist() == [x for b in want for x in b["request_ids"]]
        dispatched += sum(b["n"] for b in want)
        for i in range(nf):
            assert nat.queued(i) == ora.queued(i)
        if not want and t_ev_o <= now and (k >= len(arrivals) or arrivals[k][1] > now):
            # a ready batch that the limits keep queued: let the next poll take it with room to spare
            got, _, _, _ = nat.poll(now, running)
            _same_batches(got, ora.poll(now, running, max_batches=64, max_requests=4096))
            dispatched += sum(b["n"] for b in got)
    assert dispatched == len(arrivals)


def test_batcher_worked_example_and_argument_errors():
    g = GOLD["batching"]
    for chk in g["checks"]:
        nat = S.Batcher(g["profiles"])
        for f, t, ntok in sorted(g["arrivals"], key=lambda a: a[1]):
            nat.submit(f, ntok, t)
        got, ra, rn, ids = nat.poll(chk["now"], g["running"])
        assert [b["function"] for b in got] == chk["ready"]
        assert [b["margin_ms"] for b in got] == [chk["margins"][f] for f in chk["ready"]]
    nat = S.Batcher(g["profiles"])
    assert [nat.max_batch(i) for i in range(2)] == g["max_batch"] and [nat.delay(i) for i in range(2)] == g["delay_ms"]
    assert nat.submit(5, 1, 0.0, raw=True) == S.LORA_SCHED_ERR_INVALID_ARG       # no such function
    assert nat.submit(0, -1, 0.0, raw=True) == S.LORA_SCHED_ERR_INVALID_ARG      # negative token count
    assert nat.submit(0, 1, float("nan"), raw=True) == S.LORA_SCHED_ERR_INVALID_ARG
    assert nat.submit(0, 1, 10.0, raw=True) == S.LORA_SCHED_OK
    assert nat.submit(0, 1, 9.0, raw=True) == S.LORA_SCHED_ERR_INVALID_ARG       # time runs backwards
    assert nat.set_batch_size(0, 22, raw=True) == S.LORA_SCHED_ERR_INVALID_ARG   # beyond B = 21
    assert nat.set_batch_size(0, 0, raw=True) == S.LORA_SCHED_ERR_INVALID_ARG
    nat.set_batch_size(0, 1)
    assert nat.poll(10.0, 0, max_batches=1, max_requests=0, raw=True) == S.LORA_SCHED_ERR_CAPACITY  # ready, no room at all
    with pytest.raises(S.SchedError):
        S.Batcher([dict(t0_ms=-1.0, alpha_ms=1.0, slo_ms=10.0)])


def _random_artifacts(rng, n_fn):
    arts, size = [], {}
    for f in range(n_fn):
        for k in (R.LIB, R.BACKBONE, R.ADAPTER, R.KERNEL):
            if rng.random() < 0.8:
                a = dict(function=f * 3 + 1, kind=k, share_id=int(rng.integers(0, 3)), pinned=int(rng.random() < 0.15),
                         bytes=float(rng.integers(1, 9)) * 0.5, value=float(rng.integers(0, 40)) * 0.25)
                if k == R.BACKBONE:
                    a["bytes"] = size.setdefault(a["share_id"], a["bytes"])
                arts.append(a)
    return arts


@pytest.mark.parametrize("seed", range(25))
def test_preload_and_offload_match_the_oracle(seed):
    rng = np.random.default_rng(500 + seed)
    arts = _random_artifacts(rng, int(rng.integers(1, 12)))
    cb, gb = float(rng.integers(0, 20)), float(rng.integers(0, 30))
    assert S.lora_preload_greedy(arts, cb, gb) == R.preload_greedy(arts, cb, gb)
    on_gpu = [int(rng.random() < 0.7) for _ in arts]
    need = float(rng.integers(0, 25)) * 0.5
    assert S.lora_offload_greedy(arts, on_gpu, need) == R.offload_greedy(arts, on_gpu, need)


def test_residency_worked_examples_and_argument_errors():
    g, o = GOLD["preload"], GOLD["offload"]
    assert S.lora_preload_greedy(g["artifacts"], g["container_bytes"], g["gpu_bytes"]) == (g["place"], g["value"])
    assert S.lora_offload_greedy(g["artifacts"], o["on_gpu"], o["need_bytes"]) == (o["evict"], o["freed"], o["value_lost"], True)
    assert S.lora_offload_greedy(g["artifacts"], o["on_gpu"], 1e9)[3] is False  # not enough removable bytes: best effort, flagged
    bad = [dict(g["artifacts"][0], bytes=0.0)]
    assert S.lora_preload_greedy(bad, 1.0, 1.0, raw=True) == S.LORA_SCHED_ERR_INVALID_ARG
    twice = [g["artifacts"][2], g["artifacts"][2]]  # two adapters of one function
    assert S.lora_preload_greedy(twice, 1.0, 1.0, raw=True) == S.LORA_SCHED_ERR_INVALID_ARG
    sizes = [dict(g["artifacts"][1]), dict(g["artifacts"][5], bytes=11.0)]  # one shared backbone, two sizes
    assert S.lora_preload_greedy(sizes, 1.0, 1.0, raw=True) == S.LORA_SCHED_ERR_INVALID_ARG
    assert S.lora_preload_greedy([], 1.0, 1.0) == ([], 0.0)
