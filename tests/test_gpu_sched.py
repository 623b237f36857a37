"""The two schedulers driving the layer on the GPU: batches formed by the native batching scheduler go through
lora_plan / lora_linear and are checked against the layer's oracle; an adapter pool larger than its GPU budget is
kept resident by the greedy value-density policy (pre-load, offload, asynchronous upload) while every batch still
matches the oracle."""
import math

import numpy as np
import pytest

from workloads import make_custom

pytestmark = pytest.mark.gpu


def test_batches_from_the_batching_scheduler_run_through_the_layer():
    import torch
    from gpu_common import rt, ctx, check_against_oracle, reset_options
    from paper_2505_14468_amd import sched as S
    from workloads import to_f64
    reset_options()
    c = ctx()
    rng = np.random.default_rng(7)
    n_fn = 6
    ranks = (8, 16, 32, 8, 64, 16)
    prof = [dict(t0_ms=500.0, alpha_ms=100.0, slo_ms=2500.0, adapter=i) for i in range(n_fn)]
    prof[5]["adapter"] = -1  # a function that serves the bare backbone
    nat = S.Batcher(prof)
    for i in range(n_fn):
        nat.set_batch_size(i, int(rng.integers(2, 9)))
    arrivals = [(int(rng.integers(0, n_fn)), float(t), int(rng.integers(1, 30))) for t in np.cumsum(rng.exponential(80.0, size=120))]
    now, k, seen, calls = 0.0, 0, 0, 0
    while True:
        t = min(arrivals[k][1] if k < len(arrivals) else math.inf, nat.next_event(now, 0))
        if t == math.inf:
            break
        now = t
        while k < len(arrivals) and arrivals[k][1] <= now:
            nat.submit(arrivals[k][0], arrivals[k][2], arrivals[k][1])
            k += 1
        batches, req_adapter, req_ntok, ids = nat.poll(now, 0, max_batches=4, max_requests=256)
        if not batches:
            continue
        seen += len(ids)
        if calls >= 6:  # every dispatch is accounted for; the layer runs on the first few
            continue
        calls += 1
        wl = make_custom(seed=6000 + calls, dtype="bf16", K=264, N=200, ranks=ranks, scales=(2.0, 1.0, 0.5, 2.0, 0.25, 1.0),
                         req_adapter=req_adapter, req_ntok=req_ntok, name=f"batched_{calls}")
        X, W0, table = rt.upload_workload(wl, 0, c.device)
        pl = rt.plan(c, req_adapter, req_ntok, wl.ranks, wl.r_max)  # the scheduler's arrays, as they are
        Y = rt.linear(c, pl, X, W0, table)
        torch.cuda.synchronize()
        assert pl.status(c)[0] == 0
        e = check_against_oracle(wl, to_f64(rt.bits_from_tensor(Y)))
        print(f"dispatch {calls}: {len(batches)} batch(es), {len(ids)} requests, T={wl.T}, err/rms {e:.2e}", flush=True)
    assert seen == len(arrivals) and calls == 6


def test_adapter_pool_keeps_the_batches_adapters_resident_within_its_budget():
    import torch
    from gpu_common import B, rt, ctx, check_against_oracle, reset_options
    from workloads import to_f64
    reset_options()
    c = ctx()
    rng = np.random.default_rng(11)
    n_ad, K, N = 12, 264, 200
    ranks = tuple(int(r) for r in rng.choice([8, 16, 32], size=n_ad))
    scales = tuple(float(s) for s in rng.choice([0.5, 1.0, 2.0], size=n_ad))
    base = make_custom(seed=6100, dtype="bf16", K=K, N=N, ranks=ranks, scales=scales, req_adapter=[0], req_ntok=[1])
    sizes = [2.0 * r * (K + N) for r in ranks]
    budget = sum(sorted(sizes)[-6:])  # room for the six largest (any batch below fits), not for all twelve
    rates = [float(x) for x in rng.integers(1, 20, size=n_ad)]
    pool = rt.AdapterPool(c, [base.A(a) for a in range(n_ad)], [base.B(a) for a in range(n_ad)], scales, budget, rates)
    pool.preload()
    assert 0 < pool.used_bytes() <= budget
    first = [a for a in range(n_ad) if pool.resident[a]]
    dens = [pool.load_ms[a] * rates[a] / sizes[a] for a in range(n_ad)]
    assert min(dens[a] for a in first) >= max([dens[a] for a in range(n_ad) if a not in first and sizes[a] <= budget - pool.used_bytes()] + [0.0])
    X = rt.tensor_from_bits(base.X(0)[:0], c.device)  # (dtype only)
    W0 = rt.tensor_from_bits(base.W0(0), c.device)
    for step in range(8):
        R = int(rng.integers(3, 8))  # at most six distinct adapters per batch
        ids = rng.choice(n_ad, size=R, replace=True)
        ids[0] = -1
        L = rng.integers(1, 6 if step % 2 else 60, size=R)
        wl = make_custom(seed=6100, dtype="bf16", K=K, N=N, ranks=ranks, scales=scales, req_adapter=ids, req_ntok=L, name=f"pool_{step}")
        wl.seed = 6100  # the same adapters (and W0) as the pool holds; X is drawn per batch shape
        moved = pool.ensure(ids)
        assert pool.used_bytes() <= budget + 1e-6 and all(pool.resident[a] for a in ids if a >= 0)
        assert not set(moved["evicted"]) & set(int(a) for a in ids)
        Xb = rt.tensor_from_bits(wl.X(0), c.device)
        pl = rt.plan(c, ids, L, wl.ranks, wl.r_max)
        Y = rt.linear(c, pl, Xb, W0, pool.table)
        torch.cuda.synchronize()
        assert pl.status(c)[0] == 0
        e = check_against_oracle(wl, to_f64(rt.bits_from_tensor(Y)))
        print(f"step {step}: uploaded {moved['uploaded']} evicted {moved['evicted']} resident {sum(pool.resident)} err/rms {e:.2e}", flush=True)
    assert any(kind == "evict" for kind, _ in pool.log)
    # a batch that uses an adapter the pool has offloaded, without asking the pool first: flagged, never dereferenced
    gone = next(a for a in range(n_ad) if not pool.resident[a])
    wl = make_custom(seed=6100, dtype="bf16", K=K, N=N, ranks=ranks, scales=scales, req_adapter=[gone, -1], req_ntok=[3, 2])
    pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks, wl.r_max)
    rt.linear(c, pl, rt.tensor_from_bits(wl.X(0), c.device), W0, pool.table)
    assert pl.status(c)[0] == B.LORA_ERR_ADAPTER_NOT_RESIDENT
