#!/usr/bin/env python3
"""Benchmark of the multi-LoRA batched linear layer on one MI355X.

One "step" = the whole hot path over one batch: the device-side segment builder
(``lora_plan_device`` on request arrays already in HBM) followed by ``lora_linear``
(segmented shrink + base GEMM with the adapter term added before the single store of Y).
Consecutive steps rotate over several independent weight sets (backbone + adapters +
activations), as the layers of a model would, so that decode-sized runs stream their
weights from HBM instead of re-reading one set from the caches.

The default run times ALL FIVE workload configurations (configuration 3 as its seven
projections, plus the decoder layer as one step with one plan, with and without the fused
q/k/v and gate/up calls, and a 32-layer loop on one plan) and prints ONE JSON line: the
headline fields describe the largest one (configuration 2, the prefill-shaped MLP
up-projection; ``--steps`` / ``--warmup`` apply to it), ``per_config`` holds every
configuration's step time, step time with the plan amortised over the 7 x 32 layer calls
of a model step, per-kernel microseconds (HIP event pairs around every launch, in a second
pass over the same steps), the roofline of the dominant kernel and of each other kernel,
whole-call algorithmic bytes over time, the adapter path's GB/s, parity against the
oracle and the oracle's own throughput on the host cores.  ``--config i`` runs one
configuration alone and prints its line.

Inputs are seeded and synthetic (``workloads``), shaped like LoRA-on-Llama2 serving;
nothing is read from disk except ``profiles/hbm_traffic.json`` (HBM bytes per launch from
earlier rocprofv3 counter runs of this same command; quoted, not measured by this run).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "multi-LoRA linear TFLOP/s + adapter-path GB/s (roofline %), ms/layer"
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 matrix, published
# ceilings measured on this part (a long streaming read; a register-only bf16 MFMA loop on random operands, whose
# clock is power-limited to ~1.7 GHz): context beside the published peaks, which `frac` is computed against
MEASURED_HBM_GBPS = 6500.0
MEASURED_BF16_TFLOPS = 1700.0
HBM_BOUND = {0: False, 1: True, 2: False, 3: False, 4: False}  # which roofline bounds the dominant kernel
PLAN_REUSE = 7 * 32  # layer calls that share one plan in a model step (seven projections x 32 decoder layers)
HEADLINE = 2


def _layer_variant(wl, layer):
    """Same batch and shapes, independent weight / activation values for layer > 0."""
    if layer == 0:
        return wl
    import copy
    w2 = copy.copy(wl)
    w2.seed = wl.seed + 7919 * layer
    w2._cache = {}
    return w2


def _timed(torch, fn, k):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(k):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / k


def _upload(rt, wl, p, dev):
    """Device tensors of one projection; adapters the batch does not use share one stand-in buffer per kind
    (no kernel reads a slot the batch does not use), so that a pool of hundreds of adapters need not be drawn."""
    X, W0, table = rt.upload_workload(wl, p, dev, only_used=True)
    some = next((a for a in range(wl.n_adapters) if table.A[a] is not None), None)
    if some is not None:
        same = [a for a in range(wl.n_adapters) if table.A[a] is None and wl.ranks[a] == wl.ranks[some]]
        for a in same:
            table.set_slot(a, table.A[some], table.B[some])
    return X, W0, table


def _roof(bound, alg, us, dtype):
    """Roofline block of one kernel: alg = algorithmic bytes (hbm) or flops (mfma) per launch, us = its duration."""
    if us <= 0:
        return None
    if bound == "hbm":
        ach = alg / (us * 1e-6) / 1e9
        return {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "frac": round(ach / PEAK_HBM_GBPS, 4), "frac_of_measured_ceiling": round(ach / MEASURED_HBM_GBPS, 4)}
    peak = PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_F32_TFLOPS
    ach = alg / (us * 1e-6) / 1e12
    out = {"bound": "mfma", "achieved": round(ach, 1), "peak": peak, "unit": "TFLOP/s", "frac": round(ach / peak, 4)}
    if dtype == "bf16":
        out["frac_of_measured_ceiling"] = round(ach / MEASURED_BF16_TFLOPS, 4)
    return out


def run_projection(ctx, mods, wl, cfg_index, p, steps, warmup, cpu_seconds, options=()):
    """Times plan + lora_linear of projection p of a workload; returns the result dict of that configuration."""
    np, torch, B, rt = mods
    pr = wl.projections[p]
    K, N, T = pr.K, pr.N, wl.T
    for name, val in options:
        ctx.set_option(name, val)
    dev = ctx.device
    es = 2 if wl.dtype == "bf16" else 4
    tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    h = ctx.handle

    # ---- rotating weight sets: enough bytes to overflow L2 + Infinity Cache (256 MB) -----------------------
    used = wl.used_adapters()
    r_used = int(wl.ranks[used].astype(np.int64).sum())
    set_bytes = es * (K * N + T * K + T * N + r_used * (K + N))
    n_sets = max(1, min(16, int(np.ceil(6.0e8 / set_bytes))))
    sets = []
    for layer in range(n_sets):
        w = _layer_variant(wl, layer)
        X, W0, table = _upload(rt, w, p, dev)
        Y = torch.empty((T, N), dtype=tdtype, device=dev)
        sets.append((X, W0, table, Y))
        if layer > 0:
            w.drop_cache()
    req_adapter = torch.from_numpy(np.ascontiguousarray(wl.req_adapter)).to(dev)
    req_ntok = torch.from_numpy(np.ascontiguousarray(wl.req_ntok)).to(dev)
    ranks = torch.from_numpy(np.ascontiguousarray(wl.ranks)).to(dev)
    r_max = wl.r_max
    plan_bytes = B.lora_plan_bytes(wl.n_req, T, wl.n_adapters, r_max)
    plan_buf = torch.empty(plan_bytes, dtype=torch.uint8, device=dev)
    ws = rt.workspace(T, K, N, r_max, tdtype, dev)
    stream = int(torch.cuda.current_stream().cuda_stream)
    plan0 = rt.plan_device(ctx, req_adapter, req_ntok, ranks, r_max, T, buf=plan_buf)
    descs = [rt.linear_desc(plan0, X, W0, Y, table, ws) for (X, W0, table, Y) in sets]
    descs_base = [rt.linear_desc(plan0, X, W0, Y, None, ws) for (X, W0, table, Y) in sets]
    ra_p, rn_p, rk_p, pb_p = req_adapter.data_ptr(), req_ntok.data_ptr(), ranks.data_ptr(), plan_buf.data_ptr()

    def step(i):
        plan = B.lora_plan_device(h, ra_p, rn_p, wl.n_req, rk_p, wl.n_adapters, r_max, T, pb_p, plan_bytes, stream)
        B.lora_linear(h, plan, descs[i % n_sets], stream)

    for i in range(warmup):
        step(i)
    status, n_seg = plan0.status(ctx)
    assert status == 0, f"plan status {status}"

    # ---- the timed region: `steps` whole steps ------------------------------------------------------------
    sec_per_step = _timed(torch, step, steps)
    # ---- the same steps again with every kernel bracketed by its own HIP event pair (the events cost host time
    #      per launch, so this pass is not the one `value` comes from) -----------------------------------------
    B.lora_profile_begin(h, 2 * steps)
    sec_profiled = _timed(torch, step, steps)
    prof = B.lora_profile_end(h, stream)
    # ---- side measurements (not part of `value`) ------------------------------------------------------------
    k2 = max(10, steps // 4)
    sec_layer = _timed(torch, lambda i: B.lora_linear(h, plan0.struct, descs[i % n_sets], stream), k2)
    B.lora_profile_begin(h, 2 * k2)
    _timed(torch, lambda i: B.lora_linear(h, plan0.struct, descs_base[i % n_sets], stream), k2)
    prof_base = B.lora_profile_end(h, stream)
    base_us = (prof_base["shrink"][0] * prof_base["shrink"][1] + prof_base["gemm_expand"][0] * prof_base["gemm_expand"][1]) / k2  # (decode-sized batches: both kernels carry the base product)
    sec_hot = _timed(torch, lambda i: B.lora_linear(h, plan0.struct, descs[0], stream), k2)  # one weight set: cache-resident

    flops = wl.useful_flops(p)
    per_step = lambda pr_, kind, n: pr_[kind][0] * pr_[kind][1] / n  # (a kind may be more than one launch per step)
    k1_us, k2_us, ex_us = per_step(prof, "shrink", steps), per_step(prof, "gemm_expand", steps), per_step(prof, "expand", steps)
    plan_us = per_step(prof, "plan_segments", steps) + per_step(prof, "plan_fill", steps)
    ra_rows = wl.row_adapter()
    rows_by_ad = dict(zip(*np.unique(ra_rows[ra_rows >= 0], return_counts=True)))
    v_elems = int(sum(int(wl.ranks[a]) * int(n) for a, n in rows_by_ad.items()))  # sum over rows of their rank
    rows_ad = int((ra_rows >= 0).sum())
    gemm_name = B.lora_gemm_kernel_name(h, T, K, N, rt.dtype_code(tdtype))
    decode = gemm_name.startswith("decode")
    kernels = {}
    if decode:
        # first kernel streams W0 and the used A_a against X; second sums the slices, adds V B_a, stores Y
        b1 = es * (T * K + K * N + r_used * K)
        f1 = 2 * T * K * (N + r_used)
        b2 = es * (T * N + r_used * N)
        kernels["stream"] = {"name": gemm_name, "us": round(k1_us, 3), "algorithmic_bytes": b1, "algorithmic_flops": f1,
                             "roofline": _roof("hbm", b1, k1_us, wl.dtype)}
        kernels["reduce_expand"] = {"name": "decode_reduce", "us": round(k2_us, 3), "algorithmic_bytes": b2,
                                    "roofline": _roof("hbm", b2, k2_us, wl.dtype)}
        if ex_us > 0:  # much adapter work: V by a launch of its own (counted with the first kernel), the term by the expand kernel
            be = es * (r_used * N + v_elems)
            kernels["expand"] = {"name": "expand", "us": round(ex_us, 3), "algorithmic_bytes": be, "algorithmic_flops": 2 * N * v_elems,
                                 "roofline": _roof("hbm", be, ex_us, wl.dtype)}
        dom = "stream"
    else:
        bs = es * (r_used * K + rows_ad * K) + es * v_elems
        kernels["shrink"] = {"name": "shrink", "us": round(k1_us, 3), "algorithmic_bytes": bs, "algorithmic_flops": 2 * K * v_elems,
                             "roofline": _roof("hbm", bs, k1_us, wl.dtype)}
        split = ex_us > 0
        bg = es * (T * K + K * N + T * N) + (0 if split else es * (r_used * N + v_elems))
        fg = 2 * T * K * N + (0 if split else 2 * N * v_elems)
        kernels["gemm"] = {"name": gemm_name, "us": round(k2_us, 3), "algorithmic_bytes": bg, "algorithmic_flops": fg,
                           "roofline": _roof("hbm" if HBM_BOUND.get(cfg_index, False) else "mfma",
                                             bg if HBM_BOUND.get(cfg_index, False) else fg, k2_us, wl.dtype)}
        if split:
            be = es * (r_used * N + v_elems)
            kernels["expand"] = {"name": "expand", "us": round(ex_us, 3), "algorithmic_bytes": be, "algorithmic_flops": 2 * N * v_elems,
                                 "non_algorithmic_bytes": {"fp32 adapter term written here and read by the GEMM": 2 * 4 * rows_ad * N},
                                 "roofline": _roof("hbm", be, ex_us, wl.dtype)}
        dom = "gemm"
    roofline = dict(kernels[dom]["roofline"] or {})
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(f"{wl.name}:{pr.name}")
    roofline["traffic"] = traffic
    roofline["traffic_source"] = "profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, scaled by a copy kernel; quoted, not measured by this run"
    roofline["kernel"] = kernels[dom]["name"]
    roofline["kernel_us"] = kernels[dom]["us"]
    roofline["algorithmic_bytes"] = kernels[dom]["algorithmic_bytes"]
    roofline["algorithmic_flops"] = kernels[dom].get("algorithmic_flops")

    adapter_bytes = es * (r_used * (K + N) + rows_ad * K) + 2 * es * v_elems
    layer_us = k1_us + k2_us + ex_us
    adapter_us = max(layer_us - base_us, 1e-3)
    alg_bytes = wl.algorithmic_bytes(p)

    # ---- the cpu_baseline leg: the oracle on the host cores, timed as a reported baseline; the rows it computes are
    #      also compared with the GPU's (outside the timed region).  Nothing else in this file touches the oracle. -----
    cpu = None
    parity = None
    if cpu_seconds > 0:
        from oracle import oracle_threads, oracle_workload
        from workloads import to_f64
        est = flops / 2.0e10  # seconds at ~20 GFLOP/s (all host cores)
        n_rows = T if est <= cpu_seconds else max(1, int(T * cpu_seconds / est))
        rows = None if n_rows == T else np.arange(n_rows)
        oracle_workload(wl, p, rows=np.arange(1))  # build + page in
        t0 = time.perf_counter()
        reps = 0
        while True:
            ref = oracle_workload(wl, p, rows=rows)
            reps += 1
            if time.perf_counter() - t0 > 0.5 * cpu_seconds or reps >= 50:
                break
        dt = (time.perf_counter() - t0) / reps
        cpu = {"value": round(flops * (n_rows / T) / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle_threads(), "kind": "oracle",
               "sample": f"{n_rows} of {T} rows of the layer, {reps} repetition(s), {dt:.3f} s each"}
        torch.cuda.synchronize()
        plan = rt.plan_device(ctx, req_adapter, req_ntok, ranks, r_max, T, buf=plan_buf)
        B.lora_linear(h, plan.struct, descs[0], stream)
        torch.cuda.synchronize()
        got = to_f64(rt.bits_from_tensor(sets[0][3][:n_rows]))
        rms = float(np.sqrt((ref ** 2).mean()))
        parity = float(np.abs(got - ref).max() / rms)
        tol = 2e-2 if wl.dtype == "bf16" else 1e-5
        assert parity <= tol, f"parity {parity} > {tol}"
    for name, _ in options:
        ctx.set_option(name, -1)
    wl.drop_cache()
    amort = sec_layer + plan_us * 1e-6 / PLAN_REUSE
    return {
        "value": round(flops / sec_per_step / 1e12, 3), "unit": "TFLOP/s", "dtype": wl.dtype,
        "steps": steps, "warmup": warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5),
        "ms_per_step_plan_amortised": round(amort * 1e3, 5),
        "config": {"workload": f"{wl.name}:{pr.name}", "d_in": K, "d_out": N, "tokens": T, "requests": wl.n_req,
                   "adapters_resident": wl.n_adapters, "adapters_used": int(used.size), "segments": n_seg,
                   "rank_max": r_max, "weight_sets": n_sets, "step": "lora_plan_device + lora_linear",
                   "plan_amortised_over": PLAN_REUSE},
        "roofline": roofline,
        "kernels": kernels,
        "kernel_us": {"plan": round(plan_us, 3), **{k: v["us"] for k, v in kernels.items()}, "layer_without_adapters": round(base_us, 3)},
        "cpu_baseline": cpu,
        "ms_per_layer": round(sec_layer * 1e3, 5),
        "ms_per_layer_cached_weights": round(sec_hot * 1e3, 5),
        "ms_per_step_profiled": round(sec_profiled * 1e3, 5),
        "layer_tflops": round(flops / sec_layer / 1e12, 3),
        "whole_call": {"algorithmic_bytes": alg_bytes, "us": round(sec_layer * 1e6, 3),
                       "gbps": round(alg_bytes / sec_layer / 1e9, 1),
                       "frac_of_hbm_peak": round(alg_bytes / sec_layer / 1e9 / PEAK_HBM_GBPS, 4),
                       "tflops": round(flops / sec_layer / 1e12, 3),
                       "frac_of_mfma_peak": round(flops / sec_layer / 1e12 / (PEAK_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_F32_TFLOPS), 4)},
        "adapter_path": {"bytes": adapter_bytes, "us": round(adapter_us, 3),
                         "gbps": round(adapter_bytes / adapter_us / 1e3, 1),
                         "frac_of_hbm_peak": round(adapter_bytes / adapter_us / 1e3 / PEAK_HBM_GBPS, 4),
                         "how": "adapter bytes over (layer kernels with adapters - layer kernels with tbl = NULL)"},
        "parity_max_err_over_rms": parity,
    }


def run_layer(ctx, mods, wl, steps, warmup, fuse, n_layers=1):
    """One step = one plan + every projection of the workload (configuration 3: the seven projections of a decoder
    layer), optionally q/k/v and gate/up through lora_linear_multi on shared activations; n_layers > 1 repeats
    the layer's calls on the same plan (a model step; the layers share one weight set here)."""
    np, torch, B, rt = mods
    dev, T, r_max = ctx.device, wl.T, wl.r_max
    tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    req_adapter = torch.from_numpy(np.ascontiguousarray(wl.req_adapter)).to(dev)
    req_ntok = torch.from_numpy(np.ascontiguousarray(wl.req_ntok)).to(dev)
    ranks = torch.from_numpy(np.ascontiguousarray(wl.ranks)).to(dev)
    plan_bytes = B.lora_plan_bytes(wl.n_req, T, wl.n_adapters, r_max)
    plan_buf = torch.empty(plan_bytes, dtype=torch.uint8, device=dev)
    plan0 = rt.plan_device(ctx, req_adapter, req_ntok, ranks, r_max, T, buf=plan_buf)
    keep, descs = [], []
    for q, pr in enumerate(wl.projections):
        X, W0, table = _upload(rt, wl, q, dev)
        Y = torch.empty((T, pr.N), dtype=tdtype, device=dev)
        ws = rt.workspace(T, pr.K, pr.N, r_max, tdtype, dev)
        keep.append((X, W0, table, Y, ws))
        descs.append(rt.linear_desc(plan0, X, W0, Y, table, ws))
    wl.drop_cache()
    h, stream = ctx.handle, int(torch.cuda.current_stream().cuda_stream)
    ra_p, rn_p, rk_p, pb_p = req_adapter.data_ptr(), req_ntok.data_ptr(), ranks.data_ptr(), plan_buf.data_ptr()
    groups = [[q] for q in range(len(descs))]
    if fuse:
        names = [pr.name for pr in wl.projections]
        groups, seen = [], set()
        for fam in (("q_proj", "k_proj", "v_proj"), ("o_proj",), ("gate_proj", "up_proj"), ("down_proj",)):
            g = [names.index(n) for n in fam if n in names]
            if g:
                groups.append(g)
                seen.update(g)
        groups += [[q] for q in range(len(descs)) if q not in seen]
        for g in groups:
            for q in g[1:]:
                X0, (Xq, W0, table, Y, ws) = keep[g[0]][0], keep[q]
                assert X0.shape == Xq.shape
                keep[q] = (X0, W0, table, Y, ws)
                descs[q] = rt.linear_desc(plan0, X0, W0, Y, table, ws)

    def step(_):
        plan = B.lora_plan_device(h, ra_p, rn_p, wl.n_req, rk_p, wl.n_adapters, r_max, T, pb_p, plan_bytes, stream)
        for _layer in range(n_layers):
            for g in groups:
                if len(g) == 1:
                    B.lora_linear(h, plan, descs[g[0]], stream)
                else:
                    B.lora_linear_multi(h, plan, [descs[q] for q in g], stream)

    for i in range(warmup):
        step(i)
    status, n_seg = plan0.status(ctx)
    assert status == 0, f"plan status {status}"
    sec = _timed(torch, step, steps)
    flops = n_layers * sum(wl.useful_flops(q) for q in range(len(wl.projections)))
    return {"ms_per_step": round(sec * 1e3, 5), "tflops": round(flops / sec / 1e12, 3), "steps": steps, "warmup": warmup,
            "layers": n_layers,
            "step": "lora_plan_device + " + (f"{n_layers} x (" if n_layers > 1 else "") +
                    " + ".join("lora_linear" if len(g) == 1 else f"lora_linear_multi({len(g)})" for g in groups) +
                    (")" if n_layers > 1 else "")}


def run_fused_copies(ctx, mods, wl, n_proj, steps, warmup):
    """n_proj projections of projection 0's shape on the same activations (own weights and adapters each: q/k/v of a
    model with as many KV heads as query heads), one plan per step: one lora_linear each against one lora_linear_multi."""
    np, torch, B, rt = mods
    dev, T, r_max = ctx.device, wl.T, wl.r_max
    tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    req_adapter = torch.from_numpy(np.ascontiguousarray(wl.req_adapter)).to(dev)
    req_ntok = torch.from_numpy(np.ascontiguousarray(wl.req_ntok)).to(dev)
    ranks = torch.from_numpy(np.ascontiguousarray(wl.ranks)).to(dev)
    plan_bytes = B.lora_plan_bytes(wl.n_req, T, wl.n_adapters, r_max)
    plan_buf = torch.empty(plan_bytes, dtype=torch.uint8, device=dev)
    plan0 = rt.plan_device(ctx, req_adapter, req_ntok, ranks, r_max, T, buf=plan_buf)
    pr = wl.projections[0]
    X, W0, table = _upload(rt, wl, 0, dev)
    wl.drop_cache()
    keep, descs, outs = [], [], []
    for q in range(n_proj):
        copies = {}

        def own(t):
            if t is None:
                return None
            if id(t) not in copies:
                copies[id(t)] = t.clone()
            return copies[id(t)]
        tq = table if q == 0 else rt.AdapterTable([own(t) for t in table.A], [own(t) for t in table.B],
                                                  table.scales.cpu().numpy(), dev)
        Wq = W0 if q == 0 else W0.clone()
        ws = rt.workspace(T, pr.K, pr.N, r_max, tdtype, dev)
        for fused in (0, 1):
            Y = torch.zeros((T, pr.N), dtype=tdtype, device=dev)
            outs.append((q, fused, Y))
            descs.append(rt.linear_desc(plan0, X, Wq, Y, tq, ws))
        keep.append((Wq, tq, ws))
    seq = [d for d, (q, f, _) in zip(descs, outs) if f == 0]
    fus = [d for d, (q, f, _) in zip(descs, outs) if f == 1]
    h, stream = ctx.handle, int(torch.cuda.current_stream().cuda_stream)
    ra_p, rn_p, rk_p, pb_p = req_adapter.data_ptr(), req_ntok.data_ptr(), ranks.data_ptr(), plan_buf.data_ptr()

    def step_seq(_):
        plan = B.lora_plan_device(h, ra_p, rn_p, wl.n_req, rk_p, wl.n_adapters, r_max, T, pb_p, plan_bytes, stream)
        for d in seq:
            B.lora_linear(h, plan, d, stream)

    def step_fused(_):
        plan = B.lora_plan_device(h, ra_p, rn_p, wl.n_req, rk_p, wl.n_adapters, r_max, T, pb_p, plan_bytes, stream)
        B.lora_linear_multi(h, plan, fus, stream)

    res = {}
    for name, fn in (("one_call_each", step_seq), ("lora_linear_multi", step_fused)):
        for i in range(warmup):
            fn(i)
        res[name + "_ms_per_step"] = round(_timed(torch, fn, steps) * 1e3, 5)
    ys = {(q, f): Y for q, f, Y in outs}
    res["outputs_equal"] = bool(all(torch.equal(ys[(q, 0)], ys[(q, 1)]) for q in range(n_proj)))
    res["projections"] = n_proj
    res["steps"], res["warmup"] = steps, warmup
    return res


def run_batch_sweep(ctx, mods, options):
    """Configuration 1's layer (4096 -> 4096, 32 adapters of rank 16, one-token requests, adapter ids uniform) at other
    batch sizes: the decode path up to 128 rows, the tiled GEMM split along K up to a few hundred, the tiled GEMM."""
    from workloads import make_custom
    np = mods[0]
    rng = np.random.default_rng(11)
    rows = []
    for T in (1, 16, 64, 128, 256, 512, 1024):
        wl = make_custom(seed=900 + T, dtype="bf16", K=4096, N=4096, ranks=[16] * 32, scales=[2.0] * 32,
                         req_adapter=rng.integers(0, 32, size=T), req_ntok=np.ones(T, np.int64), name=f"decode_shape_T{T}")
        r = run_projection(ctx, mods, wl, 1, 0, 100, 20, 0.0, options)
        rows.append({"rows": T, "ms_per_layer": r["ms_per_layer"], "ms_per_step": r["ms_per_step"], "kernel": r["roofline"]["kernel"]})
    # The batching model of the paper's section 4.2 (equation 2), T(b) = T0 + alpha (b - 1), fitted to the layer's own
    # times (least squares over the measured batch sizes): what a function profile for the batcher would carry.
    b = np.array([x["rows"] for x in rows], np.float64)
    t = np.array([x["ms_per_layer"] * 1e3 for x in rows], np.float64)
    A = np.stack([np.ones_like(b), b - 1.0], axis=1)
    (t0, alpha), *_ = np.linalg.lstsq(A, t, rcond=None)
    fit = {"t0_us": round(float(t0), 3), "alpha_us_per_request": round(float(alpha), 5),
           "max_rel_err": round(float(np.abs(A @ np.array([t0, alpha]) - t).max() / t.max()), 4),
           "model": "T(b) = t0 + alpha (b - 1), one-token requests, one layer"}
    return {"rows": rows, "batching_model_fit": fit}


def run_adapter_heavy_decode(ctx, mods, options):
    """Beside the benchmark's configurations: configuration 4's layer (5120 -> 13824, adapters of rank 128) on a
    decode-sized batch -- 64 one-token requests, each on an adapter of its own (the many-functions regime of the paper
    at decode time).  HBM-bound: the figure of merit is whole_call.frac_of_hbm_peak."""
    from workloads import make_custom
    np = mods[0]
    T = 64
    wl = make_custom(seed=4242, dtype="bf16", K=5120, N=13824, ranks=[128] * T, scales=[0.5] * T, req_adapter=np.arange(T),
                     req_ntok=np.ones(T, np.int64), name="adapter_heavy_decode_64x_rank128")
    r = run_projection(ctx, mods, wl, 4, 0, 60, 15, 2.0, options)
    return {k: r[k] for k in ("config", "ms_per_step", "ms_per_layer", "kernel_us", "whole_call", "adapter_path", "parity_max_err_over_rms",
                              "cpu_baseline")}


def run_library_gemm(ctx, mods):
    """Context for the base product's figures (--library-gemm, not part of the default run): the plain GEMM of the
    vendor library (torch.nn.functional.linear, bf16, random operands of the workloads' scale) and this library's
    lora_linear without an adapter table, one after the other on the same box, at the base shapes of configurations
    2, 3 and 4.  The vendor GEMM is not used anywhere else."""
    np, torch, B, rt = mods
    dev = ctx.device
    rows = []
    for name, T, K, N in (("c2 up_proj", 7539, 4096, 11008), ("c3 q_proj", 1216, 4096, 4096), ("c3 q/k/v", 1216, 4096, 12288),
                          ("c3 gate/up", 1216, 4096, 22016), ("c3 down_proj", 1216, 11008, 4096), ("c4 up_proj", 2048, 5120, 13824)):
        g = torch.Generator(device=dev).manual_seed(T + K + N)
        X = torch.randn((T, K), device=dev, generator=g).to(torch.bfloat16)
        W = (torch.randn((N, K), device=dev, generator=g) * 0.02).to(torch.bfloat16)
        Y = torch.empty((T, N), dtype=torch.bfloat16, device=dev)
        pl = rt.plan(ctx, np.full(1, -1, np.int32), np.full(1, T, np.int32), np.full(1, 8, np.int32), 8)
        ws = rt.workspace(T, K, N, 8, torch.bfloat16, dev)
        iters = 40
        t_lib = _timed(torch, lambda i: torch.nn.functional.linear(X, W), iters + 10)  # (warm-up)
        t_lib = _timed(torch, lambda i: torch.nn.functional.linear(X, W), iters)
        t_own = _timed(torch, lambda i: rt.linear(ctx, pl, X, W, None, Y=Y, ws=ws), iters + 10)
        t_own = _timed(torch, lambda i: rt.linear(ctx, pl, X, W, None, Y=Y, ws=ws), iters)
        ref = torch.nn.functional.linear(X, W).float()
        err = float((Y.float() - ref).abs().max() / ref.pow(2).mean().sqrt())
        fl = 2.0 * T * K * N
        rows.append({"shape": name, "T": T, "K": K, "N": N, "vendor_gemm_us": round(t_lib * 1e6, 1), "vendor_gemm_tflops": round(fl / t_lib / 1e12, 1),
                     "lora_linear_no_adapters_us": round(t_own * 1e6, 1), "lora_linear_no_adapters_tflops": round(fl / t_own / 1e12, 1),
                     "kernel": B.lora_gemm_kernel_name(ctx.handle, T, K, N, 1), "max_abs_diff_over_rms": err})
    return rows


def run_schedulers(np):
    """Decision latency of the two host-side schedulers at the scale of the paper's deployment (hundreds of functions
    on a GPU; configuration 4's pool of 512 adapters): microseconds per call, single host thread."""
    from paper_2505_14468_amd import sched as S
    rng = np.random.default_rng(0)
    n_fn = 256
    bat = S.Batcher([dict(t0_ms=500.0, alpha_ms=100.0, slo_ms=2500.0, adapter=i) for i in range(n_fn)])
    now, polls, dispatched = 0.0, 0, 0
    t0 = time.perf_counter()
    for k in range(20000):
        now += 0.5
        bat.submit(int(rng.integers(0, n_fn)), 16, now)
        if k % 8 == 7:
            got, _, _, _ = bat.poll(now, 1, max_batches=8, max_requests=512)
            dispatched += sum(b["n"] for b in got)
            polls += 1
    dt = time.perf_counter() - t0
    arts = [dict(function=a, kind=2, share_id=0, pinned=int(a < 16), bytes=float(2 * 128 * (5120 + 13824)),
                 value=float(rng.integers(1, 1000))) for a in range(512)]
    arr = S.artifacts_array(arts)  # (marshalled once: the figures below are the library's decision time)
    t1 = time.perf_counter()
    for _ in range(50):
        place, _ = S.lora_preload_greedy(arr, 0.0, 200 * arts[0]["bytes"])
    t_pre = (time.perf_counter() - t1) / 50
    on_gpu = np.array([int(m & 2 != 0) for m in place], np.uint8)
    t2 = time.perf_counter()
    for _ in range(50):
        S.lora_offload_greedy(arr, on_gpu, 8 * arts[0]["bytes"])
    t_off = (time.perf_counter() - t2) / 50
    return {"batcher": {"functions": n_fn, "us_per_submit_and_poll_cycle_of_8_requests": round(dt / polls * 1e6, 2),
                        "requests_dispatched": dispatched, "note": "includes the Python binding's marshalling"},
            "preload_greedy_512_adapters_us": round(t_pre * 1e6, 1), "offload_greedy_512_adapters_us": round(t_off * 1e6, 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100, help="timed steps of the headline configuration")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=-1,
                    help="run ONE workload (index into BASELINE.json configs) and print its line; default: all five")
    ap.add_argument("--proj", type=int, default=0,
                    help="with --config: projection of a multi-projection workload (config 3); -1 = all of them in one step, with one plan")
    ap.add_argument("--fuse", action="store_true",
                    help="with --proj -1: q/k/v and gate/up share their activations and go through lora_linear_multi")
    ap.add_argument("--layers", type=int, default=1, help="with --proj -1: repeat the layer's calls this many times on one plan")
    ap.add_argument("--same-adapter", type=int, default=0, metavar="ROWS",
                    help="instead of --config: ROWS single-token requests on ONE adapter at config 1's shape "
                         "(one function's own batch, the regime of the paper's section 6)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--option", action="append", default=[], help="tuning override name=value (lora_ctx_set_option)")
    ap.add_argument("--library-gemm", action="store_true",
                    help="time the vendor library's plain bf16 GEMM and lora_linear without adapters at the base shapes of configurations 2-4 and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 256 MiB device copy kernel 5 times and exit (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU (the layer shards by requests, one library instance "
                         "per GPU, no exchange); run with --gpus 1\n")
        sys.exit(2)

    import numpy as np
    import torch
    if args.calibrate_copy:
        n = 256 << 20
        src = torch.ones(n // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read_per_launch": n, "bytes_written_per_launch": n, "launches": 5}))
        return
    from paper_2505_14468_amd import binding as B
    from paper_2505_14468_amd import runtime as rt
    from workloads import make_workload, same_adapter_decode
    mods = (np, torch, B, rt)
    ctx = rt.Context(0)
    options = [(o.split("=")[0], int(o.split("=")[1])) for o in args.option]
    cpu_s = 0.0 if args.no_cpu_baseline else 4.0
    if args.library_gemm:
        print(json.dumps({"library_gemm_reference": run_library_gemm(ctx, mods), "dtype": "bf16", "data": "synthetic"}))
        ctx.close()
        return
    common = {"metric": METRIC, "n_gpus": 1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic"}

    if args.same_adapter > 0 or args.config >= 0:  # one workload alone
        wl = same_adapter_decode(args.same_adapter) if args.same_adapter > 0 else make_workload(args.config)
        for name, val in options:
            ctx.set_option(name, val)
        if args.proj < 0:
            r = run_layer(ctx, mods, wl, args.steps, args.warmup, args.fuse, args.layers)
            out = dict(common, value=r["tflops"], unit="TFLOP/s", steps=args.steps, warmup=args.warmup, ms_per_step=r["ms_per_step"],
                       dtype=wl.dtype, config={"workload": f"{wl.name}:all_projections", "tokens": wl.T, "step": r["step"]},
                       roofline=None, cpu_baseline=None)
        else:
            r = run_projection(ctx, mods, wl, args.config if args.same_adapter == 0 else 1, args.proj, args.steps, args.warmup,
                               cpu_s * 2)
            out = dict(common, **r)
        print(json.dumps(out))
        ctx.close()
        return

    # ---- the default run: every configuration, headline = configuration 2 --------------------------------------
    per_config = []
    t_start = time.perf_counter()
    for idx in range(5):
        wl = make_workload(idx)
        if idx == HEADLINE:
            steps, warmup = args.steps, args.warmup
        else:
            steps, warmup = {0: (200, 40), 1: (400, 40), 3: (60, 15), 4: (60, 15)}[idx]
        if idx != 3:
            r = run_projection(ctx, mods, wl, idx, 0, steps, warmup, cpu_s, options)
            if idx == 1:
                r["three_projections_of_the_same_activations"] = run_fused_copies(ctx, mods, wl, 3, 200, 40)
            per_config.append(dict(index=idx, **r))
            sys.stderr.write(f"bench: config {idx} done at {time.perf_counter() - t_start:.0f} s\n")
            continue
        projs = []
        for p in range(len(wl.projections)):  # the oracle's leg on the first projection only (the others have the same shape classes)
            r = run_projection(ctx, mods, wl, idx, p, steps, warmup, cpu_s if p == 0 else 0.0, options)
            projs.append(r)
            sys.stderr.write(f"bench: config 3 projection {p} done at {time.perf_counter() - t_start:.0f} s\n")
        layer = run_layer(ctx, mods, wl, 30, 8, fuse=False)
        layer_fused = run_layer(ctx, mods, wl, 30, 8, fuse=True)
        model = run_layer(ctx, mods, wl, 3, 1, fuse=True, n_layers=32)
        tot_flops = sum(wl.useful_flops(q) for q in range(len(wl.projections)))
        sum_ms = sum(r["ms_per_layer"] for r in projs)
        per_config.append({
            "index": 3, "dtype": wl.dtype, "config": {"workload": f"{wl.name}: seven projections", "tokens": wl.T, "requests": wl.n_req},
            "ms_per_layer_sum_of_seven": round(sum_ms, 5), "value": round(tot_flops / (sum_ms * 1e-3) / 1e12, 3), "unit": "TFLOP/s",
            "projections": projs, "decoder_layer_one_plan": layer, "decoder_layer_one_plan_fused_qkv_gateup": layer_fused,
            "model_32_layers_one_plan_fused": model,
            "roofline": projs[0]["roofline"], "cpu_baseline": projs[0]["cpu_baseline"],
            "parity_max_err_over_rms": projs[0]["parity_max_err_over_rms"]})
        sys.stderr.write(f"bench: config 3 done at {time.perf_counter() - t_start:.0f} s\n")
    head = per_config[HEADLINE]
    out = dict(common)
    for k in ("value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config", "roofline", "cpu_baseline", "ms_per_layer",
              "ms_per_step_plan_amortised", "kernel_us", "whole_call", "adapter_path", "parity_max_err_over_rms"):
        out[k] = head[k]
    out["per_config"] = per_config
    out["batch_size_sweep_config1_shape"] = run_batch_sweep(ctx, mods, options)
    out["adapter_heavy_decode"] = run_adapter_heavy_decode(ctx, mods, options)
    out["schedulers"] = run_schedulers(np)
    out["targets"] = {"prefill (configs 2, 3)": ">= 0.60 of bf16 MFMA peak", "decode / adapter-heavy (configs 1, 4)": ">= 0.70 of HBM peak (whole_call.frac_of_hbm_peak)"}
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
