#!/usr/bin/env python3
"""Benchmark of the multi-LoRA batched linear layer on one MI355X.

One "step" = the whole hot path over one batch: the device-side segment builder
(``lora_plan_device`` on request arrays already in HBM) followed by ``lora_linear``
(segmented shrink + base GEMM with the expand fused before the single store of Y).
Consecutive steps rotate over several independent weight sets (backbone + adapters +
activations), as the layers of a model would, so that decode-sized runs stream their
weights from HBM instead of re-reading one set from the caches.

Prints ONE JSON line: metric, value (whole-step throughput), the roofline of the dominant kernel from live HIP event
timings, per-kernel microseconds, and the CPU oracle timed beside it.  Inputs are seeded and
synthetic (``workloads``), shaped like LoRA-on-Llama2 serving; nothing is read from disk
except the optional ``profiles/hbm_traffic.json`` produced from rocprofv3 counter runs.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 matrix, published
HBM_BOUND = {0: False, 1: True, 2: False, 3: False, 4: True}


def _layer_variant(wl, layer):
    """Same batch and shapes, independent weight / activation values for layer > 0."""
    if layer == 0:
        return wl
    import copy
    w2 = copy.copy(wl)
    w2.seed = wl.seed + 7919 * layer
    w2._cache = {}
    return w2


def _whole_layer(args, wl, B, rt, torch, np):
    """--proj -1: one step = one plan + ``lora_linear`` for every projection of the workload (config 3: the seven
    projections of a decoder layer, each with its own X, as the workload defines them); a side measurement
    with per-projection times, not the line the default run prints."""
    ctx = rt.Context(0)
    for opt in args.option:
        name, val = opt.split("=")
        ctx.set_option(name, int(val))
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
        X, W0, table = rt.upload_workload(wl, q, dev)
        Y = torch.empty((T, pr.N), dtype=tdtype, device=dev)
        ws = rt.workspace(T, pr.K, pr.N, r_max, tdtype, dev)
        keep.append((X, W0, table, Y, ws))
        descs.append(rt.linear_desc(plan0, X, W0, Y, table, ws))
    h, stream = ctx.handle, int(torch.cuda.current_stream().cuda_stream)
    ra_p, rn_p, rk_p, pb_p = req_adapter.data_ptr(), req_ntok.data_ptr(), ranks.data_ptr(), plan_buf.data_ptr()

    # --fuse: projections that read the same activations in a decoder layer (q, k, v; gate, up) go through one
    # lora_linear_multi call each, on the first one's X
    groups = [[q] for q in range(len(descs))]
    if args.fuse:
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
        for g in groups:
            if len(g) == 1:
                B.lora_linear(h, plan, descs[g[0]], stream)
            else:
                B.lora_linear_multi(h, plan, [descs[q] for q in g], stream)

    def timed(fn, k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(k):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / k

    for i in range(args.warmup):
        step(i)
    status, n_seg = plan0.status(ctx)
    assert status == 0, f"plan status {status}"
    sec = timed(step, args.steps)
    per_proj = {pr.name: round(timed(lambda i, d=d: B.lora_linear(h, plan0.struct, d, stream), max(10, args.steps // 4)) * 1e3, 5)
                for pr, d in zip(wl.projections, descs)}
    flops = sum(wl.useful_flops(q) for q in range(len(wl.projections)))
    print(json.dumps({
        "metric": "multi-LoRA linear TFLOP/s + adapter-path GB/s (roofline %), ms/layer", "value": round(flops / sec / 1e12, 3),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}:all_projections", "tokens": T, "requests": wl.n_req, "adapters_resident": wl.n_adapters,
                   "segments": n_seg, "rank_max": r_max,
                   "step": "lora_plan_device + " + " + ".join("lora_linear" if len(g) == 1 else f"lora_linear_multi({len(g)})" for g in groups)},
        "ms_per_layer_by_projection": per_proj, "roofline": None, "cpu_baseline": None}))
    ctx.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=1, help="workload: index into BASELINE.json configs (default 1)")
    ap.add_argument("--proj", type=int, default=0,
                    help="projection of a multi-projection workload (config 3); -1 = all of them in one step, with one plan")
    ap.add_argument("--fuse", action="store_true",
                    help="with --proj -1: q/k/v and gate/up share their activations and go through lora_linear_multi")
    ap.add_argument("--same-adapter", type=int, default=0, metavar="ROWS",
                    help="instead of --config: ROWS single-token requests on ONE adapter at config 1's shape "
                         "(one function's own batch, the regime of the paper's section 6)")
    ap.add_argument("--weight-sets", type=int, default=0, help="rotating weight sets (0 = sized to exceed the caches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true",
                    help="skip comparing the rows the cpu_baseline leg computes with the GPU's")
    ap.add_argument("--option", action="append", default=[], help="tuning override name=value (lora_ctx_set_option)")
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
    from workloads import make_workload, same_adapter_decode, to_f64

    wl = same_adapter_decode(args.same_adapter) if args.same_adapter > 0 else make_workload(args.config)
    if args.proj < 0:
        _whole_layer(args, wl, B, rt, torch, np)
        return
    p = args.proj
    pr = wl.projections[p]
    K, N, T = pr.K, pr.N, wl.T
    ctx = rt.Context(0)
    for opt in args.option:
        name, val = opt.split("=")
        ctx.set_option(name, int(val))
    dev = ctx.device
    es = 2 if wl.dtype == "bf16" else 4
    tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32

    # ---- weight sets --------------------------------------------------------------------------
    used = wl.used_adapters()
    r_used = int(wl.ranks[used].astype(np.int64).sum())
    set_bytes = es * (K * N + T * K + T * N + int(wl.ranks.astype(np.int64).sum()) * (K + N))
    n_sets = args.weight_sets or max(1, min(16, int(np.ceil(1.0e9 / set_bytes))))
    sets = []
    for layer in range(n_sets):
        w = _layer_variant(wl, layer)
        X, W0, table = rt.upload_workload(w, p, dev)
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

    h = ctx.handle
    ra_p, rn_p, rk_p, pb_p = req_adapter.data_ptr(), req_ntok.data_ptr(), ranks.data_ptr(), plan_buf.data_ptr()

    def step(i):
        plan = B.lora_plan_device(h, ra_p, rn_p, wl.n_req, rk_p, wl.n_adapters, r_max, T, pb_p, plan_bytes, stream)
        B.lora_linear(h, plan, descs[i % n_sets], stream)

    def timed(fn, k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(k):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / k

    for i in range(args.warmup):
        step(i)
    status, n_seg = plan0.status(ctx)
    assert status == 0, f"plan status {status}"

    # ---- the timed region: K whole steps ------------------------------------------------------------
    sec_per_step = timed(step, args.steps)

    # ---- the same K steps again with every kernel bracketed by its own HIP event pair (the events
    #      cost host time per launch, so this pass is not the one `value` comes from) -----------------
    B.lora_profile_begin(h, args.steps)
    sec_profiled = timed(step, args.steps)
    prof = B.lora_profile_end(h, stream)

    # ---- side measurements (not part of `value`) ----------------------------------------------------
    k2 = max(20, args.steps // 4)
    sec_layer = timed(lambda i: B.lora_linear(h, plan0.struct, descs[i % n_sets], stream), k2)
    B.lora_profile_begin(h, k2)
    timed(lambda i: B.lora_gemm_expand(h, plan0.struct, descs_base[i % n_sets], stream), k2)
    base_gemm_us = B.lora_profile_end(h, stream)["gemm_expand"][0]
    sec_hot = timed(lambda i: B.lora_linear(h, plan0.struct, descs[0], stream), k2)  # one weight set: cache-resident

    flops = wl.useful_flops(p)
    gemm_us, shrink_us = prof["gemm_expand"][0], prof["shrink"][0]
    plan_us = prof["plan_segments"][0] + prof["plan_fill"][0]
    # algorithmic bytes of the fused GEMM kernel: X, W0, Y, every used B_a and V, each once
    v_bytes = es * int(sum(int(wl.ranks[a]) * int(n) for a, n in zip(*np.unique(wl.row_adapter()[wl.row_adapter() >= 0], return_counts=True))))
    gemm_bytes = es * (T * K + K * N + T * N + r_used * N) + v_bytes
    gemm_flops = 2 * T * K * N + 2 * N * v_bytes // es
    hbm_bound = T <= 256 if args.same_adapter > 0 else HBM_BOUND.get(args.config, T <= 256)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(f"{wl.name}:{pr.name}")
    if hbm_bound:
        achieved = gemm_bytes / (gemm_us * 1e-6) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBPS, 4), "traffic": traffic}
    else:
        peak = PEAK_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_F32_TFLOPS
        achieved = gemm_flops / (gemm_us * 1e-6) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 1), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(achieved / peak, 4), "traffic": traffic}
    roofline["kernel"] = "gemm_expand:" + B.lora_gemm_kernel_name(h, T, K, N, rt.dtype_code(tdtype))
    roofline["kernel_us"] = round(gemm_us, 3)
    roofline["algorithmic_bytes"] = gemm_bytes
    roofline["algorithmic_flops"] = gemm_flops

    adapter_bytes = es * (r_used * (K + N) + T * K) + 2 * v_bytes
    adapter_us = shrink_us + max(gemm_us - base_gemm_us, 0.0)

    # ---- the cpu_baseline leg: the oracle on the host cores, timed as a reported baseline; the rows it computes are
    #      also compared with the GPU's (outside the timed region).  Nothing else in this file touches the oracle. -----
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import oracle_threads, oracle_workload
        est = flops / 2.0e9  # seconds at ~2 GFLOP/s
        n_rows = T if est <= 20 else max(1, int(T * 15 / est))
        rows = None if n_rows == T else np.arange(n_rows)
        oracle_workload(wl, p, rows=np.arange(1))  # build + page in
        t0 = time.perf_counter()
        reps = 0
        while True:
            ref = oracle_workload(wl, p, rows=rows)
            reps += 1
            if time.perf_counter() - t0 > 8.0 or reps >= 50:
                break
        dt = (time.perf_counter() - t0) / reps
        frac = n_rows / T
        cpu = {"value": round(flops * frac / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle_threads(), "kind": "oracle",
               "sample": f"{n_rows} of {T} rows of the layer, {reps} repetition(s), {dt:.3f} s each"}
        if not args.no_check:
            torch.cuda.synchronize()
            plan = rt.plan_device(ctx, req_adapter, req_ntok, ranks, r_max, T, buf=plan_buf)
            X, W0, table, Y = sets[0]
            B.lora_linear(h, plan.struct, descs[0], stream)
            torch.cuda.synchronize()
            got = to_f64(rt.bits_from_tensor(Y[:n_rows]))
            rms = float(np.sqrt((ref ** 2).mean()))
            parity = float(np.abs(got - ref).max() / rms)
            tol = 2e-2 if wl.dtype == "bf16" else 1e-5
            assert parity <= tol, f"parity {parity} > {tol}"

    out = {
        "metric": "multi-LoRA linear TFLOP/s + adapter-path GB/s (roofline %), ms/layer",
        "value": round(flops / sec_per_step / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": f"{wl.name}:{pr.name}", "d_in": K, "d_out": N, "tokens": T, "requests": wl.n_req,
                   "adapters_resident": wl.n_adapters, "adapters_used": int(used.size), "segments": n_seg,
                   "rank_max": r_max, "weight_sets": n_sets, "step": "lora_plan_device + lora_linear"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "ms_per_layer": round(sec_layer * 1e3, 5),
        "ms_per_layer_cached_weights": round(sec_hot * 1e3, 5),
        "ms_per_step_profiled": round(sec_profiled * 1e3, 5),
        "layer_tflops": round(flops / sec_layer / 1e12, 3),
        "layer_gbps": round(wl.algorithmic_bytes(p) / sec_layer / 1e9, 1),
        "kernel_us": {"plan": round(plan_us, 3), "shrink": round(shrink_us, 3), "gemm_expand": round(gemm_us, 3),
                      "gemm_base_only": round(base_gemm_us, 3)},
        "adapter_path": {"bytes": adapter_bytes, "us": round(adapter_us, 3),
                         "gbps": round(adapter_bytes / max(adapter_us, 1e-3) / 1e3, 1),
                         "frac_of_hbm_peak": round(adapter_bytes / max(adapter_us, 1e-3) / 1e3 / PEAK_HBM_GBPS, 4)},
        "parity_max_err_over_rms": parity,
    }
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
