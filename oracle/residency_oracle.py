"""Plain, slow reference of the greedy value-density residency policy: pre-loading (paper section 4.1,
equation 1) and offloading (section 4.3, equations 6-7).  TEST INFRASTRUCTURE ONLY; shares no code with the C++
behind include/lora_sched.h.  Also holds exhaustive optimal solvers for tiny instances, used to pin the greedy.

Artifacts: dicts with function, kind (0 library, 1 backbone, 2 adapter, 3 kernel), share_id, pinned, bytes, value.
Backbones with the same share_id are ONE object (sized and placed once; the values of its functions add up).
Places: 1 = container, 2 = GPU.  Libraries: container only; kernels: GPU only; backbones, adapters: either.
Precedence (section 4.1: "models require libraries first, and CUDA kernels require models on GPU first";
backbone-adapter coupling): a backbone or adapter (either place) needs its function's library in the container
(a shared backbone: of at least one of its functions; a function without a library artifact needs none); an adapter
on the GPU needs its function's backbone on the GPU; a kernel needs its function's backbone and adapter on the GPU.
"""
from __future__ import annotations

import itertools

LIB, BACKBONE, ADAPTER, KERNEL = 0, 1, 2, 3
CONTAINER, GPU = 1, 2


def _objects(arts):
    """Objects = artifacts with shared backbones merged: list of dict(members, kind, bytes, value, first)."""
    objs, by_share = [], {}
    for idx, a in enumerate(arts):
        if a["kind"] == BACKBONE:
            key = a["share_id"]
            if key in by_share:
                o = objs[by_share[key]]
                o["members"].append(idx)
                o["value"] += a["value"]
                continue
            by_share[key] = len(objs)
        objs.append(dict(members=[idx], kind=a["kind"], bytes=a["bytes"], value=a["value"], first=idx))
    return objs


def _obj_of(objs, n):
    of = [None] * n
    for k, o in enumerate(objs):
        for m in o["members"]:
            of[m] = k
    return of


def _fn_index(arts):
    """function -> {kind: artifact index} (one artifact per kind and function)."""
    fn = {}
    for idx, a in enumerate(arts):
        fn.setdefault(a["function"], {})[a["kind"]] = idx
    return fn


def _allowed_places(kind):
    return {LIB: (CONTAINER,), KERNEL: (GPU,)}.get(kind, (CONTAINER, GPU))


def _feasible(arts, objs, of, fn, placed, k, place):
    """May object k go to `place` given the set `placed` of (object, place) pairs?"""
    o = objs[k]
    if (k, place) in placed or place not in _allowed_places(o["kind"]):
        return False
    fns = [arts[m]["function"] for m in o["members"]]
    if o["kind"] in (BACKBONE, ADAPTER):
        ok = False
        for f in fns:
            lib = fn[f].get(LIB)
            if lib is None or (of[lib], CONTAINER) in placed:
                ok = True
        if not ok:
            return False
    if place == GPU and o["kind"] == ADAPTER:
        bb = fn[fns[0]].get(BACKBONE)
        if bb is not None and (of[bb], GPU) not in placed:
            return False
    if o["kind"] == KERNEL:
        for need in (BACKBONE, ADAPTER):
            dep = fn[fns[0]].get(need)
            if dep is not None and (of[dep], GPU) not in placed:
                return False
    return True


def preload_greedy(arts, container_bytes, gpu_bytes):
    """Returns (mask per artifact: bit 0 container, bit 1 GPU; objective value of equation 1)."""
    objs = _objects(arts)
    of = _obj_of(objs, len(arts))
    fn = _fn_index(arts)
    cands = [(k, pl) for k, o in enumerate(objs) for pl in _allowed_places(o["kind"])]
    cands.sort(key=lambda c: (-(objs[c[0]]["value"] / objs[c[0]]["bytes"]), objs[c[0]]["first"], c[1]))
    placed, used = set(), {CONTAINER: 0.0, GPU: 0.0}
    cap = {CONTAINER: container_bytes, GPU: gpu_bytes}
    progress = True
    while progress:
        progress = False
        for k, pl in cands:
            if used[pl] + objs[k]["bytes"] <= cap[pl] and _feasible(arts, objs, of, fn, placed, k, pl):
                placed.add((k, pl))
                used[pl] += objs[k]["bytes"]
                progress = True
                break
    return _masks(arts, objs, placed), sum(objs[k]["value"] for k, _ in placed)


def _masks(arts, objs, placed):
    mask = [0] * len(arts)
    for k, pl in placed:
        for m in objs[k]["members"]:
            mask[m] |= 1 if pl == CONTAINER else 2
    return mask


def preload_optimal(arts, container_bytes, gpu_bytes):
    """Exhaustive maximum of equation 1 over all constraint-respecting placements (tiny instances only)."""
    objs = _objects(arts)
    of = _obj_of(objs, len(arts))
    fn = _fn_index(arts)
    cands = [(k, pl) for k, o in enumerate(objs) for pl in _allowed_places(o["kind"])]
    best = 0.0
    for r in range(len(cands) + 1):
        for sub in itertools.combinations(cands, r):
            S = set(sub)
            if sum(objs[k]["bytes"] for k, pl in S if pl == CONTAINER) > container_bytes:
                continue
            if sum(objs[k]["bytes"] for k, pl in S if pl == GPU) > gpu_bytes:
                continue
            if all(_feasible(arts, objs, of, fn, S - {c}, c[0], c[1]) for c in S):
                best = max(best, sum(objs[k]["value"] for k, _ in S))
    return best


def _gpu_state(arts, on_gpu):
    objs = _objects(arts)
    of = _obj_of(objs, len(arts))
    fn = _fn_index(arts)
    here = [any(on_gpu[m] for m in o["members"]) and o["kind"] != LIB for o in objs]
    pinned = [any(arts[m]["pinned"] for m in o["members"]) for o in objs]
    # dependents[k]: objects on the GPU that need k there
    dependents = [set() for _ in objs]
    for f, kinds in fn.items():
        bb, ad, ke = kinds.get(BACKBONE), kinds.get(ADAPTER), kinds.get(KERNEL)
        if bb is not None:
            for d in (ad, ke):
                if d is not None and here[of[d]]:
                    dependents[of[bb]].add(of[d])
        if ad is not None and ke is not None and here[of[ke]]:
            dependents[of[ad]].add(of[ke])
    return objs, here, pinned, dependents


def offload_greedy(arts, on_gpu, need_bytes):
    """Returns (evict flag per artifact, bytes freed, value lost, enough: freed >= need_bytes)."""
    objs, here, pinned, dependents = _gpu_state(arts, on_gpu)
    chosen, freed, lost = set(), 0.0, 0.0
    while freed < need_bytes:
        cand = [k for k, o in enumerate(objs) if here[k] and not pinned[k] and k not in chosen and dependents[k] <= chosen]
        if not cand:
            break
        k = min(cand, key=lambda k: (objs[k]["value"] / objs[k]["bytes"], -objs[k]["first"]))
        chosen.add(k)
        freed += objs[k]["bytes"]
        lost += objs[k]["value"]
    evict = [0] * len(arts)
    for k in chosen:
        for m in objs[k]["members"]:
            if on_gpu[m]:
                evict[m] = 1
    return evict, freed, lost, freed >= need_bytes


def offload_optimal(arts, on_gpu, need_bytes):
    """Exhaustive minimum of equation 7 subject to equation 6 and the dependency order; None if infeasible."""
    objs, here, pinned, dependents = _gpu_state(arts, on_gpu)
    pool = [k for k in range(len(objs)) if here[k] and not pinned[k]]
    best = None
    for r in range(len(pool) + 1):
        for sub in itertools.combinations(pool, r):
            S = set(sub)
            if any(not dependents[k] <= S for k in S):
                continue
            if sum(objs[k]["bytes"] for k in S) >= need_bytes:
                v = sum(objs[k]["value"] for k in S)
                best = v if best is None else min(best, v)
    return best
