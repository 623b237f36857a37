"""ctypes binding of include/lora_sched.h: the adaptive batching scheduler and the greedy residency policy (host code
in the same shared library as the layer).  Same names as the C ABI; argument marshalling only."""
from __future__ import annotations

import ctypes as C
import math
from typing import List, Sequence

import numpy as np

from .binding import lib as _layer_lib

LORA_SCHED_OK = 0
LORA_SCHED_ERR_INVALID_ARG = -1
LORA_SCHED_ERR_CAPACITY = -2

EXPORTS = [
    "lora_batcher_create", "lora_batcher_destroy", "lora_batcher_max_batch", "lora_batcher_set_batch_size",
    "lora_batcher_batch_size", "lora_batcher_delay", "lora_batcher_submit", "lora_batcher_poll",
    "lora_batcher_next_event", "lora_batcher_queued", "lora_preload_greedy", "lora_offload_greedy", "lora_sched_strerror",
]


class lora_function_profile(C.Structure):
    _fields_ = [("t0_ms", C.c_double), ("alpha_ms", C.c_double), ("slo_ms", C.c_double), ("adapter", C.c_int32),
                ("max_batch", C.c_int32)]


class lora_batch(C.Structure):
    _fields_ = [("function", C.c_int32), ("adapter", C.c_int32), ("n", C.c_int32), ("first", C.c_int32),
                ("wait_ms", C.c_double), ("margin_ms", C.c_double), ("t_batch_ms", C.c_double)]


class lora_artifact(C.Structure):
    _fields_ = [("function", C.c_int32), ("kind", C.c_int32), ("share_id", C.c_int32), ("pinned", C.c_int32),
                ("bytes", C.c_double), ("value", C.c_double)]


class SchedError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().lora_sched_strerror(status).decode()} [{status}]")


_ready = False


def lib():
    global _ready
    L = _layer_lib()
    if not _ready:
        i32p, f64p = C.POINTER(C.c_int32), C.POINTER(C.c_double)
        L.lora_batcher_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(lora_function_profile), C.c_int32]
        L.lora_batcher_destroy.argtypes = [C.c_void_p]
        L.lora_batcher_max_batch.argtypes = [C.c_void_p, C.c_int32, i32p]
        L.lora_batcher_set_batch_size.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.lora_batcher_batch_size.argtypes = [C.c_void_p, C.c_int32, i32p]
        L.lora_batcher_delay.argtypes = [C.c_void_p, C.c_int32, f64p]
        L.lora_batcher_submit.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.POINTER(C.c_int64)]
        L.lora_batcher_poll.argtypes = [C.c_void_p, C.c_double, C.c_int32, C.c_int32, C.POINTER(lora_batch), C.c_int32,
                                        C.c_void_p, C.c_void_p, C.c_void_p, i32p, i32p]
        L.lora_batcher_next_event.argtypes = [C.c_void_p, C.c_double, C.c_int32, f64p]
        L.lora_batcher_queued.argtypes = [C.c_void_p, C.c_int32, i32p]
        L.lora_preload_greedy.argtypes = [C.POINTER(lora_artifact), C.c_int32, C.c_double, C.c_double, C.c_void_p, f64p]
        L.lora_offload_greedy.argtypes = [C.POINTER(lora_artifact), C.c_int32, C.c_void_p, C.c_double, C.c_void_p, f64p, f64p]
        L.lora_sched_strerror.argtypes = [C.c_int]
        L.lora_sched_strerror.restype = C.c_char_p
        _ready = True
    return L


def _check(st: int, where: str) -> None:
    if st != LORA_SCHED_OK:
        raise SchedError(st, where)


class Batcher:
    """lora_batcher: per-function fill-or-expire queues, dispatch in order of deadline margin."""

    def __init__(self, profiles: Sequence[dict]):
        arr = (lora_function_profile * max(len(profiles), 1))()
        for i, p in enumerate(profiles):
            arr[i] = lora_function_profile(float(p["t0_ms"]), float(p["alpha_ms"]), float(p["slo_ms"]),
                                           int(p.get("adapter", -1)), int(p.get("max_batch", 0)))
        h = C.c_void_p()
        _check(lib().lora_batcher_create(C.byref(h), arr, len(profiles)), "lora_batcher_create")
        self.h, self.n_functions = h, len(profiles)

    def close(self):
        if self.h:
            lib().lora_batcher_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _int(self, fn, i):
        out = C.c_int32()
        _check(fn(self.h, int(i), C.byref(out)), "lora_batcher")
        return int(out.value)

    def max_batch(self, i):
        return self._int(lib().lora_batcher_max_batch, i)

    def batch_size(self, i):
        return self._int(lib().lora_batcher_batch_size, i)

    def queued(self, i):
        return self._int(lib().lora_batcher_queued, i)

    def set_batch_size(self, i, n, raw=False):
        st = lib().lora_batcher_set_batch_size(self.h, int(i), int(n))
        if raw:
            return st
        _check(st, "lora_batcher_set_batch_size")

    def delay(self, i):
        out = C.c_double()
        _check(lib().lora_batcher_delay(self.h, int(i), C.byref(out)), "lora_batcher_delay")
        return float(out.value)

    def submit(self, i, ntok, now, raw=False):
        rid = C.c_int64()
        st = lib().lora_batcher_submit(self.h, int(i), int(ntok), float(now), C.byref(rid))
        if raw:
            return st
        _check(st, "lora_batcher_submit")
        return int(rid.value)

    def poll(self, now, running, max_batches=64, max_requests=4096, raw=False):
        """Returns (batches, req_adapter, req_ntok, request_ids): the last three are the arrays of the multi-LoRA batch
        made of all dispatched batches -- req_adapter / req_ntok are what lora_plan() takes."""
        bs = (lora_batch * max(max_batches, 1))()
        ids = np.zeros(max(max_requests, 1), np.int64)
        ra = np.zeros(max(max_requests, 1), np.int32)
        rn = np.zeros(max(max_requests, 1), np.int32)
        nb, nr = C.c_int32(), C.c_int32()
        st = lib().lora_batcher_poll(self.h, float(now), int(running), int(max_batches), bs, int(max_requests),
                                     ids.ctypes.data_as(C.c_void_p), ra.ctypes.data_as(C.c_void_p),
                                     rn.ctypes.data_as(C.c_void_p), C.byref(nb), C.byref(nr))
        if raw:
            return st
        _check(st, "lora_batcher_poll")
        out = []
        for k in range(nb.value):
            b = bs[k]
            out.append(dict(function=b.function, adapter=b.adapter, n=b.n, first=b.first, wait_ms=b.wait_ms,
                            margin_ms=b.margin_ms, t_batch_ms=b.t_batch_ms,
                            request_ids=ids[b.first:b.first + b.n].tolist(), ntok=rn[b.first:b.first + b.n].tolist()))
        return out, ra[:nr.value].copy(), rn[:nr.value].copy(), ids[:nr.value].copy()

    def next_event(self, now, running):
        out = C.c_double()
        _check(lib().lora_batcher_next_event(self.h, float(now), int(running), C.byref(out)), "lora_batcher_next_event")
        return math.inf if out.value == math.inf else float(out.value)


def artifacts_array(arts):
    """A ctypes array of lora_artifact from a sequence of dicts (or such an array, passed through)."""
    if isinstance(arts, C.Array):
        return arts
    arr = (lora_artifact * max(len(arts), 1))()
    for i, a in enumerate(arts):
        arr[i] = lora_artifact(int(a["function"]), int(a["kind"]), int(a.get("share_id", 0)), int(a.get("pinned", 0)),
                               float(a["bytes"]), float(a["value"]))
    return arr


def lora_preload_greedy(arts: Sequence[dict], container_bytes: float, gpu_bytes: float, raw: bool = False):
    """Returns (mask per artifact: bit 0 container, bit 1 GPU; objective value)."""
    place = np.zeros(max(len(arts), 1), np.uint8)
    value = C.c_double()
    st = lib().lora_preload_greedy(artifacts_array(arts), len(arts), float(container_bytes), float(gpu_bytes),
                                   place.ctypes.data_as(C.c_void_p), C.byref(value))
    if raw:
        return st
    _check(st, "lora_preload_greedy")
    return place[:len(arts)].tolist(), float(value.value)


def lora_offload_greedy(arts: Sequence[dict], on_gpu: Sequence[int], need_bytes: float):
    """Returns (evict flag per artifact, bytes freed, value lost, enough)."""
    flags = np.ascontiguousarray(on_gpu, np.uint8)
    if flags.size == 0:
        flags = np.zeros(1, np.uint8)
    evict = np.zeros(max(len(arts), 1), np.uint8)
    freed, lost = C.c_double(), C.c_double()
    st = lib().lora_offload_greedy(artifacts_array(arts), len(arts), flags.ctypes.data_as(C.c_void_p), float(need_bytes),
                                   evict.ctypes.data_as(C.c_void_p), C.byref(freed), C.byref(lost))
    if st not in (LORA_SCHED_OK, LORA_SCHED_ERR_CAPACITY):
        raise SchedError(st, "lora_offload_greedy")
    return evict[:len(arts)].tolist(), float(freed.value), float(lost.value), st == LORA_SCHED_OK
