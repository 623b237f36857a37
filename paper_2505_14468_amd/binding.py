"""ctypes binding of include/lora_mi355x.h: same names, argument marshalling only.

Every function takes raw addresses (ints) for device memory, exactly as the C
ABI does; ``paper_2505_14468_amd.runtime`` adds the torch plumbing (buffers,
pointer tables, current stream).  The library must have been built
(``python -m paper_2505_14468_amd.build`` or ``__graft_entry__.build()``);
loading fails loudly otherwise -- there is no other code path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "liblora_mi355x.so")

LORA_DTYPE_F32 = 0
LORA_DTYPE_BF16 = 1

LORA_OK = 0
LORA_ERR_INVALID_ARG = -1
LORA_ERR_BAD_ADAPTER_ID = -2
LORA_ERR_LENGTH_MISMATCH = -3
LORA_ERR_ADAPTER_NOT_RESIDENT = -4
LORA_ERR_RANK_TOO_LARGE = -5
LORA_ERR_WORKSPACE_TOO_SMALL = -6
LORA_ERR_ALIGNMENT = -7
LORA_ERR_SHAPE = -8
LORA_ERR_HIP = -9
LORA_ERR_PLAN = -10

EXPORTS = [
    "lora_ctx_create", "lora_ctx_destroy", "lora_ctx_set_option",
    "lora_plan_validate", "lora_plan_bytes", "lora_plan", "lora_plan_device", "lora_plan_status",
    "lora_linear_workspace_bytes", "lora_linear_workspace_bytes_preferred", "lora_shrink", "lora_gemm_expand", "lora_linear",
    "lora_linear_multi", "lora_linear_static",
    "lora_profile_begin", "lora_profile_end",
    "lora_gemm_kernel_name", "lora_strerror", "lora_last_hip_error",
    "lora_backbone_alloc", "lora_backbone_free", "lora_backbone_export", "lora_backbone_open", "lora_backbone_close",
]


class lora_adapter_table_t(C.Structure):
    _fields_ = [("n_adapters", C.c_int32), ("reserved", C.c_int32),
                ("A", C.c_void_p), ("B", C.c_void_p), ("scale", C.c_void_p)]


class lora_plan_t(C.Structure):
    _fields_ = [("T", C.c_int64), ("n_req", C.c_int32), ("n_adapters", C.c_int32), ("r_max", C.c_int32),
                ("seg_cap", C.c_int32), ("ext_cap", C.c_int32), ("magic", C.c_int32), ("unit_rows", C.c_int32),
                ("perm", C.c_void_p), ("row_seg", C.c_void_p), ("row_adapter", C.c_void_p), ("row_ext", C.c_void_p), ("seg_adapter", C.c_void_p),
                ("seg_indptr", C.c_void_p), ("seg_rank", C.c_void_p), ("seg_ext", C.c_void_p),
                ("seg_unit", C.c_void_p), ("unit_rec", C.c_void_p), ("ext_rec", C.c_void_p), ("tok_off", C.c_void_p),
                ("scalars", C.c_void_p)]


class lora_linear_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("K", C.c_int32), ("N", C.c_int32), ("flags", C.c_int32),
                ("X", C.c_void_p), ("ldx", C.c_int64), ("W0", C.c_void_p), ("ldw", C.c_int64),
                ("Y", C.c_void_p), ("ldy", C.c_int64), ("tbl", C.POINTER(lora_adapter_table_t)),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class LoraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lora_strerror(status)
        if status == LORA_ERR_HIP:
            msg += f" (hipError {lora_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


_lib = None


def lib():
    """The loaded shared library; raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2505_14468_amd.build`")
        L = C.CDLL(LIB_PATH)
        i32p = C.POINTER(C.c_int32)
        L.lora_ctx_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
        L.lora_ctx_destroy.argtypes = [C.c_void_p]
        L.lora_ctx_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int]
        L.lora_plan_validate.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                         C.c_int64, i32p, C.POINTER(C.c_int64)]
        L.lora_plan_bytes.argtypes = [C.c_int32, C.c_int64, C.c_int32, C.c_int32]
        L.lora_plan_bytes.restype = C.c_size_t
        plan_args = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
                     C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(lora_plan_t)]
        L.lora_plan.argtypes = plan_args
        L.lora_plan_device.argtypes = plan_args
        L.lora_plan_status.argtypes = [C.c_void_p, C.POINTER(lora_plan_t), C.c_void_p, i32p]
        L.lora_linear_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.lora_linear_workspace_bytes.restype = C.c_size_t
        L.lora_linear_workspace_bytes_preferred.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.lora_linear_workspace_bytes_preferred.restype = C.c_size_t
        for name in ("lora_shrink", "lora_gemm_expand", "lora_linear", "lora_linear_static"):
            getattr(L, name).argtypes = [C.c_void_p, C.POINTER(lora_plan_t), C.POINTER(lora_linear_desc), C.c_void_p]
        L.lora_linear_multi.argtypes = [C.c_void_p, C.POINTER(lora_plan_t), C.POINTER(C.POINTER(lora_linear_desc)), C.c_int32,
                                        C.c_void_p]
        L.lora_profile_begin.argtypes = [C.c_void_p, C.c_int]
        L.lora_profile_end.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double), i32p]
        L.lora_gemm_kernel_name.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32]
        L.lora_gemm_kernel_name.restype = C.c_char_p
        L.lora_backbone_alloc.argtypes = [C.c_int, C.c_size_t, C.POINTER(C.c_void_p)]
        L.lora_backbone_free.argtypes = [C.c_int, C.c_void_p]
        L.lora_backbone_export.argtypes = [C.c_int, C.c_void_p, C.c_char_p]
        L.lora_backbone_open.argtypes = [C.c_int, C.c_char_p, C.POINTER(C.c_void_p)]
        L.lora_backbone_close.argtypes = [C.c_int, C.c_void_p]
        L.lora_strerror.argtypes = [C.c_int]
        L.lora_strerror.restype = C.c_char_p
        L.lora_last_hip_error.restype = C.c_int
        _lib = L
    return _lib


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, np.int32)


def _np_ptr(a):
    return None if a is None or a.size == 0 else a.ctypes.data_as(C.c_void_p)


# ---- errors ---------------------------------------------------------------
def lora_strerror(status: int) -> str:
    return lib().lora_strerror(int(status)).decode()


def lora_last_hip_error() -> int:
    return int(lib().lora_last_hip_error())


def _check(status: int, where: str) -> None:
    if status != LORA_OK:
        raise LoraError(status, where)


# ---- context ----------------------------------------------------------------
def lora_ctx_create(device_ordinal: int = 0) -> int:
    h = C.c_void_p()
    _check(lib().lora_ctx_create(C.byref(h), int(device_ordinal)), "lora_ctx_create")
    return h.value


def lora_ctx_destroy(ctx: int) -> None:
    _check(lib().lora_ctx_destroy(C.c_void_p(ctx)), "lora_ctx_destroy")


def lora_ctx_set_option(ctx: int, name: str, value: int) -> None:
    _check(lib().lora_ctx_set_option(C.c_void_p(ctx), name.encode(), int(value)), "lora_ctx_set_option")


# ---- plan ---------------------------------------------------------------------
def lora_plan_validate(req_adapter, req_ntok, adapter_rank, r_max: int, T_expected: int, *, raw: bool = False):
    """Host-only check; returns (n_seg, ext_total), or the status code when raw=True."""
    ra, rn, rk = _i32(req_adapter), _i32(req_ntok), _i32(adapter_rank)
    n_seg, ext = C.c_int32(0), C.c_int64(0)
    st = lib().lora_plan_validate(_np_ptr(ra), _np_ptr(rn), ra.shape[0], _np_ptr(rk), rk.shape[0], int(r_max),
                                  int(T_expected), C.byref(n_seg), C.byref(ext))
    if raw:
        return st
    _check(st, "lora_plan_validate")
    return n_seg.value, ext.value


def lora_plan_bytes(n_req: int, T: int, n_adapters: int, r_max: int) -> int:
    return int(lib().lora_plan_bytes(int(n_req), int(T), int(n_adapters), int(r_max)))


def lora_plan(ctx, req_adapter, req_ntok, adapter_rank, r_max: int, T_expected: int,
              plan_buf: int, plan_buf_bytes: int, stream: int, *, raw: bool = False):
    """Host arrays in; returns a filled lora_plan_t (or the status when raw=True)."""
    ra, rn, rk = _i32(req_adapter), _i32(req_ntok), _i32(adapter_rank)
    out = lora_plan_t()
    st = lib().lora_plan(C.c_void_p(ctx), _np_ptr(ra), _np_ptr(rn), ra.shape[0], _np_ptr(rk), rk.shape[0], int(r_max),
                         int(T_expected), C.c_void_p(plan_buf), int(plan_buf_bytes), C.c_void_p(stream), C.byref(out))
    if raw:
        return st
    _check(st, "lora_plan")
    return out


def lora_plan_device(ctx, req_adapter_ptr: int, req_ntok_ptr: int, n_req: int, adapter_rank_ptr: int,
                     n_adapters: int, r_max: int, T_expected: int, plan_buf: int, plan_buf_bytes: int, stream: int):
    out = lora_plan_t()
    st = lib().lora_plan_device(C.c_void_p(ctx), C.c_void_p(req_adapter_ptr), C.c_void_p(req_ntok_ptr), int(n_req),
                                C.c_void_p(adapter_rank_ptr), int(n_adapters), int(r_max), int(T_expected),
                                C.c_void_p(plan_buf), int(plan_buf_bytes), C.c_void_p(stream), C.byref(out))
    _check(st, "lora_plan_device")
    return out


def lora_plan_status(ctx, plan: lora_plan_t, stream: int):
    """Synchronises the stream; returns (status, n_seg)."""
    n_seg = C.c_int32(0)
    st = lib().lora_plan_status(C.c_void_p(ctx), C.byref(plan), C.c_void_p(stream), C.byref(n_seg))
    return int(st), int(n_seg.value)


# ---- the layer ------------------------------------------------------------------
def lora_linear_workspace_bytes(T: int, K: int, N: int, r_max: int, dtype: int) -> int:
    return int(lib().lora_linear_workspace_bytes(int(T), int(K), int(N), int(r_max), int(dtype)))


def lora_linear_workspace_bytes_preferred(T: int, K: int, N: int, r_max: int, dtype: int) -> int:
    return int(lib().lora_linear_workspace_bytes_preferred(int(T), int(K), int(N), int(r_max), int(dtype)))


def make_adapter_table(n_adapters: int, A_ptrs: int, B_ptrs: int, scale_ptr: int) -> lora_adapter_table_t:
    return lora_adapter_table_t(int(n_adapters), 0, C.c_void_p(A_ptrs), C.c_void_p(B_ptrs), C.c_void_p(scale_ptr))


def make_linear_desc(dtype: int, K: int, N: int, X: int, ldx: int, W0: int, ldw: int, Y: int, ldy: int,
                     tbl, workspace: int, workspace_bytes: int) -> lora_linear_desc:
    d = lora_linear_desc()
    d.dtype, d.K, d.N, d.flags = int(dtype), int(K), int(N), 0
    d.X, d.ldx, d.W0, d.ldw, d.Y, d.ldy = X, int(ldx), W0, int(ldw), Y, int(ldy)
    d.tbl = C.pointer(tbl) if tbl is not None else None
    d.workspace, d.workspace_bytes = workspace, int(workspace_bytes)
    d._keep = tbl
    return d


def _stage(name: str, ctx, plan, desc, stream, raw):
    st = getattr(lib(), name)(C.c_void_p(ctx), C.byref(plan), C.byref(desc), C.c_void_p(stream))
    if raw:
        return st
    _check(st, name)
    return None


def lora_shrink(ctx, plan, desc, stream: int, *, raw: bool = False):
    return _stage("lora_shrink", ctx, plan, desc, stream, raw)


def lora_gemm_expand(ctx, plan, desc, stream: int, *, raw: bool = False):
    return _stage("lora_gemm_expand", ctx, plan, desc, stream, raw)


def lora_linear(ctx, plan, desc, stream: int, *, raw: bool = False):
    return _stage("lora_linear", ctx, plan, desc, stream, raw)


def lora_linear_static(ctx, plan, desc, stream: int, *, raw: bool = False):
    """desc.workspace must be NULL / 0: the library's static scratch is the workspace."""
    return _stage("lora_linear_static", ctx, plan, desc, stream, raw)


LORA_MAX_MULTI = 4
LORA_STATIC_SCRATCH_BYTES = 32 << 20


def lora_linear_multi(ctx, plan, descs, stream: int, *, raw: bool = False):
    """descs: a sequence of lora_linear_desc that share X, ldx, K and dtype."""
    n = len(descs)
    arr = (C.POINTER(lora_linear_desc) * max(n, 1))(*[C.pointer(d) for d in descs])
    st = lib().lora_linear_multi(C.c_void_p(ctx), C.byref(plan), arr, C.c_int32(n), C.c_void_p(stream))
    if raw:
        return st
    _check(st, "lora_linear_multi")
    return None


PROFILE_KINDS = ("plan_segments", "plan_fill", "shrink", "gemm_expand", "expand")


def lora_profile_begin(ctx, max_launches: int) -> None:
    _check(lib().lora_profile_begin(C.c_void_p(ctx), int(max_launches)), "lora_profile_begin")


def lora_profile_end(ctx, stream: int) -> dict:
    """{kind: (average microseconds, timed launches)} for every kernel kind."""
    avg = (C.c_double * len(PROFILE_KINDS))()
    cnt = (C.c_int32 * len(PROFILE_KINDS))()
    _check(lib().lora_profile_end(C.c_void_p(ctx), C.c_void_p(stream), avg, cnt), "lora_profile_end")
    return {k: (float(avg[i]), int(cnt[i])) for i, k in enumerate(PROFILE_KINDS)}


LORA_IPC_HANDLE_BYTES = 64


def lora_backbone_alloc(device_ordinal: int, nbytes: int) -> int:
    p = C.c_void_p()
    _check(lib().lora_backbone_alloc(int(device_ordinal), int(nbytes), C.byref(p)), "lora_backbone_alloc")
    return int(p.value)


def lora_backbone_free(device_ordinal: int, ptr: int) -> None:
    _check(lib().lora_backbone_free(int(device_ordinal), C.c_void_p(ptr)), "lora_backbone_free")


def lora_backbone_export(device_ordinal: int, ptr: int) -> bytes:
    buf = C.create_string_buffer(LORA_IPC_HANDLE_BYTES)
    _check(lib().lora_backbone_export(int(device_ordinal), C.c_void_p(ptr), buf), "lora_backbone_export")
    return buf.raw


def lora_backbone_open(device_ordinal: int, handle: bytes) -> int:
    assert len(handle) == LORA_IPC_HANDLE_BYTES
    p = C.c_void_p()
    _check(lib().lora_backbone_open(int(device_ordinal), C.create_string_buffer(handle, LORA_IPC_HANDLE_BYTES), C.byref(p)),
           "lora_backbone_open")
    return int(p.value)


def lora_backbone_close(device_ordinal: int, ptr: int) -> None:
    _check(lib().lora_backbone_close(int(device_ordinal), C.c_void_p(ptr)), "lora_backbone_close")


def lora_gemm_kernel_name(ctx, T: int, K: int, N: int, dtype: int) -> str:
    return lib().lora_gemm_kernel_name(C.c_void_p(ctx), int(T), int(K), int(N), int(dtype)).decode()
