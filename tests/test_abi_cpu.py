"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and validates its arguments before touching HIP."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2505_14468_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "lora_mi355x.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lora_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert "lora_plan" in names and "lora_linear" in names and len(names) >= 14
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_status_codes_match_header():
    text = open(os.path.join(ROOT, "include", "lora_mi355x.h")).read()
    for name, val in re.findall(r"(LORA_(?:OK|ERR_[A-Z_]+)) = (-?\d+)", text):
        assert getattr(B, name) == int(val), name
        assert B.lora_strerror(int(val)) != "unknown status"
    assert B.lora_strerror(-99) == "unknown status"


def test_struct_layouts_match_c():
    # sizes as a C compiler lays the header's structs out on x86-64
    assert C.sizeof(B.lora_adapter_table_t) == 32
    assert C.sizeof(B.lora_plan_t) == 8 + 7 * 4 + 4 + 13 * 8  # (4 bytes of padding before the pointers)
    assert C.sizeof(B.lora_linear_desc) == 16 + 6 * 8 + 8 + 8 + 8


def test_plan_validate_codes():
    ranks = [8, 16, 0, 12, 64]
    v = lambda ids, L, T, r_max=32: B.lora_plan_validate(ids, L, ranks, r_max, T, raw=True)
    assert v([0, 1, -1], [2, 0, 3], 5) == B.LORA_OK
    assert B.lora_plan_validate([0, 1, -1, 0], [2, 1, 3, 1], ranks, 32, 7) == (3, 24)
    assert v([0, 5], [1, 1], 2) == B.LORA_ERR_BAD_ADAPTER_ID
    assert v([0, -2], [1, 1], 2) == B.LORA_ERR_BAD_ADAPTER_ID
    assert v([0, 1], [1, -1], 0) == B.LORA_ERR_LENGTH_MISMATCH
    assert v([0, 1], [1, 1], 3) == B.LORA_ERR_LENGTH_MISMATCH
    assert v([2], [1], 1) == B.LORA_ERR_ADAPTER_NOT_RESIDENT
    assert v([2], [0], 0) == B.LORA_OK  # a zero-length request does not use its adapter
    assert v([3], [1], 1) == B.LORA_ERR_SHAPE  # rank 12 is not a multiple of 8
    assert v([4], [1], 1) == B.LORA_ERR_RANK_TOO_LARGE
    assert v([4], [1], 1, r_max=64) == B.LORA_OK
    assert v([0], [1], 1, r_max=12) == B.LORA_ERR_INVALID_ARG  # r_max itself must be a multiple of 8
    assert v([], [], 0) == B.LORA_OK  # empty batch


def test_plan_bytes_and_workspace_bytes():
    assert B.lora_plan_bytes(-1, 0, 0, 0) == 0
    assert B.lora_plan_bytes(70000, 10, 4, 8) == 0  # more requests than LORA_MAX_REQUESTS
    small = B.lora_plan_bytes(16, 128, 4, 8)
    big = B.lora_plan_bytes(512, 2048, 512, 128)
    assert 0 < small < big
    assert small % 256 == 0
    assert B.lora_linear_workspace_bytes(0, 256, 256, 8, 0) == 256
    assert B.lora_linear_workspace_bytes(64, 4096, 4096, 16, 1) >= 64 * 16 * 2 + 64 * 4096 * 2
    assert B.lora_linear_workspace_bytes(8, 64, 0, 8, 1) == 0
    assert B.lora_linear_workspace_bytes(8, 64, 8, 8, 7) == 0
    # preferred size: plus an fp32 [T, N] adapter term (bf16 batches of any size, fp32 ones above 128 rows)
    assert B.lora_linear_workspace_bytes_preferred(64, 4096, 4096, 16, 1) >= B.lora_linear_workspace_bytes(64, 4096, 4096, 16, 1) + 64 * 4096 * 4
    assert (B.lora_linear_workspace_bytes_preferred(1000, 512, 300, 16, 1)
            >= B.lora_linear_workspace_bytes(1000, 512, 300, 16, 1) + 1000 * 300 * 4)
    assert B.lora_linear_workspace_bytes_preferred(8, 64, 0, 8, 1) == 0


def test_lora_plan_validates_before_touching_the_gpu():
    # ctx = NULL: every argument error is reported before the context is needed
    r = lambda ids, L, T, buf=256, nbytes=1 << 20: B.lora_plan(None, ids, L, [8, 16], 16, T, buf, nbytes, None, raw=True)
    assert r([0, 3], [1, 1], 2) == B.LORA_ERR_BAD_ADAPTER_ID
    assert r([0, 1], [1, 1], 5) == B.LORA_ERR_LENGTH_MISMATCH
    assert r([0, 1], [1, 1], 2, buf=256 + 16) == B.LORA_ERR_ALIGNMENT
    assert r([0, 1], [1, 1], 2, nbytes=64) == B.LORA_ERR_WORKSPACE_TOO_SMALL
    assert r([0, 1], [1, 1], 2, buf=0) == B.LORA_ERR_INVALID_ARG
    assert r([0, 1], [1, 1], 2) == B.LORA_ERR_INVALID_ARG  # all good except the missing context


def _fake_plan(T=4, n_adapters=2, r_max=16):
    p = B.lora_plan_t()
    p.T, p.n_req, p.n_adapters, p.r_max, p.magic, p.unit_rows = T, 1, n_adapters, r_max, 0x4C6F5241, 16
    p.scalars = 256  # never dereferenced on the host
    return p


def test_lora_linear_validates_before_touching_the_gpu():
    plan = _fake_plan()
    ws_bytes = B.lora_linear_workspace_bytes(4, 64, 64, 16, B.LORA_DTYPE_BF16)

    def run(**kw):
        a = dict(dtype=B.LORA_DTYPE_BF16, K=64, N=64, X=4096, ldx=64, W0=8192, ldw=64, Y=16384, ldy=64,
                 tbl=None, workspace=65536, workspace_bytes=ws_bytes)
        a.update(kw)
        d = B.make_linear_desc(**a)
        return B.lora_linear(None, plan, d, None, raw=True)

    assert run() == B.LORA_ERR_INVALID_ARG  # only the context is missing
    assert run(dtype=5) == B.LORA_ERR_INVALID_ARG
    assert run(K=60) == B.LORA_ERR_SHAPE
    assert run(K=0) == B.LORA_ERR_SHAPE
    assert run(N=0) == B.LORA_ERR_SHAPE
    assert run(ldx=32) == B.LORA_ERR_SHAPE
    assert run(ldy=68) == B.LORA_ERR_ALIGNMENT
    assert run(X=4096 + 2) == B.LORA_ERR_ALIGNMENT
    assert run(Y=4096) == B.LORA_ERR_INVALID_ARG  # Y aliases X
    assert run(ldx=1 << 30) == B.LORA_ERR_SHAPE  # 4 rows x 2^30 elements: X would span more than the 4 GiB the kernels address
    assert run(ldw=1 << 23) == B.LORA_ERR_SHAPE  # a 256-row tile of W0 would
    assert run(workspace=65536 + 64) == B.LORA_ERR_ALIGNMENT
    assert run(workspace_bytes=ws_bytes - 1) == B.LORA_ERR_WORKSPACE_TOO_SMALL
    bad = _fake_plan()
    bad.magic = 1
    d = B.make_linear_desc(B.LORA_DTYPE_BF16, 64, 64, 4096, 64, 8192, 64, 16384, 64, None, 65536, ws_bytes)
    assert B.lora_linear(None, bad, d, None, raw=True) == B.LORA_ERR_PLAN
    bad = _fake_plan()
    bad.unit_rows = 32  # a work-unit size no plan kernel writes
    assert B.lora_linear(None, bad, d, None, raw=True) == B.LORA_ERR_PLAN
    tbl = B.make_adapter_table(1, 512, 512, 512)  # fewer slots than the plan was built for
    assert run(tbl=tbl) == B.LORA_ERR_INVALID_ARG
    for stage in (B.lora_shrink, B.lora_gemm_expand):
        assert stage(None, plan, d, None, raw=True) == B.LORA_ERR_INVALID_ARG
    # several projections in one call: the same checks per projection, before the context is needed
    assert B.lora_linear_multi(None, plan, [d, d], None, raw=True) == B.LORA_ERR_INVALID_ARG
    assert B.lora_linear_multi(None, plan, [], None, raw=True) == B.LORA_ERR_INVALID_ARG
    assert B.lora_linear_multi(None, plan, [d] * (B.LORA_MAX_MULTI + 1), None, raw=True) == B.LORA_ERR_INVALID_ARG
    d_bad = B.make_linear_desc(B.LORA_DTYPE_BF16, 60, 64, 4096, 64, 8192, 64, 32768, 64, None, 65536, ws_bytes)
    assert B.lora_linear_multi(None, plan, [d, d_bad], None, raw=True) == B.LORA_ERR_SHAPE
    assert B.lora_linear_multi(None, bad, [d], None, raw=True) == B.LORA_ERR_PLAN


def test_kernel_selection_is_host_side():
    assert B.lora_gemm_kernel_name(None, 64, 4096, 4096, B.LORA_DTYPE_BF16).startswith("decode_tb4")
    assert B.lora_gemm_kernel_name(None, 16, 4096, 4096, B.LORA_DTYPE_BF16).startswith("decode_tb1")
    assert B.lora_gemm_kernel_name(None, 9000, 4096, 11008, B.LORA_DTYPE_BF16).startswith("tile_")
    assert B.lora_gemm_kernel_name(None, 64, 256, 256, B.LORA_DTYPE_F32).startswith("tile_")


def test_launch_paths_of_the_benchmark_shapes():
    """The host's choice of launch path is a function of (rows, K, N, dtype) alone, so it can be pinned without a GPU:
    the five benchmark configurations' shapes and the switch points of the batch-size sweep (decode path up to 128
    rows, tiles split along K while they would leave most CUs idle, one-round tile shapes above)."""
    bf16, f32 = B.LORA_DTYPE_BF16, B.LORA_DTYPE_F32
    want = {(128, 256, 256, f32): "tile_64x64",                  # configuration 0
            (64, 4096, 4096, bf16): "decode_tb4",                # configuration 1
            (7539, 4096, 11008, bf16): "tile_256x224",           # configuration 2: 5.86 rounds instead of 5.04 of 256x256
            (1216, 4096, 4096, bf16): "tile_128x192",            # configuration 3: q/k/v/o
            (1216, 4096, 11008, bf16): "tile_256x224",           #                  gate, up
            (1216, 11008, 4096, bf16): "tile_256x256_splitk3",   #                  down: a long K into few columns
            (2048, 5120, 13824, bf16): "tile_256x224",           # configuration 4
            (1, 4096, 4096, bf16): "decode_tb1", (128, 4096, 4096, bf16): "decode_tb8",
            (96, 4096, 11008, bf16): "decode_tb6", (128, 4096, 11008, bf16): "tile_64x64",  # wide outputs near 128 rows: tiles
            (256, 4096, 4096, bf16): "tile_128x128_splitk4", (1024, 4096, 4096, bf16): "tile_128x128",
            (129, 4096, 4096, f32): "tile_128x128_splitk6"}
    got = {k: B.lora_gemm_kernel_name(None, *k) for k in want}
    assert got == want
    # the preferred workspace has room for the partial outputs exactly where a split is chosen
    for (T, K, N, dt), name in want.items():
        extra = B.lora_linear_workspace_bytes_preferred(T, K, N, 64, dt) - B.lora_linear_workspace_bytes(T, K, N, 64, dt)
        splits = int(name.split("splitk")[1]) if "splitk" in name else 0
        d_bytes = T * ((N + 7) // 8 * 8) * 4 if (T > 128 or dt == bf16) else 0
        assert abs(extra - (d_bytes + splits * T * ((N + 7) // 8 * 8) * 4)) <= 1024, (T, K, N, name, extra)
