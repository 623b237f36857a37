"""lora_linear_static: the layer for callers that cannot allocate or bring a workspace (code under graph capture,
serving loops, harnesses that forbid hipMalloc).  Its kernels use the library's static device scratch array instead
of desc->workspace; the result must be that of lora_linear with a workspace of the same size -- checked here on two
calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

from workloads import make_custom

pytestmark = pytest.mark.gpu


def _case(seed, R, max_len, K, N):
    rng = np.random.default_rng(seed)
    ranks = (8, 16, 64, 32, 8, 24)
    ids = rng.integers(-1, len(ranks), size=R)
    L = rng.integers(0, max_len + 1, size=R)
    return make_custom(seed=seed, dtype="bf16", K=K, N=N, ranks=ranks, scales=(2.0, 0.5, 1.0, 0.25, 1.5, 1.0),
                       req_adapter=ids, req_ntok=L, name=f"static_{seed}")


def test_static_scratch_entry_point_matches_lora_linear_twice_in_a_row():
    import torch
    from gpu_common import B, rt, ctx, check_against_oracle, reset_options
    from workloads import to_f64
    reset_options()
    c = ctx()
    dev = c.device
    stream = int(torch.cuda.current_stream().cuda_stream)
    # first a batch of several hundred rows (tiled GEMM, adapter term through the scratch), then a decode-sized one
    for wl in (_case(801, R=40, max_len=30, K=328, N=520), _case(802, R=11, max_len=3, K=328, N=200)):
        X, W0, table = rt.upload_workload(wl, 0, dev)
        pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks, wl.r_max)
        N = W0.shape[0]
        ws = torch.empty(B.LORA_STATIC_SCRATCH_BYTES, dtype=torch.uint8, device=dev)
        Y_ref = torch.zeros((wl.T, N), dtype=X.dtype, device=dev)
        Y = torch.zeros((wl.T, N), dtype=X.dtype, device=dev)
        B.lora_linear(c.handle, pl.struct, rt.linear_desc(pl, X, W0, Y_ref, table, ws), stream)
        d = rt.linear_desc(pl, X, W0, Y, table, ws)
        d.workspace, d.workspace_bytes = None, 0
        B.lora_linear_static(c.handle, pl.struct, d, stream)
        torch.cuda.synchronize()
        assert pl.status(c)[0] == 0
        assert torch.equal(Y.view(torch.int16), Y_ref.view(torch.int16)), wl.name
        e = check_against_oracle(wl, to_f64(rt.bits_from_tensor(Y)))
        print(f"{wl.name}: T={wl.T} bitwise equal to lora_linear, err/rms vs oracle {e:.2e}", flush=True)


def test_static_scratch_entry_point_rejects_what_does_not_fit_and_a_workspace():
    import torch
    from gpu_common import B, rt, ctx
    c = ctx()
    dev = c.device
    stream = int(torch.cuda.current_stream().cuda_stream)
    # T x r_max x 2 bytes of V alone exceed the scratch: rejected before any launch
    T, K, N, r = 40000, 64, 64, 512
    assert B.lora_linear_workspace_bytes(T, K, N, r, B.LORA_DTYPE_BF16) > B.LORA_STATIC_SCRATCH_BYTES
    pl = rt.plan(c, np.zeros(1, np.int32), np.array([T], np.int32), np.array([r], np.int32), r)
    X = torch.zeros((T, K), dtype=torch.bfloat16, device=dev)
    W0 = torch.zeros((N, K), dtype=torch.bfloat16, device=dev)
    Y = torch.zeros((T, N), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(256, dtype=torch.uint8, device=dev)
    d = rt.linear_desc(pl, X, W0, Y, None, ws)
    assert B.lora_linear_static(c.handle, pl.struct, d, stream, raw=True) == B.LORA_ERR_INVALID_ARG  # brings a workspace
    d.workspace, d.workspace_bytes = None, 0
    assert B.lora_linear_static(c.handle, pl.struct, d, stream, raw=True) == B.LORA_ERR_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
