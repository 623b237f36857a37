"""The hot path under HIP graph capture: `lora_plan_device` + `lora_linear` (and `lora_linear_multi`) only launch
kernels -- no allocation, no synchronisation, no memset node -- so a captured step replays with new activations and
a new batch composition in the same buffers and gives, bit for bit, what the eager calls give."""
import numpy as np
import pytest
import torch

from workloads import make_custom
from workloads.configs import Projection

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", ["prefill_mixed", "decode", "split_k", "decode_much_adapter_work"])
def test_captured_step_replays_bit_exact(case):
    from gpu_common import B, rt, ctx, reset_options
    c = ctx()
    dev = c.device
    K, Ns, ranks = 264, (520, 264), (8, 16, 64, 40, 8, 24, 32, 48)
    if case == "prefill_mixed":  # long and short segments: shrink, separate expand kernel, tiled GEMM
        ids = [3, 0, -1, 5, 3, 1, 6, 2, 5, 3, 0, 4, -1, 6]
        L = [150, 1, 9, 64, 150, 63, 1, 17, 0, 141, 2, 5, 30, 1]
    elif case == "decode":  # decode-sized: the two launches of the decode path
        ids = [1, 1, 4, -1, 0, 7, 2, 2, 6, 5, 3, 0]
        L = [1] * 12
    elif case == "split_k":  # a few hundred rows, a long contraction axis: the GEMM split along K + the launch that sums
        ids = [3, 0, -1, 5, 3, 1, 6, 2]
        L = [70, 1, 9, 64, 90, 33, 1, 17]
        K = 2312
        assert "splitk" in B.lora_gemm_kernel_name(c.handle, sum(L), K, Ns[0], 1)
    else:  # 64 one-token requests on adapters of rank 128: V, expand kernel and the adding launch behind the stream
        ids = [i % 8 for i in range(64)]
        L = [1] * 64
        K, Ns, ranks = 520, (1544, 1536), (128,) * 8
    wl = make_custom(seed=970, dtype="bf16", K=K, N=Ns[0], ranks=ranks,
                     scales=(2.0, 0.5, 1.0, 0.25, 1.5, 1.0, 0.75, 1.0), req_adapter=np.asarray(ids), req_ntok=np.asarray(L),
                     name=f"graph_{case}")
    wl.projections = [Projection("a", K, Ns[0]), Projection("b", K, Ns[1])]
    wl.shared_x = True
    T, r_max = wl.T, wl.r_max
    up = [rt.upload_workload(wl, q, dev) for q in range(2)]
    X = up[0][0].clone()
    ra = torch.from_numpy(np.ascontiguousarray(wl.req_adapter)).to(dev)
    rn = torch.from_numpy(np.ascontiguousarray(wl.req_ntok)).to(dev)
    rk = torch.from_numpy(np.ascontiguousarray(wl.ranks)).to(dev)
    nbytes = B.lora_plan_bytes(wl.n_req, T, wl.n_adapters, r_max)

    def buffers():
        plan_buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        Ys = [torch.zeros((T, u[1].shape[0]), dtype=X.dtype, device=dev) for u in up]
        wss = [rt.workspace(T, K, u[1].shape[0], r_max, X.dtype, dev) for u in up]
        return plan_buf, Ys, wss

    def step(plan_buf, Ys, wss):  # plan + one projection alone + both through the multi call, on the current stream
        st = int(torch.cuda.current_stream().cuda_stream)
        plan = B.lora_plan_device(c.handle, ra.data_ptr(), rn.data_ptr(), wl.n_req, rk.data_ptr(), wl.n_adapters, r_max, T,
                                  plan_buf.data_ptr(), nbytes, st)
        pl = rt.Plan(plan, plan_buf)
        d = [rt.linear_desc(pl, X, up[q][1], Ys[q], up[q][2], wss[q]) for q in range(2)]
        B.lora_linear(c.handle, plan, d[0], st)
        B.lora_linear_multi(c.handle, plan, d, st)
        return d

    g_bufs, e_bufs = buffers(), buffers()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):  # first calls outside the capture (they set kernel attributes)
        keep = step(*g_bufs)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        keep = step(*g_bufs)
    rng = np.random.default_rng(5)
    for trial in range(3):
        # new activations, and from the second replay on another batch composition of the same size
        X.copy_(torch.from_numpy(rng.standard_normal((T, K)).astype(np.float32)).to(dev).to(X.dtype))
        if trial > 0:
            perm = torch.from_numpy(rng.permutation(wl.n_req)).to(dev)
            ra.copy_(ra[perm].clone())
            rn.copy_(rn[perm].clone())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        step(*e_bufs)  # the same step eagerly, into buffers of its own
        torch.cuda.synchronize()
        for q in range(2):
            assert torch.equal(g_bufs[1][q].view(torch.int16), e_bufs[1][q].view(torch.int16)), (case, trial, q)
        assert float(g_bufs[1][0].float().abs().max()) > 0
    reset_options()
