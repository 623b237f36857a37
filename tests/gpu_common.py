"""Shared helpers of the GPU parity tests (imported lazily: needs torch + a GPU)."""
import numpy as np
import torch

from oracle import oracle_workload, plan_reference
from paper_2505_14468_amd import binding as B
from paper_2505_14468_amd import runtime as rt
from workloads import to_f64

TOL = {"bf16": 2e-2, "f32": 1e-5}  # max |Y_gpu - Y_oracle| <= TOL * RMS(Y_oracle)


def tol(dtype, K):
    """Tolerance as a fraction of the output's RMS.  bf16: 2e-2.  fp32: 1e-5 up to K = 1111; beyond, the rounding of
    K sequential fp32 additions (each within 2^-24 of the running sum) is what remains: an error of RMS
    ~0.3 * sqrt(K) * 2^-24 * RMS(Y), its maximum over 10^5..10^6 outputs ~11 times that (rows of X differ in norm)
    -- 3e-7 * sqrt(K), with margin 1.5 over what the unsplit kernels measure at K = 10264 (2.0e-5)."""
    if dtype == "bf16":
        return TOL["bf16"]
    return max(TOL["f32"], 3e-7 * float(K) ** 0.5)

_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        _ctx = rt.Context(0)
    return _ctx


def reset_options():
    for name in ("gemm_variant", "decode_waves", "decode_max_rows", "plan_fused_rows", "plan_variant", "expand_split", "gemm_split_k",
                 "shrink_rank_block"):
        ctx().set_option(name, -1)


def gpu_linear(wl, p=0, device_plan=False, stage="linear", only_used=False, return_all=False):
    """Run projection p of a workload through the C ABI; returns Y as fp64 numpy."""
    c = ctx()
    dev = c.device
    X, W0, table = rt.upload_workload(wl, p, dev, only_used=only_used)
    if device_plan:
        ra = torch.from_numpy(np.ascontiguousarray(wl.req_adapter)).to(dev)
        rn = torch.from_numpy(np.ascontiguousarray(wl.req_ntok)).to(dev)
        rk = torch.from_numpy(np.ascontiguousarray(wl.ranks)).to(dev)
        pl = rt.plan_device(c, ra, rn, rk, wl.r_max, wl.T)
    else:
        pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks, wl.r_max)
    Y = rt.linear(c, pl, X, W0, table, stage=stage)
    torch.cuda.synchronize()
    out = to_f64(rt.bits_from_tensor(Y))
    if return_all:
        return out, (X, W0, table, pl, Y)
    return out


def check_against_oracle(wl, Y_gpu, p=0, rows=None):
    """Element-by-element comparison with the fp64 oracle; returns max error / RMS."""
    Y_ref = oracle_workload(wl, p, rows=rows)
    got = Y_gpu if rows is None else Y_gpu[rows]
    assert got.shape == Y_ref.shape
    if Y_ref.size == 0:
        return 0.0
    rms = float(np.sqrt((Y_ref ** 2).mean()))
    err = float(np.abs(got - Y_ref).max())
    assert np.isfinite(got).all()
    t = tol(wl.dtype, wl.projections[p].K)
    assert err <= t * rms, f"max abs err {err:.3e} vs {t} * rms {rms:.3e} ({wl.name})"
    return err / rms


__all__ = ["B", "rt", "ctx", "reset_options", "gpu_linear", "check_against_oracle", "plan_reference", "TOL", "tol"]
