"""Torch plumbing around the C ABI: device buffers, pointer tables, the current
stream.  Nothing here computes: every step of the layer runs in the HIP kernels
behind ``binding``.  PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def tensor_from_bits(a: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 tensor; float32 -> fp32 tensor (bit-exact)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    if a.dtype == np.float32:
        return torch.from_numpy(a).to(device)
    raise TypeError(a.dtype)


def bits_from_tensor(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns; fp32 tensor -> float32 (bit-exact, on host)."""
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def dtype_code(t: torch.dtype) -> int:
    if t == torch.bfloat16:
        return B.LORA_DTYPE_BF16
    if t == torch.float32:
        return B.LORA_DTYPE_F32
    raise TypeError(f"unsupported dtype {t}")


class Context:
    """Owns a lora_ctx on one device."""

    def __init__(self, device: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the multi-LoRA linear layer has no CPU path")
        self.device = torch.device("cuda", device)
        self.handle = B.lora_ctx_create(device)

    def set_option(self, name: str, value: int) -> None:
        B.lora_ctx_set_option(self.handle, name, value)

    def close(self) -> None:
        if self.handle:
            B.lora_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class AdapterTable:
    """Device-resident pointer table over per-adapter weight tensors.

    ``A[a]`` is ``[r_a, K]``, ``B[a]`` is ``[N, r_a]`` (or None for a slot that
    is not resident); ``scales`` has one fp32 per slot."""

    def __init__(self, A: Sequence[Optional[torch.Tensor]], Bw: Sequence[Optional[torch.Tensor]], scales, device):
        assert len(A) == len(Bw)
        self.A = list(A)
        self.B = list(Bw)
        self.n = len(self.A)
        for t in self.A + self.B:
            assert t is None or (t.is_contiguous() and t.is_cuda)
        a_ptrs = np.array([0 if t is None else t.data_ptr() for t in self.A], np.int64)
        b_ptrs = np.array([0 if t is None else t.data_ptr() for t in self.B], np.int64)
        self.a_ptrs = torch.from_numpy(a_ptrs).to(device) if self.n else torch.zeros(1, dtype=torch.int64, device=device)
        self.b_ptrs = torch.from_numpy(b_ptrs).to(device) if self.n else torch.zeros(1, dtype=torch.int64, device=device)
        sc = np.ascontiguousarray(scales, np.float32).reshape(-1)
        assert sc.shape[0] == self.n
        self.scales = torch.from_numpy(sc).to(device) if self.n else torch.zeros(1, dtype=torch.float32, device=device)
        self.struct = B.make_adapter_table(self.n, self.a_ptrs.data_ptr(), self.b_ptrs.data_ptr(), self.scales.data_ptr())

    def set_slot(self, a: int, A: Optional[torch.Tensor], Bw: Optional[torch.Tensor]) -> None:
        """Load / evict one adapter (stream-ordered edit of the pointer table)."""
        self.A[a], self.B[a] = A, Bw
        self.a_ptrs[a] = 0 if A is None else A.data_ptr()
        self.b_ptrs[a] = 0 if Bw is None else Bw.data_ptr()


class Plan:
    """A lora_plan_t plus the device buffer it points into."""

    def __init__(self, struct: B.lora_plan_t, buf: torch.Tensor, keep=()):
        self.struct = struct
        self.buf = buf
        self._keep = keep

    @property
    def T(self) -> int:
        return int(self.struct.T)

    @property
    def r_max(self) -> int:
        return int(self.struct.r_max)

    def status(self, ctx: Context):
        return B.lora_plan_status(ctx.handle, self.struct, _stream())

    def _arr(self, ptr_name: str, count: int) -> np.ndarray:
        """Copy one of the plan's device int32 arrays to the host (tests / debugging)."""
        base = self.buf.data_ptr()
        off = getattr(self.struct, ptr_name) - base
        assert off >= 0 and off % 4 == 0
        view = self.buf.view(torch.int32)[off // 4: off // 4 + count]
        return view.cpu().numpy().copy()

    def to_host(self, ctx: Context) -> dict:
        status, n_seg = self.status(ctx)
        out = dict(status=status, n_seg=n_seg, unit_rows=int(self.struct.unit_rows))
        if status != 0:
            return out
        T = self.T
        sc = self._arr("scalars", 8)
        out.update(perm=self._arr("perm", T), row_seg=self._arr("row_seg", T), row_adapter=self._arr("row_adapter", T), row_ext=self._arr("row_ext", T),
                   seg_adapter=self._arr("seg_adapter", n_seg), seg_indptr=self._arr("seg_indptr", n_seg + 1),
                   seg_rank=self._arr("seg_rank", n_seg), seg_ext=self._arr("seg_ext", n_seg + 1),
                   seg_unit=self._arr("seg_unit", n_seg + 1), ext_total=int(sc[2]), n_units=int(sc[3]),
                   ext_rec=self._arr("ext_rec", (int(sc[2]) // 8) * 4).reshape(-1, 4),
                   unit_rec=self._arr("unit_rec", int(sc[3]) * 4).reshape(-1, 4),
                   tok_off=self._arr("tok_off", int(self.struct.n_req) + 1))
        return out


def _plan_buf(n_req: int, T: int, n_adapters: int, r_max: int, device) -> torch.Tensor:
    nbytes = B.lora_plan_bytes(n_req, T, n_adapters, r_max)
    if nbytes == 0:
        raise B.LoraError(B.LORA_ERR_INVALID_ARG, "lora_plan_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def plan(ctx: Context, req_adapter, req_ntok, adapter_rank, r_max: Optional[int] = None,
         buf: Optional[torch.Tensor] = None) -> Plan:
    """lora_plan() from host request arrays."""
    ra = np.ascontiguousarray(req_adapter, np.int32)
    rn = np.ascontiguousarray(req_ntok, np.int32)
    rk = np.ascontiguousarray(adapter_rank, np.int32)
    T = int(rn.astype(np.int64).sum())
    if r_max is None:
        r_max = int(rk.max()) if rk.size else 0
    if buf is None:
        buf = _plan_buf(ra.shape[0], T, rk.shape[0], r_max, ctx.device)
    st = B.lora_plan(ctx.handle, ra, rn, rk, r_max, T, buf.data_ptr(), buf.numel(), _stream())
    return Plan(st, buf)


def plan_device(ctx: Context, req_adapter: torch.Tensor, req_ntok: torch.Tensor, adapter_rank: torch.Tensor,
                r_max: int, T: int, buf: Optional[torch.Tensor] = None) -> Plan:
    """lora_plan_device() from int32 tensors already on the GPU."""
    for t in (req_adapter, req_ntok, adapter_rank):
        assert t.dtype == torch.int32 and t.is_cuda and t.is_contiguous()
    n_req, n_ad = req_adapter.numel(), adapter_rank.numel()
    if buf is None:
        buf = _plan_buf(n_req, T, n_ad, r_max, ctx.device)
    st = B.lora_plan_device(ctx.handle, req_adapter.data_ptr(), req_ntok.data_ptr(), n_req, adapter_rank.data_ptr(),
                            n_ad, r_max, T, buf.data_ptr(), buf.numel(), _stream())
    return Plan(st, buf, keep=(req_adapter, req_ntok, adapter_rank))


def workspace(T: int, K: int, N: int, r_max: int, dtype: torch.dtype, device, minimal: bool = False) -> torch.Tensor:
    """Workspace of the preferred size (every batch can take its fastest path), or of the minimal one."""
    fn = B.lora_linear_workspace_bytes if minimal else B.lora_linear_workspace_bytes_preferred
    nbytes = fn(T, K, N, r_max, dtype_code(dtype))
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def linear_desc(pl: Plan, X: torch.Tensor, W0: torch.Tensor, Y: torch.Tensor, table: Optional[AdapterTable],
                ws: torch.Tensor) -> B.lora_linear_desc:
    assert X.dim() == 2 and W0.dim() == 2 and Y.dim() == 2
    assert X.stride(1) == 1 and W0.stride(1) == 1 and Y.stride(1) == 1
    assert X.dtype == W0.dtype == Y.dtype
    K, N = W0.shape[1], W0.shape[0]
    assert X.shape[1] == K and Y.shape[1] == N and X.shape[0] == pl.T and Y.shape[0] == pl.T
    ldx = X.stride(0) if X.shape[0] > 1 else max(K, X.stride(0))
    ldy = Y.stride(0) if Y.shape[0] > 1 else max(N, Y.stride(0))
    return B.make_linear_desc(dtype_code(X.dtype), K, N, X.data_ptr(), ldx, W0.data_ptr(), W0.stride(0),
                              Y.data_ptr(), ldy, table.struct if table is not None else None,
                              ws.data_ptr(), ws.numel())


def linear(ctx: Context, pl: Plan, X: torch.Tensor, W0: torch.Tensor, table: Optional[AdapterTable],
           Y: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stage: str = "linear") -> torch.Tensor:
    """Run lora_linear (or one of its two stages) on the current stream; returns Y."""
    N = W0.shape[0]
    if Y is None:  # rows padded to a 16-byte multiple, as the ABI requires of ldy
        ce = 8 if X.dtype == torch.bfloat16 else 4
        Y = torch.empty((pl.T, (N + ce - 1) // ce * ce), dtype=X.dtype, device=X.device)[:, :N]
    if ws is None:
        ws = workspace(pl.T, W0.shape[1], N, pl.r_max, X.dtype, X.device)
    d = linear_desc(pl, X, W0, Y, table, ws)
    fn = {"linear": B.lora_linear, "shrink": B.lora_shrink, "gemm_expand": B.lora_gemm_expand}[stage]
    fn(ctx.handle, pl.struct, d, _stream())
    return Y


def linear_multi(ctx: Context, pl: Plan, X: torch.Tensor, projections) -> List[torch.Tensor]:
    """Run lora_linear_multi on the current stream: ``projections`` is a list of (W0, table) that share X;
    returns the list of outputs."""
    ce = 8 if X.dtype == torch.bfloat16 else 4
    descs, outs, keep = [], [], []
    for W0, table in projections:
        N = W0.shape[0]
        Y = torch.empty((pl.T, (N + ce - 1) // ce * ce), dtype=X.dtype, device=X.device)[:, :N]
        ws = workspace(pl.T, W0.shape[1], N, pl.r_max, X.dtype, X.device)
        descs.append(linear_desc(pl, X, W0, Y, table, ws))
        outs.append(Y)
        keep.append(ws)
    B.lora_linear_multi(ctx.handle, pl.struct, descs, _stream())
    pl._keep_multi = keep  # the workspaces live until the plan does (the kernels are still in flight)
    return outs


def upload_workload(wl, p: int, device, only_used: bool = False):
    """Device tensors of projection ``p`` of a ``workloads.Workload``: X, W0 and the adapter table."""
    X = tensor_from_bits(wl.X(p), device)
    W0 = tensor_from_bits(wl.W0(p), device)
    used = set(int(a) for a in wl.used_adapters())
    A: List[Optional[torch.Tensor]] = []
    Bw: List[Optional[torch.Tensor]] = []
    for a in range(wl.n_adapters):
        if only_used and a not in used:
            A.append(None)
            Bw.append(None)
        else:
            A.append(tensor_from_bits(wl.A(a, p), device))
            Bw.append(tensor_from_bits(wl.B(a, p), device))
    return X, W0, AdapterTable(A, Bw, wl.scales, device)


class AdapterPool:
    """Adapters of many functions on one GPU with room for only some of them: host copies (pinned) of every
    adapter, a byte budget on the GPU, and the greedy value-density policy of ``sched`` deciding what is
    pre-loaded and what is offloaded when a batch needs adapters that are not resident.  Uploads run on a side
    stream (default priority) and the pointer table is edited in stream order, so the layer's kernels never see a
    half-loaded adapter.  Decisions are the library's (``lora_preload_greedy`` / ``lora_offload_greedy``); this
    class only moves bytes and edits ``AdapterTable`` slots."""

    def __init__(self, ctx: Context, host_A: Sequence[np.ndarray], host_B: Sequence[np.ndarray], scales, gpu_bytes: float,
                 rates: Sequence[float], load_ms: Optional[Sequence[float]] = None):
        from . import sched
        self._sched = sched
        self.ctx, self.device = ctx, ctx.device
        self.n = len(host_A)

        def pin(a):
            t = tensor_from_bits(a, "cpu")
            p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
            p.copy_(t)
            return p
        self.host_A = [pin(a) for a in host_A]
        self.host_B = [pin(b) for b in host_B]
        self.bytes = [float(a.numel() * a.element_size() + b.numel() * b.element_size()) for a, b in zip(self.host_A, self.host_B)]
        self.rates = [float(r) for r in rates]
        # loading delay of an adapter: its bytes over the host link, plus a fixed cost (overridable per adapter)
        self.load_ms = [float(x) for x in load_ms] if load_ms is not None else [b / 25.0e6 + 0.05 for b in self.bytes]
        self.gpu_bytes = float(gpu_bytes)
        self.table = AdapterTable([None] * self.n, [None] * self.n, scales, self.device)
        self.resident = [False] * self.n
        self.side = torch.cuda.Stream(device=self.device)
        self.log: List[tuple] = []

    def _artifacts(self, pinned=()):
        pinned = set(int(a) for a in pinned)
        return [dict(function=a, kind=2, share_id=0, pinned=int(a in pinned), bytes=self.bytes[a],
                     value=self.load_ms[a] * self.rates[a]) for a in range(self.n)]

    def used_bytes(self) -> float:
        return sum(b for b, r in zip(self.bytes, self.resident) if r)

    def _upload(self, adapters):
        if not adapters:
            return
        main = torch.cuda.current_stream(self.device)
        fresh = []
        for a in adapters:  # allocate in the main stream's order, copy on the side stream
            A = torch.empty(self.host_A[a].shape, dtype=self.host_A[a].dtype, device=self.device)
            Bw = torch.empty(self.host_B[a].shape, dtype=self.host_B[a].dtype, device=self.device)
            fresh.append((a, A, Bw))
        self.side.wait_stream(main)
        with torch.cuda.stream(self.side):
            for a, A, Bw in fresh:
                A.copy_(self.host_A[a], non_blocking=True)
                Bw.copy_(self.host_B[a], non_blocking=True)
                A.record_stream(self.side)
                Bw.record_stream(self.side)
        main.wait_stream(self.side)
        for a, A, Bw in fresh:
            self.table.set_slot(a, A, Bw)
            self.resident[a] = True
            self.log.append(("load", a))

    def _evict(self, adapters):
        for a in adapters:
            self.table.set_slot(a, None, None)  # stream-ordered edit; the tensors are released in stream order too
            self.resident[a] = False
            self.log.append(("evict", a))

    def preload(self):
        """Section 4.1: fill the GPU budget in order of value density."""
        place, _ = self._sched.lora_preload_greedy(self._artifacts(), 0.0, self.gpu_bytes)
        self._upload([a for a in range(self.n) if (place[a] & 2) and not self.resident[a]])

    def ensure(self, needed: Sequence[int]) -> dict:
        """Make every adapter of ``needed`` resident before the next batch (section 4.3): offload the least valuable
        adapters that the batch does not use until the missing ones fit, then upload those."""
        needed = sorted(set(int(a) for a in needed if a >= 0))
        missing = [a for a in needed if not self.resident[a]]
        need = self.used_bytes() + sum(self.bytes[a] for a in missing) - self.gpu_bytes
        evicted = []
        if need > 0:
            ev, _, _, enough = self._sched.lora_offload_greedy(self._artifacts(pinned=needed), [int(r) for r in self.resident], need)
            if not enough:
                raise RuntimeError("the batch's adapters do not fit the GPU budget")
            evicted = [a for a in range(self.n) if ev[a]]
            self._evict(evicted)
        self._upload(missing)
        return dict(uploaded=missing, evicted=evicted)
