"""The five benchmark configurations and a free-form builder for test cases.

Every tensor has a random stream of its own, keyed by (seed, tensor kind,
projection, adapter), so any tensor can be drawn lazily and independently of
the others; values are drawn in fp32 and, for the bf16 configurations, rounded
once (round-to-nearest-even) to the bit patterns that both the CPU oracle and
the GPU receive.

Storage layouts (the ones a PyTorch / PEFT model holds):
  X   [T, K]    row-major, rows of one request contiguous, requests in order
  W0  [N, K]    row-major (``nn.Linear.weight``)
  A_a [r_a, K]  row-major (LoRA "down" weight)
  B_a [N, r_a]  row-major (LoRA "up" weight)
bf16 tensors are returned as ``uint16`` bit patterns, fp32 tensors as ``float32``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

from .bits import bf16_bits_from_f32

CONFIG_NAMES = [
    "c0_tiny_fp32",
    "c1_decode_qproj",
    "c2_prefill_mlp_up",
    "c3_layer7_mixed",
    "c4_adapter_heavy_13b",
]

_TAG_X, _TAG_W, _TAG_A, _TAG_B, _TAG_REQ = 1, 2, 3, 4, 5


@dataclass(frozen=True)
class Projection:
    name: str
    K: int  # d_in
    N: int  # d_out


@dataclass
class Workload:
    name: str
    seed: int
    dtype: str  # "bf16" or "f32"
    ranks: np.ndarray  # int32 [n_adapters]
    scales: np.ndarray  # float32 [n_adapters]
    req_adapter: np.ndarray  # int32 [R], -1 = no adapter
    req_ntok: np.ndarray  # int32 [R]
    projections: List[Projection]
    sigma_x: float = 1.0
    sigma_w: float = 0.02
    sigma_b: float = 0.02
    sigma_a: Optional[float] = None  # None -> 1/sqrt(K) of the projection
    integer_valued: bool = False  # small integers in [-4, 4] (exact in every precision)
    shared_x: bool = False  # every projection reads projection 0's X (fused QKV, gate + up; same K required)
    _cache: dict = field(default_factory=dict, repr=False)

    # ---- batch geometry -------------------------------------------------
    @property
    def n_adapters(self) -> int:
        return int(self.ranks.shape[0])

    @property
    def n_req(self) -> int:
        return int(self.req_adapter.shape[0])

    @property
    def T(self) -> int:
        return int(self.req_ntok.astype(np.int64).sum())

    @property
    def r_max(self) -> int:
        return int(self.ranks.max()) if self.n_adapters else 0

    def used_adapters(self) -> np.ndarray:
        m = (self.req_ntok > 0) & (self.req_adapter >= 0)
        return np.unique(self.req_adapter[m])

    def row_adapter(self) -> np.ndarray:
        """Adapter id of every token row, in request order (bookkeeping only)."""
        return np.repeat(self.req_adapter, self.req_ntok).astype(np.int32)

    # ---- tensors --------------------------------------------------------
    def _draw(self, tag: int, proj: int, idx: int, shape, sigma: float) -> np.ndarray:
        rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([self.seed, tag, proj, idx])))
        if self.integer_valued:
            v = rng.integers(-4, 5, size=shape).astype(np.float32)
        else:
            v = rng.standard_normal(size=shape, dtype=np.float32)
            v *= np.float32(sigma)
        if self.dtype == "bf16":
            return bf16_bits_from_f32(v)
        return v

    def _get(self, key, make):
        if key not in self._cache:
            self._cache[key] = make()
        return self._cache[key]

    def X(self, p: int = 0) -> np.ndarray:
        if self.shared_x:
            assert self.projections[p].K == self.projections[0].K
            p = 0
        pr = self.projections[p]
        return self._get(("X", p), lambda: self._draw(_TAG_X, p, 0, (self.T, pr.K), self.sigma_x))

    def W0(self, p: int = 0) -> np.ndarray:
        pr = self.projections[p]
        return self._get(("W", p), lambda: self._draw(_TAG_W, p, 0, (pr.N, pr.K), self.sigma_w))

    def A(self, a: int, p: int = 0) -> np.ndarray:
        pr = self.projections[p]
        sa = self.sigma_a if self.sigma_a is not None else 1.0 / np.sqrt(pr.K)
        return self._get(("A", p, a), lambda: self._draw(_TAG_A, p, a, (int(self.ranks[a]), pr.K), sa))

    def B(self, a: int, p: int = 0) -> np.ndarray:
        pr = self.projections[p]
        return self._get(("B", p, a), lambda: self._draw(_TAG_B, p, a, (pr.N, int(self.ranks[a])), self.sigma_b))

    def drop_cache(self) -> None:
        self._cache.clear()

    # ---- accounting used by the benchmark (no arithmetic of the layer) ---
    def useful_flops(self, p: int = 0) -> int:
        pr = self.projections[p]
        ra = self.row_adapter()
        r_rows = np.where(ra >= 0, self.ranks[np.maximum(ra, 0)], 0).astype(np.int64)
        return int(2 * self.T * pr.K * pr.N + 2 * int(r_rows.sum()) * (pr.K + pr.N))

    def algorithmic_bytes(self, p: int = 0) -> int:
        """Every operand touched once; each *used* adapter counted once."""
        pr = self.projections[p]
        e = 2 if self.dtype == "bf16" else 4
        r_used = int(self.ranks[self.used_adapters()].astype(np.int64).sum())
        return e * (self.T * pr.K + pr.K * pr.N + self.T * pr.N + r_used * (pr.K + pr.N))


def _req_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, _TAG_REQ])))


def _bounded_zipf(rng: np.random.Generator, n: int, size: int, alpha: float = 1.0) -> np.ndarray:
    """Ids in [0, n) with P(id = k-1) proportional to k^-alpha, k = 1..n."""
    w = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** alpha
    cdf = np.cumsum(w) / w.sum()
    u = rng.random(size)
    return np.minimum(np.searchsorted(cdf, u, side="right"), n - 1).astype(np.int32)


def _fix_total(lengths: np.ndarray, total: int) -> np.ndarray:
    """Deterministically adjust positive lengths to a fixed sum: shave the
    currently largest entry (lowest index on ties) while too long, hand out
    +1 round-robin from index 0 while too short.  Every entry stays >= 1."""
    L = lengths.astype(np.int64).copy()
    while L.sum() > total:
        i = int(np.argmax(L))
        if L[i] <= 1:
            raise ValueError("cannot shrink lengths to the requested total")
        L[i] -= 1
    j = 0
    while L.sum() < total:
        L[j % L.size] += 1
        j += 1
    return L.astype(np.int32)


def make_workload(index: int) -> Workload:
    """Benchmark configuration ``index`` (0..4); seed = 1000 + index."""
    seed = 1000 + index
    rng = _req_rng(seed)
    name = CONFIG_NAMES[index]
    if index == 0:
        ranks = np.full(4, 8, np.int32)
        scales = np.full(4, 2.0, np.float32)
        ids = rng.integers(0, 4, size=16).astype(np.int32)
        ntok = np.full(16, 8, np.int32)
        return Workload(name, seed, "f32", ranks, scales, ids, ntok, [Projection("linear", 256, 256)])
    if index == 1:
        ranks = np.full(32, 16, np.int32)
        scales = np.full(32, 2.0, np.float32)
        ids = rng.integers(0, 32, size=64).astype(np.int32)
        ntok = np.ones(64, np.int32)
        return Workload(name, seed, "bf16", ranks, scales, ids, ntok, [Projection("q_proj", 4096, 4096)])
    if index == 2:
        ranks = np.full(8, 64, np.int32)
        scales = np.full(8, 1.0, np.float32)
        ntok = rng.integers(128, 1025, size=16).astype(np.int32)
        ids = _bounded_zipf(rng, 8, 16)
        return Workload(name, seed, "bf16", ranks, scales, ids, ntok, [Projection("up_proj", 4096, 11008)])
    if index == 3:
        ranks = rng.choice(np.array([8, 16, 32, 64], np.int32), size=100).astype(np.int32)
        scales = (16.0 / ranks).astype(np.float32)
        ntok = np.concatenate([np.full(4, 256, np.int32), np.ones(192, np.int32)])
        ids = rng.integers(0, 100, size=196).astype(np.int32)
        order = rng.permutation(196)
        projs = [
            Projection("q_proj", 4096, 4096),
            Projection("k_proj", 4096, 4096),
            Projection("v_proj", 4096, 4096),
            Projection("o_proj", 4096, 4096),
            Projection("gate_proj", 4096, 11008),
            Projection("up_proj", 4096, 11008),
            Projection("down_proj", 11008, 4096),
        ]
        return Workload(name, seed, "bf16", ranks, scales, ids[order], ntok[order], projs)
    if index == 4:
        ranks = np.full(512, 128, np.int32)
        scales = np.full(512, 0.5, np.float32)
        ntok = _fix_total(rng.geometric(0.25, size=512), 2048)
        ids = _bounded_zipf(rng, 512, 512)
        return Workload(name, seed, "bf16", ranks, scales, ids, ntok, [Projection("up_proj", 5120, 13824)])
    raise IndexError(index)


def same_adapter_decode(batch: int, adapter: int = 3, seed: int = 2000) -> Workload:
    """``batch`` one-token requests that all use one adapter, at configuration
    1's shape: the one-adapter-per-function regime."""
    ranks = np.full(32, 16, np.int32)
    scales = np.full(32, 2.0, np.float32)
    ids = np.full(batch, adapter, np.int32)
    ntok = np.ones(batch, np.int32)
    return Workload(f"decode_same_adapter_b{batch}", seed + batch, "bf16", ranks, scales, ids, ntok,
                    [Projection("q_proj", 4096, 4096)])


def make_custom(
    *,
    seed: int,
    dtype: str,
    K: int,
    N: int,
    ranks: Sequence[int],
    scales: Sequence[float],
    req_adapter: Sequence[int],
    req_ntok: Sequence[int],
    name: str = "custom",
    integer_valued: bool = False,
    sigma_a: Optional[float] = None,
    sigma_b: float = 0.02,
    sigma_w: float = 0.02,
) -> Workload:
    return Workload(
        name,
        seed,
        dtype,
        np.asarray(ranks, np.int32).reshape(-1),
        np.asarray(scales, np.float32).reshape(-1),
        np.asarray(req_adapter, np.int32).reshape(-1),
        np.asarray(req_ntok, np.int32).reshape(-1),
        [Projection("linear", int(K), int(N))],
        sigma_a=sigma_a,
        sigma_b=sigma_b,
        sigma_w=sigma_w,
        integer_valued=integer_valued,
    )
