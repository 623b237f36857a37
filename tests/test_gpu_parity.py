"""GPU parity of the layer (steps a2-a4) against the fp64 CPU oracle, element by element,
through the C ABI.  Tolerance: max |Y_gpu - Y_oracle| <= 2e-2 * RMS(Y_oracle) for bf16 inputs
with fp32 accumulation, 1e-5 * RMS for the fp32 configuration."""
import numpy as np
import pytest

from workloads import make_custom, make_workload, same_adapter_decode, to_f64

pytestmark = pytest.mark.gpu

VARIANTS = {"tile_128x128": 0, "tile_256x128": 1, "tile_64x64": 3, "decode": 4, "tile_256x256w4": 5,
            "tile_128x192": 9, "tile_256x192": 10, "tile_256x224": 11}


def _mixed_batch(seed, R, n_ad, max_len, with_none=True, zero_len=True):
    rng = np.random.default_rng(seed)
    ids = rng.integers(-1 if with_none else 0, n_ad, size=R)
    L = rng.integers(0 if zero_len else 1, max_len + 1, size=R)
    return ids, L


def test_config0_fp32_all_tile_variants():
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options
    wl = make_workload(0)
    for name in ("tile_64x64", "tile_128x128", "tile_256x128", "tile_256x256w4", "tile_128x192", None):
        ctx().set_option("gemm_variant", VARIANTS[name] if name else -1)
        Y = gpu_linear(wl)
        e = check_against_oracle(wl, Y)
        print(f"config0 fp32 {name}: err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("variant", ["tile_64x64", "tile_128x128", "tile_256x128", "tile_256x256w4", "tile_128x192", "tile_256x192", "tile_256x224"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tile_kernels_ragged_multi_tile(variant, dtype):
    """Several tiles in both directions, ragged tails in T, N and K, mixed ranks, rows without
    an adapter, zero-length requests; host-built and device-built plans."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options
    ids, L = _mixed_batch(3, R=37, n_ad=6, max_len=24)
    wl = make_custom(seed=31, dtype=dtype, K=328, N=300, ranks=(8, 16, 64, 32, 8, 24), scales=(2.0, 0.5, 1.0, 0.25, 1.5, 1.0),
                     req_adapter=ids, req_ntok=L, name=f"ragged_{variant}_{dtype}")
    assert wl.T > 256
    ctx().set_option("gemm_variant", VARIANTS[variant])
    for device_plan in (False, True):
        Y = gpu_linear(wl, device_plan=device_plan)
        e = check_against_oracle(wl, Y)
    print(f"{wl.name}: T={wl.T} err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("variant", ["tile_64x64", "tile_128x128", "tile_256x128", "tile_256x256w4", "tile_128x192", "tile_256x192", "tile_256x224"])
def test_tile_kernels_short_contraction_axes(variant):
    """One to five stages of the contraction axis, with and without a partial last stage: the prologue and
    the last stages of the software-pipelined loops (two stages of loads ahead) for every stage count."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options
    ids, L = _mixed_batch(19, R=9, n_ad=3, max_len=40, zero_len=False)
    ctx().set_option("gemm_variant", VARIANTS[variant])
    for dtype, Ks in (("bf16", (24, 64, 72, 128, 136, 192, 200, 256, 264, 320)), ("f32", (8, 32, 40, 64, 72, 96, 104, 160))):
        for K in Ks:
            wl = make_custom(seed=600 + K, dtype=dtype, K=K, N=72, ranks=(8, 16, 24), scales=(1.0, 0.5, 2.0),
                             req_adapter=ids, req_ntok=L, name=f"shortk_{variant}_{dtype}_{K}")
            e = check_against_oracle(wl, gpu_linear(wl))
    print(f"{variant}: last err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_separate_expand_kernel_ragged(dtype):
    """The adapter term added by the expand kernel of its own (many small segments) instead of inside the
    GEMM: ragged N, ranks that are not multiples of 32, segments of more than 16 and more than 64 rows,
    rows without an adapter, zero-length requests; both results against the oracle and against each other."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options, TOL
    ids, L = _mixed_batch(11, R=60, n_ad=7, max_len=30)
    ids[:6] = 3  # one adapter with a long segment
    L[:6] = 29
    wl = make_custom(seed=77, dtype=dtype, K=264, N=1100, ranks=(8, 16, 64, 40, 8, 24, 128), scales=(2.0, 0.5, 1.0, 0.25, 1.5, 1.0, 0.75),
                     req_adapter=ids, req_ntok=L, name=f"expand_split_{dtype}")
    assert wl.T > 256
    out = {}
    for split in (0, 1):
        ctx().set_option("expand_split", split)
        for device_plan in (False, True):
            out[split] = gpu_linear(wl, device_plan=device_plan)
            e = check_against_oracle(wl, out[split])
        print(f"{wl.name} split={split}: T={wl.T} err/rms {e:.2e}", flush=True)
    rms = float(np.sqrt((out[0] ** 2).mean()))
    assert float(np.abs(out[0] - out[1]).max()) <= TOL[dtype] * rms
    reset_options()


@pytest.mark.parametrize("variant", ["tile_64x64", "tile_128x128", "tile_256x128", "tile_256x256w4", "tile_128x192",
                                     "tile_256x192", "tile_256x224"])
def test_long_segments_in_the_gemm_short_ones_in_the_expand_kernel(variant):
    """Ranks up to 64 with the separate expand kernel on: the tiled GEMM computes the term of segments of 64 rows
    and more itself and adds the expand kernel's result for the shorter ones (the other GEMM kernels take all of
    it from the expand kernel).  Segments of exactly 63 and 64 rows, one spanning several M tiles, single rows,
    rows without an adapter, an adapter that is resident but unused; plans of 16-row and of 64-row units."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options, TOL
    for dtype in ("bf16", "f32"):
        for case, (ids, L) in enumerate([
                # few requests: T/16 + segments fits the CUs -> 16-row units
                ([3, 0, -1, 5, 3, 1, 6, 2, 5, 3, 0, 4, -1, 6], [150, 1, 9, 64, 150, 63, 1, 17, 0, 141, 2, 5, 30, 1]),
                # many one-row requests around two long segments -> 64-row units
                ([2] * 70 + list(np.arange(400) % 7) + [-1] * 33 + [4] * 30, [30] * 70 + [1] * 400 + [1] * 33 + [80] * 30)]):
            wl = make_custom(seed=910 + case, dtype=dtype, K=200, N=1100, ranks=(8, 16, 64, 40, 8, 24, 32, 48),
                             scales=(2.0, 0.5, 1.0, 0.25, 1.5, 1.0, 0.75, 1.0), req_adapter=np.asarray(ids), req_ntok=np.asarray(L),
                             name=f"hybrid_{variant}_{dtype}_{case}")
            assert wl.T > 256 and (wl.T // 16 + 8 > 256) == bool(case)
            out = {}
            ctx().set_option("gemm_variant", VARIANTS[variant])
            for split in (1, 0):
                ctx().set_option("expand_split", split)
                out[split] = gpu_linear(wl, device_plan=bool(case))
                e = check_against_oracle(wl, out[split])
            rms = float(np.sqrt((out[0] ** 2).mean()))
            assert float(np.abs(out[0] - out[1]).max()) <= TOL[dtype] * rms
            print(f"{wl.name}: T={wl.T} err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("seed", range(4))
def test_random_segment_mixes_fused_and_separate(seed):
    """Random batches of long and short segments, ranks 8..64, with the adapter term fused, separate, and by the
    built-in choice; in the fused runs an M tile of 256 rows holds up to ~150 adapters (more than 4096 ranks: the
    extension table of a tile is built in more than one batch)."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options, TOL
    rng = np.random.default_rng(4000 + seed)
    n_ad = 400
    ranks = tuple(int(r) for r in rng.choice([8, 16, 24, 32, 48, 64], size=n_ad, p=[0.05, 0.05, 0.05, 0.1, 0.15, 0.6]))
    scales = tuple(float(x) for x in rng.choice([0.25, 0.5, 1.0, 2.0], size=n_ad))
    R = 800
    ids = rng.integers(-1, n_ad, size=R)
    L = rng.integers(0, 3, size=R)
    for a in rng.choice(n_ad, size=3, replace=False):  # three adapters with long segments
        k = rng.integers(0, R, size=4)
        ids[k] = a
        L[k] = rng.integers(20, 90, size=4)
    dtype = "bf16" if seed % 2 == 0 else "f32"
    wl = make_custom(seed=4100 + seed, dtype=dtype, K=136, N=520, ranks=ranks, scales=scales, req_adapter=ids, req_ntok=L,
                     name=f"random_mix_{seed}")
    assert wl.T > 600
    out = {}
    for variant in ("tile_256x224", "tile_128x192", None):
        ctx().set_option("gemm_variant", VARIANTS[variant] if variant else -1)
        for split in (0, 1, -1):
            ctx().set_option("expand_split", split)
            out[split] = gpu_linear(wl, device_plan=bool(seed & 1))
            e = check_against_oracle(wl, out[split])
        rms = float(np.sqrt((out[0] ** 2).mean()))
        assert float(np.abs(out[0] - out[1]).max()) <= TOL[dtype] * rms
    print(f"{wl.name}: T={wl.T} {dtype} err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_linear_multi_projections_of_the_same_activations(dtype):
    """lora_linear_multi: three projections of one X (different widths, one ragged) in one call -- every output
    against the oracle and against the single-projection call; tile shapes, adapter term fused / separate; a
    decode-sized batch (bf16: the decode path's two launches cover all three); argument errors."""
    import torch
    from workloads.configs import Projection
    from gpu_common import B, rt, ctx, check_against_oracle, reset_options, TOL
    from workloads import to_f64
    c = ctx()
    for case, (ids, L) in enumerate([([3, 0, -1, 5, 3, 1, 6, 2, 5, 3, 0, 4, -1, 6], [150, 1, 9, 64, 150, 63, 1, 17, 0, 141, 2, 5, 30, 1]),
                                     ([1, 1, 4, -1, 0, 7, 2], [3, 9, 1, 5, 7, 11, 4])]):
        wl = make_custom(seed=930 + case, dtype=dtype, K=200, N=520, ranks=(8, 16, 64, 40, 8, 24, 32, 48),
                         scales=(2.0, 0.5, 1.0, 0.25, 1.5, 1.0, 0.75, 1.0), req_adapter=np.asarray(ids), req_ntok=np.asarray(L),
                         name=f"multi_{dtype}_{case}")
        wl.projections = [Projection("a", 200, 520), Projection("b", 200, 264), Projection("c", 200, 1100)]
        wl.shared_x = True
        dev = c.device
        up = [rt.upload_workload(wl, q, dev) for q in range(3)]
        X = up[0][0]
        assert all(torch.equal(u[0], X) for u in up)
        pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks, wl.r_max)
        for variant in (None, "tile_256x224", "tile_128x192", "tile_64x64"):
            c.set_option("gemm_variant", VARIANTS[variant] if variant else -1)
            for split in (-1, 0, 1):
                c.set_option("expand_split", split)
                outs = rt.linear_multi(c, pl, X, [(u[1], u[2]) for u in up])
                torch.cuda.synchronize()
                for q in range(3):
                    got = to_f64(rt.bits_from_tensor(outs[q]))
                    e = check_against_oracle(wl, got, p=q)
                    single = to_f64(rt.bits_from_tensor(rt.linear(c, pl, X, up[q][1], up[q][2])))
                    torch.cuda.synchronize()
                    rms = float(np.sqrt((single ** 2).mean()))
                    # (each is within TOL of the oracle; the single call may take a path that rounds V to bf16 where
                    # the fused one keeps it in fp32, so the two may differ by the sum of their errors)
                    assert float(np.abs(got - single).max()) <= 2 * TOL[dtype] * rms
        print(f"{wl.name}: T={wl.T} err/rms {e:.2e}", flush=True)
        reset_options()
        # one of the projections without an adapter table: the backbone product alone for that one
        outs = rt.linear_multi(c, pl, X, [(up[0][1], up[0][2]), (up[1][1], None), (up[2][1], up[2][2])])
        torch.cuda.synchronize()
        base = to_f64(rt.bits_from_tensor(rt.linear(c, pl, X, up[1][1], None)))
        torch.cuda.synchronize()
        assert float(np.abs(to_f64(rt.bits_from_tensor(outs[1])) - base).max()) <= TOL[dtype] * float(np.sqrt((base ** 2).mean()))
        check_against_oracle(wl, to_f64(rt.bits_from_tensor(outs[0])), p=0)
        check_against_oracle(wl, to_f64(rt.bits_from_tensor(outs[2])), p=2)
        # argument errors: more projections than the limit, projections of different activations, one output twice
        ws = [rt.workspace(pl.T, 200, u[1].shape[0], pl.r_max, X.dtype, dev) for u in up]
        Ys = [torch.empty((pl.T, (u[1].shape[0] + 7) // 8 * 8), dtype=X.dtype, device=dev)[:, :u[1].shape[0]] for u in up]
        d = [rt.linear_desc(pl, X, up[q][1], Ys[q], up[q][2], ws[q]) for q in range(3)]
        st = torch.cuda.current_stream().cuda_stream
        assert B.lora_linear_multi(c.handle, pl.struct, d + d[:2], st, raw=True) == B.LORA_ERR_INVALID_ARG
        assert B.lora_linear_multi(c.handle, pl.struct, [], st, raw=True) == B.LORA_ERR_INVALID_ARG
        X2 = X.clone()
        d_other = rt.linear_desc(pl, X2, up[1][1], Ys[1], up[1][2], ws[1])
        assert B.lora_linear_multi(c.handle, pl.struct, [d[0], d_other], st, raw=True) == B.LORA_ERR_INVALID_ARG
        d_same_y = rt.linear_desc(pl, X, up[0][1], Ys[0], up[0][2], torch.empty_like(ws[0]))
        assert B.lora_linear_multi(c.handle, pl.struct, [d[0], d_same_y], st, raw=True) == B.LORA_ERR_INVALID_ARG
        assert B.lora_linear_multi(c.handle, pl.struct, d, st, raw=True) == B.LORA_OK
        torch.cuda.synchronize()


@pytest.mark.parametrize("seed", [11, 12, 13, 14, 15, 16])
def test_random_shapes_ranks_and_batch_mixes(seed):
    """Ten random cases per seed over dtype, K, N, batch size (decode-sized to a few thousand rows), adapter pool, ranks
    and segment lengths, each on whatever launch path the library picks for it (printed), host- and device-built
    plans alternating: every output element against the oracle at the stated tolerance."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options, B
    reset_options()
    rng = np.random.default_rng(seed)
    for case in range(10):
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        K = int(rng.choice([264, 520, 1032, 2056, 4104])) if dtype == "bf16" else int(rng.choice([264, 520, 1032]))
        N = int(rng.choice([24, 72, 264, 520, 1100, 2056]))
        T = int(rng.choice([rng.integers(1, 33), rng.integers(33, 129), rng.integers(129, 700), rng.integers(700, 2200)]))
        n_ad = int(rng.choice([1, 2, 5, 17, 70]))
        ranks = [int(min(rng.choice([8, 16, 24, 40, 64, 128]), (K // 64) * 8)) for _ in range(n_ad)]
        scales = [float(rng.choice([0.25, 0.5, 1.0])) for _ in range(n_ad)]
        lens, left = [], T
        while left > 0:
            n = int(min(left, rng.choice([1, 1, 2, 5, 17, 64, 200, 500])))
            lens.append(n)
            left -= n
        if rng.random() < 0.3:
            lens.insert(int(rng.integers(0, len(lens) + 1)), 0)  # a request without tokens
        ids = rng.integers(-1, n_ad, size=len(lens))
        wl = make_custom(seed=100 * seed + case, dtype=dtype, K=K, N=N, ranks=ranks, scales=scales, req_adapter=ids,
                         req_ntok=np.asarray(lens), name=f"random_{seed}_{case}")
        name = B.lora_gemm_kernel_name(ctx().handle, wl.T, K, N, 1 if dtype == "bf16" else 0)
        print(f"{wl.name}: {dtype} T={wl.T} K={K} N={N} adapters={n_ad} r_max={max(ranks)} requests={len(lens)} {name}", end=" ", flush=True)
        e = check_against_oracle(wl, gpu_linear(wl, device_plan=bool(case & 1)))
        print(f"err/rms {e:.2e}", flush=True)


@pytest.mark.parametrize("dtype,K,N,T", [("bf16", 2312, 520, 129), ("bf16", 2312, 520, 384), ("bf16", 8200, 264, 200),
                                          ("bf16", 4096, 1100, 300), ("f32", 1032, 264, 150), ("f32", 2056, 520, 140),
                                          ("bf16", 10248, 520, 1100), ("bf16", 11008, 1000, 1301), ("f32", 10264, 264, 1030)])
def test_mid_sized_batches_split_along_k(dtype, K, N, T):
    """Batches whose tiles would not fill the chip (128x128 up to 1024 rows; 256x256 above, for a long contraction axis
    into few columns) go through the GEMM split along K (fp32 partial outputs, a
    second launch that sums them in order, adds the adapter term and rounds once): ragged N, a last stretch of K
    that ends in a partial stage, rows without an adapter, short and long segments -- against the oracle, against the
    unsplit path, with and without an adapter table, and bit-equal from run to run."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options, tol
    reset_options()
    rng = np.random.default_rng(T + K)
    ranks = (8, 16, 64, 40, 8, 24, 128)
    lens, ids = [], []
    left = T
    while left > 0:
        n = int(min(left, rng.choice([1, 1, 2, 7, 33, 90])))
        lens.append(n)
        ids.append(int(rng.integers(-1, len(ranks))))
        left -= n
    wl = make_custom(seed=300 + T, dtype=dtype, K=K, N=N, ranks=ranks, scales=(2.0, 0.5, 1.0, 0.25, 1.5, 1.0, 0.75),
                     req_adapter=np.asarray(ids), req_ntok=np.asarray(lens), name=f"split_k_{dtype}_{K}_{N}_{T}")
    assert wl.T == T
    from gpu_common import B
    code = 1 if dtype == "bf16" else 0
    out = {}
    for split in (-1, 0):
        ctx().set_option("gemm_split_k", split)
        assert ("splitk" in B.lora_gemm_kernel_name(ctx().handle, T, K, N, code)) == (split == -1)
        out[split] = gpu_linear(wl, device_plan=bool(T & 1))
        e = check_against_oracle(wl, out[split])
    again = gpu_linear(wl, device_plan=bool(T & 1))
    ctx().set_option("gemm_split_k", -1)
    again = gpu_linear(wl, device_plan=bool(T & 1))
    assert np.array_equal(again, out[-1])
    rms = float(np.sqrt((out[0] ** 2).mean()))
    assert float(np.abs(out[0] - out[-1]).max()) <= tol(dtype, K) * rms
    assert not np.array_equal(out[0], out[-1]) or dtype == "bf16"  # (fp32: another summation order shows in the last bits)
    print(f"{wl.name}: err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("T,n_proj", [(1, 2), (9, 3), (24, 4), (50, 3), (90, 2), (128, 3)])
def test_decode_sized_multi_projections(T, n_proj):
    """lora_linear_multi on decode-sized bf16 batches: projections of different widths (one ragged, one without
    adapters), several K slices with a ragged last one -- each output against the oracle, and bit-equal to the
    single-projection call (the same partial tiles summed in the same order)."""
    import torch
    from workloads.configs import Projection
    from gpu_common import rt, ctx, check_against_oracle, reset_options
    from workloads import to_f64
    c = ctx()
    reset_options()
    rng = np.random.default_rng(77 + T)
    ranks = (8, 16, 64, 40, 8, 24, 32, 48, 128)
    ids = rng.integers(-1, len(ranks), size=T)
    wl = make_custom(seed=1200 + T, dtype="bf16", K=1288, N=520, ranks=ranks, scales=tuple(0.5 + 0.25 * i for i in range(len(ranks))),
                     req_adapter=ids, req_ntok=np.ones(T, np.int64), name=f"decode_multi_{T}")
    widths = [520, 264, 1100, 48][:n_proj]
    wl.projections = [Projection(chr(97 + q), 1288, n) for q, n in enumerate(widths)]
    wl.shared_x = True
    dev = c.device
    up = [rt.upload_workload(wl, q, dev) for q in range(n_proj)]
    X = up[0][0]
    pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks, wl.r_max)
    bare = 1  # this projection goes without its adapter table
    for mode in (0, -1):  # 0: the reduction's own expand whatever the adapter work (the fused launches at every size)
        c.set_option("expand_split", mode)
        outs = rt.linear_multi(c, pl, X, [(u[1], None if q == bare else u[2]) for q, u in enumerate(up)])
        torch.cuda.synchronize()
        for q in range(n_proj):
            got = rt.bits_from_tensor(outs[q])
            single = rt.bits_from_tensor(rt.linear(c, pl, X, up[q][1], None if q == bare else up[q][2]))
            torch.cuda.synchronize()
            assert np.array_equal(got, single), f"projection {q}"
            if q != bare:
                e = check_against_oracle(wl, to_f64(got), p=q)
    reset_options()
    assert pl.status(c)[0] == 0
    print(f"{wl.name}: T={T} n_proj={n_proj} err/rms {e:.2e}", flush=True)


@pytest.mark.parametrize("T", [1, 5, 16, 17, 32, 33, 64, 73, 100, 128])
def test_decode_path_row_counts(T):
    """Decode-sized batches of one-token requests (1, ..., 73 = the paper's peak batch, ..., 128): every
    instantiation of the two decode kernels, ragged N (200 = 12.5 blocks of 16 columns) and K (520 = one whole slice
    of 512 and a slice of one chunk), workgroups of 8 to 12 waves."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options, B
    rng = np.random.default_rng(T)
    n_ad = 12
    ids = rng.integers(-1, n_ad, size=T)
    wl = make_custom(seed=40 + T, dtype="bf16", K=520, N=200, ranks=rng.choice([8, 16, 32], size=n_ad),
                     scales=rng.choice([0.5, 1.0, 2.0], size=n_ad), req_adapter=ids, req_ntok=np.ones(T, int),
                     name=f"decode_T{T}")
    assert B.lora_gemm_kernel_name(ctx().handle, T, 520, 200, B.LORA_DTYPE_BF16).startswith("decode")
    for nb in (8, 10, 12, -1):
        ctx().set_option("decode_waves", nb if T <= 64 else -1)  # (more than 64 rows: always 8 waves)
        Y = gpu_linear(wl, device_plan=(nb == 10))
        e = check_against_oracle(wl, Y)
    print(f"{wl.name}: err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("T", [3, 70])
def test_decode_kernels_long_contraction_axis(T):
    """K of a down projection (11016 = 172 stages of 64 + one chunk): more than one W0 window per wave in the
    decode GEMM, many load batches per wave in the shrink, rows of X too long to be staged in LDS; ranks up
    to 128 (several rank blocks per unit)."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options
    rng = np.random.default_rng(900 + T)
    ranks = (8, 128, 64, 16)
    ids = rng.integers(-1, len(ranks), size=T)
    wl = make_custom(seed=500 + T, dtype="bf16", K=11016, N=40, ranks=ranks, scales=(1.0, 0.5, 2.0, 1.0),
                     req_adapter=ids, req_ntok=np.ones(T, int), name=f"long_k_T{T}")
    for rb in (-1, 64):
        ctx().set_option("shrink_rank_block", rb)
        e = check_against_oracle(wl, gpu_linear(wl, device_plan=True))
    print(f"{wl.name}: err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("K", [64, 128])
def test_adapter_dominated_output_at_the_default_distributions(K):
    """Short contraction axis, rank 64, s = 2, B ~ N(0, 0.02): the adapter term (RMS 0.32) is the larger part of Y
    (backbone part 0.16-0.23).  Decode-sized and tiled paths, adapter term fused and separate."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options
    for T_per, tag in ((3, "decode"), (40, "tiled")):
        ids = np.arange(12) % 3
        wl = make_custom(seed=7000 + K, dtype="bf16", K=K, N=512, ranks=(64, 64, 64), scales=(2.0, 2.0, 2.0),
                         req_adapter=ids, req_ntok=np.full(12, T_per), name=f"adapter_dominated_{tag}_K{K}")
        for split in ((-1,) if T_per == 3 else (0, 1)):
            ctx().set_option("expand_split", split)
            e = check_against_oracle(wl, gpu_linear(wl, device_plan=True))
            print(f"{wl.name} split={split}: T={wl.T} err/rms {e:.2e}", flush=True)
    reset_options()


def test_decode_path_equals_tile_path_within_tolerance_and_tile_handles_small_T():
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options
    ids, L = _mixed_batch(8, R=20, n_ad=5, max_len=6)
    wl = make_custom(seed=77, dtype="bf16", K=1024, N=512, ranks=(16, 8, 32, 16, 64), scales=(1.0, 2.0, 0.5, 1.0, 1.0),
                     req_adapter=ids, req_ntok=L, name="small_T_both_paths")
    assert wl.T <= 128
    ctx().set_option("decode_max_rows", 0)  # force the tiled kernel
    check_against_oracle(wl, gpu_linear(wl))
    reset_options()
    check_against_oracle(wl, gpu_linear(wl))


def test_shrink_stage_matches_oracle_intermediate():
    """Step a2 alone: V = s_a X A_a, one row per token row (bf16 path: rounded once to bf16)."""
    import torch
    from gpu_common import ctx, gpu_linear, rt
    from oracle import oracle_workload
    for dtype, tol in (("bf16", 2 ** -8), ("f32", 1e-5)):
        ids, L = _mixed_batch(12, R=30, n_ad=5, max_len=90)
        wl = make_custom(seed=5, dtype=dtype, K=456, N=64, ranks=(8, 72, 16, 128, 32), scales=(2.0, 0.5, 1.0, 0.25, 1.5),
                         req_adapter=ids, req_ntok=L, name=f"shrink_{dtype}")
        _, (X, W0, table, pl, Y) = gpu_linear(wl, stage="shrink", return_all=True)
        c = ctx()
        ws = rt.workspace(wl.T, 456, 64, wl.r_max, X.dtype, X.device)
        rt.linear(c, pl, X, W0, table, Y=Y, ws=ws, stage="shrink")
        torch.cuda.synchronize()
        es = 2 if dtype == "bf16" else 4
        vbytes = ws[: wl.T * wl.r_max * es]
        Vg = vbytes.view(torch.bfloat16 if dtype == "bf16" else torch.float32).reshape(wl.T, wl.r_max)
        Vg = to_f64(rt.bits_from_tensor(Vg))
        _, Vo = oracle_workload(wl, return_v=True)
        ra = wl.row_adapter()
        worst = 0.0
        for row in range(wl.T):  # V is stored in original row order
            a = ra[row]
            if a < 0:
                continue
            r = int(wl.ranks[a])
            want = float(wl.scales[a]) * Vo[row, :r]
            scale = max(np.abs(want).max(), 1e-3)
            worst = max(worst, np.abs(Vg[row, :r] - want).max() / scale)
        assert worst <= tol, (dtype, worst)
        print(f"shrink {dtype}: worst rel err {worst:.2e}", flush=True)


def test_zero_b_reproduces_base_and_no_table_equals_all_minus_one():
    """Zero-B adapters give exactly the backbone product; so do tbl = NULL and ids = -1 (bitwise on GPU)."""
    import torch
    from gpu_common import ctx, rt
    from paper_2505_14468_amd.runtime import tensor_from_bits, bits_from_tensor
    c = ctx()
    for T in (40, 400):
        ids = np.arange(10) % 4
        L = np.full(10, T // 10)
        wl = make_custom(seed=9, dtype="bf16", K=256, N=192, ranks=(8, 16, 8, 32), scales=(1.0,) * 4,
                         req_adapter=ids, req_ntok=L)
        X, W0, table = rt.upload_workload(wl, 0, c.device)
        for b in table.B:
            b.zero_()
        pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks)
        Y0 = bits_from_tensor(rt.linear(c, pl, X, W0, table))
        Y1 = bits_from_tensor(rt.linear(c, pl, X, W0, None))
        pl2 = rt.plan(c, np.full(10, -1), wl.req_ntok, wl.ranks)
        Y2 = bits_from_tensor(rt.linear(c, pl2, X, W0, table))
        torch.cuda.synchronize()
        assert np.array_equal(Y1, Y2)
        assert np.array_equal(to_f64(Y0), to_f64(Y1))  # +0 contributions: equal as values


def test_determinism_w0_untouched_and_permutation_invariance():
    import torch
    from gpu_common import ctx, rt, reset_options
    from paper_2505_14468_amd.runtime import bits_from_tensor
    c = ctx()
    for T_scale, opts in ((1, {}), (12, {})):
        rng = np.random.default_rng(T_scale)
        R, n_ad = 24, 6
        ids = rng.integers(-1, n_ad, size=R)
        L = rng.integers(1, 4, size=R) * T_scale
        wl = make_custom(seed=123, dtype="bf16", K=512, N=384, ranks=(8, 16, 32, 64, 16, 8), scales=(1.0, 2.0, 0.5, 1.0, 1.0, 2.0),
                         req_adapter=ids, req_ntok=L)
        X, W0, table = rt.upload_workload(wl, 0, c.device)
        frozen = [t.clone() for t in [W0, X] + table.A + table.B]
        pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks)
        Y1 = bits_from_tensor(rt.linear(c, pl, X, W0, table))
        Y2 = bits_from_tensor(rt.linear(c, pl, X, W0, table))
        assert np.array_equal(Y1, Y2), "run-to-run results differ"
        for before, after in zip(frozen, [W0, X] + table.A + table.B):
            assert torch.equal(before, after), "an input tensor was written"
        # permute the requests (and X's row blocks): output row blocks permute with them
        off = np.concatenate([[0], np.cumsum(L)])
        order = rng.permutation(R)
        rows = np.concatenate([np.arange(off[i], off[i + 1]) for i in order])
        Xp = X[torch.from_numpy(rows).to(c.device)].contiguous()
        plp = rt.plan(c, ids[order], L[order], wl.ranks)
        Yp = bits_from_tensor(rt.linear(c, plp, Xp, W0, table))
        assert np.array_equal(Yp, Y1[rows]), "a row's result depends on the order of the batch"
    reset_options()


def test_p5_exact_integers_on_gpu():
    """Small integers, power-of-two scales: every product and sum is exact in bf16 x bf16 -> fp32,
    so the GPU must equal the oracle exactly (|Y| stays representable in bf16)."""
    from gpu_common import gpu_linear
    from oracle import oracle_workload
    for dtype in ("bf16", "f32"):
        wl = make_custom(seed=3, dtype=dtype, K=16, N=8, ranks=(8, 8), scales=(0.5, 0.25),
                         req_adapter=(0, 1, -1, 0), req_ntok=(2, 3, 1, 2), integer_valued=True)
        Y = gpu_linear(wl)
        Yo = oracle_workload(wl)
        if dtype == "bf16":  # one rounding of the exact result to bf16
            from workloads import bf16_bits_from_f32, f32_from_bf16_bits
            Yo = f32_from_bf16_bits(bf16_bits_from_f32(Yo.astype(np.float32))).astype(np.float64)
        assert np.array_equal(Y, Yo), dtype


def _integer_batch(seed, T, n_ad):
    rng = np.random.default_rng(seed)
    lens, ids = [], []
    left = T
    while left > 0:
        n = int(min(left, rng.choice([1, 2, 5, 40, 70, 150])))
        lens.append(n)
        ids.append(int(rng.integers(-1, n_ad)))
        left -= n
    return np.asarray(ids), np.asarray(lens)


@pytest.mark.parametrize("T,K,N,variant", [(150, 1032, 264, None), (300, 2056, 520, None), (1100, 10264, 264, None),
                                           (700, 1000, 300, "tile_64x64"), (700, 1000, 300, "tile_128x128"),
                                           (700, 1000, 300, "tile_256x128"), (700, 1000, 300, "tile_256x256w4"),
                                           (700, 1000, 300, "tile_128x192"), (700, 1000, 300, "tile_256x192"),
                                           (700, 1000, 300, "tile_256x224")])
def test_fp32_integer_inputs_are_exact_on_every_tiled_path(T, K, N, variant):
    """Small integers and power-of-two scales in fp32: every product and every partial sum, in any order, is an
    integer multiple of 1/8 far below 2^24, so shrink, expand kernel, in-GEMM extension, every tile shape and the
    launches split along K must reproduce the oracle bit for bit -- a dropped or doubled piece of the contraction
    axis, of a rank axis or of a segment cannot hide inside a tolerance."""
    from gpu_common import ctx, gpu_linear, reset_options
    from oracle import oracle_workload
    reset_options()
    ranks = (8, 16, 64, 128, 24)
    ids, lens = _integer_batch(T + K, T, len(ranks))
    wl = make_custom(seed=900 + T, dtype="f32", K=K, N=N, ranks=ranks, scales=(0.5, 0.25, 1.0, 0.125, 2.0),
                     req_adapter=ids, req_ntok=lens, name=f"integers_f32_{T}_{K}_{N}_{variant}", integer_valued=True)
    Yo = oracle_workload(wl)
    assert np.abs(Yo).max() < 2 ** 22 and np.array_equal(Yo, Yo.astype(np.float32).astype(np.float64))
    if variant:
        ctx().set_option("gemm_variant", VARIANTS[variant])
    for expand_split in (-1, 0):  # the expand kernel for the short segments where the host picks it / everything in the GEMM
        ctx().set_option("expand_split", expand_split)
        Y = gpu_linear(wl, device_plan=bool(T & 2))
        assert np.array_equal(Y, Yo), (variant, expand_split)
    reset_options()


@pytest.mark.parametrize("variant", [None, "tile_64x64", "tile_128x128", "tile_256x128", "tile_256x256w4", "tile_128x192",
                                     "tile_256x192", "tile_256x224"])
def test_bf16_base_product_integer_inputs_are_exact(variant):
    """The bf16 MFMA base product alone (every request without an adapter), 65 stages of K with a partial last one,
    ragged rows and columns: the exact integer result rounded once to bf16, on every tile shape and split along K."""
    from gpu_common import ctx, gpu_linear, reset_options
    from oracle import oracle_workload
    from workloads import bf16_bits_from_f32, f32_from_bf16_bits
    reset_options()
    T = 700 if variant else 300  # (300 rows: the host's own choice is the launch split along K)
    wl = make_custom(seed=990, dtype="bf16", K=4104, N=300, ranks=(8,), scales=(1.0,), req_adapter=np.full(7, -1),
                     req_ntok=np.asarray([T - 6, 1, 1, 1, 1, 1, 1]), name=f"integers_base_{variant}", integer_valued=True)
    if variant:
        ctx().set_option("gemm_variant", VARIANTS[variant])
    Yo = oracle_workload(wl)
    Yo = f32_from_bf16_bits(bf16_bits_from_f32(Yo.astype(np.float32))).astype(np.float64)
    assert np.array_equal(gpu_linear(wl), Yo)
    reset_options()


@pytest.mark.parametrize("T", [1, 17, 64, 128])
def test_bf16_decode_path_integer_inputs_are_exact(T):
    """The decode path keeps V in fp32, so with small integers and power-of-two scales its result is the exact one,
    rounded once to bf16, at any length of the contraction axis (here 9 slices, the last one partial)."""
    from gpu_common import ctx, gpu_linear, reset_options, B
    from oracle import oracle_workload
    from workloads import bf16_bits_from_f32, f32_from_bf16_bits
    reset_options()
    ranks = (8, 16, 64, 24)
    rng = np.random.default_rng(T)
    ids = rng.integers(-1, len(ranks), size=T)
    wl = make_custom(seed=950 + T, dtype="bf16", K=4104, N=520, ranks=ranks, scales=(0.5, 0.25, 1.0, 2.0),
                     req_adapter=ids, req_ntok=np.ones(T, np.int64), name=f"integers_decode_{T}", integer_valued=True)
    assert B.lora_gemm_kernel_name(ctx().handle, T, 4104, 520, 1).startswith("decode")
    Yo = oracle_workload(wl)
    Yo = f32_from_bf16_bits(bf16_bits_from_f32(Yo.astype(np.float32))).astype(np.float64)
    assert np.array_equal(gpu_linear(wl, device_plan=bool(T & 1)), Yo)


@pytest.mark.parametrize("dtype,T,K", [("f32", 500, 1000), ("f32", 140, 2056), ("bf16", 50, 2056), ("bf16", 128, 1544)])
def test_linear_multi_integer_inputs_are_exact(dtype, T, K):
    """lora_linear_multi on small integers: three projections of one X through the fused launches (fp32: shrink,
    expand and tiled GEMM over the projections side by side; bf16 at up to 128 rows: the decode path's two launches)
    equal the oracle bit for bit (bf16: the exact result rounded once)."""
    import torch
    from workloads.configs import Projection
    from workloads import to_f64, bf16_bits_from_f32, f32_from_bf16_bits
    from oracle import oracle_workload
    from gpu_common import rt, ctx, reset_options
    reset_options()
    c = ctx()
    ranks = (8, 16, 64, 24)
    if dtype == "bf16":
        rng = np.random.default_rng(T)
        ids, lens = rng.integers(-1, len(ranks), size=T), np.ones(T, np.int64)
    else:
        ids, lens = _integer_batch(T, T, len(ranks))
    wl = make_custom(seed=970 + T, dtype=dtype, K=K, N=520, ranks=ranks, scales=(0.5, 0.25, 1.0, 2.0), req_adapter=ids,
                     req_ntok=lens, name=f"multi_integers_{dtype}_{T}", integer_valued=True)
    wl.projections = [Projection("a", K, 520), Projection("b", K, 264), Projection("c", K, 1100)]
    wl.shared_x = True
    up = [rt.upload_workload(wl, q, c.device) for q in range(3)]
    pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks, wl.r_max)
    outs = rt.linear_multi(c, pl, up[0][0], [(u[1], u[2]) for u in up])
    torch.cuda.synchronize()
    for q in range(3):
        Yo = oracle_workload(wl, q)
        if dtype == "bf16":
            Yo = f32_from_bf16_bits(bf16_bits_from_f32(Yo.astype(np.float32))).astype(np.float64)
        assert np.array_equal(to_f64(rt.bits_from_tensor(outs[q])), Yo), q


def test_strided_inputs_and_adapter_eviction():
    """ld > width for X, W0 and Y; a NULL table slot that the batch uses is reported, not dereferenced."""
    import torch
    from gpu_common import ctx, rt, check_against_oracle, B
    from paper_2505_14468_amd.runtime import bits_from_tensor
    c = ctx()
    wl = make_custom(seed=55, dtype="bf16", K=128, N=96, ranks=(8, 16), scales=(1.0, 2.0),
                     req_adapter=(0, 1, 0), req_ntok=(30, 50, 70))
    X, W0, table = rt.upload_workload(wl, 0, c.device)
    Xs = torch.zeros((wl.T, 128 + 64), dtype=X.dtype, device=c.device)
    Xs[:, :128] = X
    Ws = torch.zeros((96, 128 + 8), dtype=X.dtype, device=c.device)
    Ws[:, :128] = W0
    Ys = torch.full((wl.T, 96 + 32), 3.0, dtype=X.dtype, device=c.device)
    pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks)
    rt.linear(c, pl, Xs[:, :128], Ws[:, :128], table, Y=Ys[:, :96])
    torch.cuda.synchronize()
    check_against_oracle(wl, to_f64(bits_from_tensor(Ys[:, :96])))
    assert bool((Ys[:, 96:] == 3.0).all()), "wrote outside Y's N columns"
    # evict adapter 1 after planning: the kernels skip it and record ADAPTER_NOT_RESIDENT
    table.set_slot(1, None, None)
    rt.linear(c, pl, X, W0, table)
    status, _ = pl.status(c)
    assert status == B.LORA_ERR_ADAPTER_NOT_RESIDENT


@pytest.mark.parametrize("T", [5, 40, 100, 128])
def test_decode_path_adapter_term_through_the_expand_kernel(T):
    """Decode-sized batches with much adapter work: V reduced by a launch of its own, the term by the expand kernel,
    added by the reduction -- against the oracle and against the reduction's own expand, forced either way."""
    from gpu_common import ctx, gpu_linear, check_against_oracle, reset_options, TOL
    reset_options()
    rng = np.random.default_rng(40 + T)
    ranks = (128, 8, 64, 16, 40, 128)
    ids = rng.integers(-1, len(ranks), size=T)
    wl = make_custom(seed=500 + T, dtype="bf16", K=1288, N=1100, ranks=ranks, scales=(0.5, 2.0, 1.0, 1.0, 0.25, 0.75),
                     req_adapter=ids, req_ntok=np.ones(T, np.int64), name=f"decode_heavy_{T}")
    out = {}
    for mode in (1, 0, -1):
        ctx().set_option("expand_split", mode)
        out[mode] = gpu_linear(wl, device_plan=bool(T & 1))
        e = check_against_oracle(wl, out[mode])
    rms = float(np.sqrt((out[0] ** 2).mean()))
    assert float(np.abs(out[0] - out[1]).max()) <= 2 * TOL["bf16"] * rms  # (each within TOL of the oracle)
    assert not np.array_equal(out[0], out[1])  # (V rounded to bf16 on the one path, kept in fp32 on the other)
    ctx().set_option("expand_split", 1)
    assert np.array_equal(gpu_linear(wl, device_plan=bool(T & 1)), out[1])
    print(f"{wl.name}: err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("T,K,heavy", [(20, 264, 0), (20, 264, 1), (200, 2312, 0), (700, 264, 0)])
def test_largest_rank_and_eviction_on_every_path(T, K, heavy):
    """Adapters of the largest rank the library takes (512) beside small ones, on the decode path (20 rows), the GEMM
    split along K (200 rows) and the tiled GEMM (700 rows); then one used adapter is evicted after planning: every
    path reports it, the rows of the other adapters keep their results."""
    import torch
    from gpu_common import ctx, rt, check_against_oracle, B, reset_options
    from paper_2505_14468_amd.runtime import bits_from_tensor
    reset_options()
    c = ctx()
    if heavy:
        c.set_option("expand_split", 1)  # (decode path: the adapter term through the expand kernel)
    rng = np.random.default_rng(T)
    ranks = (512, 8, 256, 16)
    lens = [1, 2, 3, 1]  # every adapter in use
    left = T - sum(lens)
    while left > 0:
        n = int(min(left, rng.choice([1, 3, 40])))
        lens.append(n)
        left -= n
    ids = rng.integers(-1, len(ranks), size=len(lens))
    ids[:4] = (0, 1, 2, 3)
    wl = make_custom(seed=77 + T, dtype="bf16", K=K, N=328, ranks=ranks, scales=(0.05, 2.0, 0.1, 1.0), req_adapter=ids,
                     req_ntok=np.asarray(lens), name=f"rank512_T{T}")
    X, W0, table = rt.upload_workload(wl, 0, c.device)
    pl = rt.plan(c, wl.req_adapter, wl.req_ntok, wl.ranks)
    Y = rt.linear(c, pl, X, W0, table)
    torch.cuda.synchronize()
    full = to_f64(bits_from_tensor(Y))
    e = check_against_oracle(wl, full)
    assert pl.status(c)[0] == 0
    table.set_slot(2, None, None)
    Y2 = rt.linear(c, pl, X, W0, table)
    torch.cuda.synchronize()
    assert pl.status(c)[0] == B.LORA_ERR_ADAPTER_NOT_RESIDENT
    part = to_f64(bits_from_tensor(Y2))
    row_ad = np.repeat(wl.req_adapter, wl.req_ntok)
    keep = row_ad != 2
    assert np.array_equal(part[keep], full[keep]), "rows of resident adapters changed"
    base = to_f64(bits_from_tensor(rt.linear(c, pl, X, W0, None)))
    torch.cuda.synchronize()
    rms = float(np.sqrt((base ** 2).mean()))
    assert float(np.abs(part[~keep] - base[~keep]).max()) <= 2e-2 * rms, "rows of the evicted adapter: the base product alone"
    print(f"{wl.name}: {B.lora_gemm_kernel_name(c.handle, T, K, 328, 1)} err/rms {e:.2e}", flush=True)
    reset_options()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_worked_example_derived_by_hand_is_exact(dtype):
    """tests/golden/worked_example.json: three rows, one adapter, every number exactly representable -- the GPU's
    output equals the hand-derived Y exactly, through the decode-sized kernel (bf16) and the tiled one (fp32, and
    bf16 when forced)."""
    import json
    import os
    import torch
    from workloads.bits import bf16_bits_from_f32
    from gpu_common import rt, ctx, reset_options
    fx = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")))
    conv = (lambda a: bf16_bits_from_f32(np.asarray(a, np.float32))) if dtype == "bf16" else (lambda a: np.asarray(a, np.float32))
    c = ctx()
    dev = c.device
    X, W0 = rt.tensor_from_bits(conv(fx["X"]), dev), rt.tensor_from_bits(conv(fx["W0"]), dev)
    table = rt.AdapterTable([rt.tensor_from_bits(conv(fx["A0"]), dev)], [rt.tensor_from_bits(conv(fx["B0"]), dev)],
                            np.asarray(fx["scale"], np.float32), dev)
    pl = rt.plan(c, np.asarray(fx["req_adapter"], np.int32), np.asarray(fx["req_ntok"], np.int32), np.asarray(fx["rank"], np.int32), 8)
    for variant in (None, "tile_64x64", "tile_128x192"):
        c.set_option("gemm_variant", VARIANTS[variant] if variant else -1)
        Y = rt.linear(c, pl, X, W0, table)
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(rt.bits_from_tensor(Y)), np.asarray(fx["Y"], np.float64)), variant
    reset_options()


def test_layer_at_the_most_requests_and_adapter_slots():
    """65536 one- and two-token requests on 65536 adapter slots (the header's maxima): ~98 000 rows, tens of thousands
    of shrink units, 384 row tiles.  Small integers and power-of-two scales on a short contraction axis, so that every
    intermediate is exact (V <= 256 in bf16) and the 7 million outputs must equal the oracle's, rounded once to bf16,
    bit for bit -- a maximum error over that many Gaussian outputs would sit at the bf16 format's own rounding of the
    largest of them (5.8 x RMS: 1.7e-2 x RMS)."""
    from gpu_common import gpu_linear, reset_options
    from oracle import oracle_workload
    from workloads import bf16_bits_from_f32, f32_from_bf16_bits
    reset_options()
    rng = np.random.default_rng(12)
    R = n_ad = 65536
    ranks = rng.choice([8, 16], size=n_ad)
    ids = rng.permutation(n_ad)
    ids[rng.integers(0, R, size=300)] = -1
    lens = rng.integers(1, 3, size=R)
    wl = make_custom(seed=4242, dtype="bf16", K=16, N=72, ranks=ranks, scales=rng.choice([0.25, 0.5], size=n_ad),
                     req_adapter=ids, req_ntok=lens, name="max_requests_and_slots", integer_valued=True)
    Y = gpu_linear(wl, device_plan=True)
    Yo = oracle_workload(wl)
    Yo = f32_from_bf16_bits(bf16_bits_from_f32(Yo.astype(np.float32))).astype(np.float64)
    assert Y.shape == Yo.shape and np.array_equal(Y, Yo)
    assert np.abs(Yo).max() > 100  # (the adapter term is there)


def test_empty_batch_is_a_noop():
    import torch
    from gpu_common import ctx, rt
    c = ctx()
    pl = rt.plan(c, [0, 1], [0, 0], [8, 8])
    X = torch.zeros((0, 64), dtype=torch.bfloat16, device=c.device)
    W0 = torch.zeros((32, 64), dtype=torch.bfloat16, device=c.device)
    Y = rt.linear(c, pl, X, W0, None)
    torch.cuda.synchronize()
    assert Y.shape == (0, 32)
