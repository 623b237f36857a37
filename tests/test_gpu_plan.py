"""GPU parity of step a1, the device-side segment builder, against the stable-sort reference
(bit-exact: integer work)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _check_plan(ids, L, ranks, device_plan, fused_rows=-1, plan_variant=-1):
    import torch
    from gpu_common import ctx, rt, plan_reference
    c = ctx()
    c.set_option("plan_fused_rows", fused_rows)
    c.set_option("plan_variant", plan_variant)
    ids, L, ranks = np.asarray(ids, np.int32), np.asarray(L, np.int32), np.asarray(ranks, np.int32)
    r_max = int(ranks.max()) if ranks.size else 0
    if device_plan:
        dev = c.device
        mk = lambda a: torch.from_numpy(a if a.size else np.zeros(1, np.int32)).to(dev)[: a.size].contiguous()
        pl = rt.plan_device(c, mk(ids), mk(L), mk(ranks), r_max, int(L.sum()))
    else:
        pl = rt.plan(c, ids, L, ranks, r_max)
    got = pl.to_host(c)
    c.set_option("plan_fused_rows", -1)
    c.set_option("plan_variant", -1)
    assert got["status"] == 0
    ref = plan_reference(ids, L, ranks)
    assert got["n_seg"] == ref["n_seg"]
    for k in ("perm", "row_seg", "seg_adapter", "seg_indptr", "seg_rank", "seg_ext"):
        assert np.array_equal(got[k], ref[k]), k
    assert got["ext_total"] == int(ref["seg_ext"][-1])
    assert np.array_equal(got["row_adapter"], np.repeat(ids, L))
    # derived tables: shrink work list and one record per 8 ranks
    rows = np.diff(ref["seg_indptr"])
    ur = got["unit_rows"]  # 16 for plans of few rows and segments (they then fill more of the chip), else 64
    seg_bound = min(len(ids), len(ranks), int(L.sum()))
    assert ur == (16 if int(L.sum()) // 16 + seg_bound <= 256 else 64)  # (256 CUs)
    units = np.where(ref["seg_adapter"] >= 0, (rows + ur - 1) // ur, 0)
    assert np.array_equal(got["seg_unit"], np.concatenate([[0], np.cumsum(units)]))
    want_units = []
    for s in range(ref["n_seg"]):
        if ref["seg_adapter"][s] < 0:
            continue
        for slot0 in range(int(ref["seg_indptr"][s]), int(ref["seg_indptr"][s + 1]), ur):
            long_flag = 0x10000 if int(ref["seg_indptr"][s + 1]) - int(ref["seg_indptr"][s]) >= 64 else 0
            want_units.append([int(ref["seg_adapter"][s]), int(ref["seg_rank"][s]) | long_flag, slot0,
                               min(ur, int(ref["seg_indptr"][s + 1]) - slot0)])
    assert got["unit_rec"].tolist() == want_units
    rec = got["ext_rec"]
    q = 0
    for s in range(ref["n_seg"]):
        for j0 in range(0, int(ref["seg_rank"][s]), 8):
            assert rec[q].tolist() == [int(ref["seg_adapter"][s]), (int(ref["seg_rank"][s]) << 16) | j0,
                                       int(ref["seg_indptr"][s]), int(ref["seg_indptr"][s + 1])]
            q += 1
    assert q == rec.shape[0]
    assert np.array_equal(got["tok_off"], np.concatenate([[0], np.cumsum(L)]))
    # per row (original order): first extension column of its adapter and its rank, packed
    seg_of_row = np.empty(len(ref["perm"]), np.int64)
    seg_of_row[ref["perm"]] = ref["row_seg"]
    want = ((ref["seg_ext"][:-1][seg_of_row] >> 3) << 7) | (ref["seg_rank"][seg_of_row] >> 3)
    assert np.array_equal(got["row_ext"], want.astype(np.int32))


@pytest.mark.parametrize("device_plan", [False, True])
@pytest.mark.parametrize("seed", range(4))
def test_plan_random(seed, device_plan):
    rng = np.random.default_rng(100 + seed)
    n_ad = int(rng.integers(1, 40))
    R = int(rng.integers(1, 300))
    ranks = rng.choice([8, 16, 32, 64], size=n_ad)
    ids = rng.integers(-1, n_ad, size=R)
    L = rng.integers(0, 9, size=R)
    _check_plan(ids, L, ranks, device_plan)                 # LDS-resident small-batch kernel
    _check_plan(ids, L, ranks, device_plan, fused_rows=0)   # general kernels (segments + grid-wide fill)


@pytest.mark.parametrize("seed", range(6))
def test_plan_decode_sized_batches(seed):
    """At most 64 requests: the one-lane-per-request kernel, against the reference and with the same
    batch through the other kernels (plan_variant=1)."""
    rng = np.random.default_rng(300 + seed)
    n_ad = int(rng.choice([1, 3, 32, 200, 5000]))
    R = int(rng.choice([1, 2, 17, 63, 64]))
    ranks = rng.choice([8, 16, 24, 64], size=n_ad)
    ids = rng.integers(-1, n_ad, size=R)
    if seed % 2 == 0:
        ids[rng.integers(0, R, size=R // 2)] = ids[0]  # repeated keys: several requests per segment
    L = rng.integers(0, 3, size=R) if seed < 3 else rng.integers(0, 60, size=R)  # decode-like / short prefills
    for variant in (-1, 1):
        _check_plan(ids, L, ranks, True, plan_variant=variant)
        _check_plan(ids, L, ranks, False, plan_variant=variant)


@pytest.mark.parametrize("seed", range(8))
def test_plan_65_to_128_requests(seed):
    """65..128 requests: the one-lane-per-request kernel on all 16 waves, against the reference and with the
    same batch through the general kernels (plan_variant=1); larger batches for the general kernels alone."""
    rng = np.random.default_rng(700 + seed)
    n_ad = int(rng.choice([1, 2, 7, 100, 300, 3000]))
    R = int(rng.choice([65, 73, 100, 127, 128, 129, 200, 256]))
    ranks = rng.choice([8, 16, 24, 64], size=n_ad)
    ids = rng.integers(-1, n_ad, size=R)
    if seed % 2 == 0:
        ids[rng.integers(0, R, size=R // 2)] = ids[0]  # one long segment: several shrink units
    L = rng.integers(0, 3, size=R) if seed < 4 else rng.integers(0, 30, size=R)
    for variant in (-1, 1):
        _check_plan(ids, L, ranks, True, plan_variant=variant)
        _check_plan(ids, L, ranks, False, plan_variant=variant)


@pytest.mark.parametrize("fused_rows", [0, 1 << 20])
def test_plan_both_fill_paths_and_many_requests(fused_rows):
    rng = np.random.default_rng(5)
    n_ad, R = 700, 5000  # more than one 1024-wide scan chunk of requests; many 64-request waves
    ranks = rng.choice([8, 16], size=n_ad)
    ids = rng.integers(-1, n_ad, size=R)
    L = rng.integers(0, 4, size=R)
    _check_plan(ids, L, ranks, False, fused_rows=fused_rows)


@pytest.mark.parametrize("device_plan", [False, True])
def test_plan_at_the_documented_maxima(device_plan):
    """LORA_MAX_REQUESTS requests on LORA_MAX_ADAPTERS adapter slots, ranks from 8 to LORA_MAX_RANK, almost every
    request its own segment."""
    rng = np.random.default_rng(11)
    R = n_ad = 65536
    ranks = rng.choice([8, 16, 512], size=n_ad, p=[0.6, 0.39, 0.01])
    ids = rng.permutation(n_ad).astype(np.int32)
    ids[rng.integers(0, R, size=500)] = -1
    ids[rng.integers(0, R, size=500)] = ids[7]
    L = rng.integers(0, 3, size=R)
    _check_plan(ids, L, ranks, device_plan)


def test_plan_edge_cases():
    _check_plan([], [], [8, 8], False)                      # empty batch
    _check_plan([0, 1], [0, 0], [8, 8], True)               # only zero-length requests
    _check_plan([-1, -1], [3, 2], [8], False)               # nobody uses an adapter
    _check_plan([2, 2, 2], [1, 70, 130], [8, 8, 16], True)  # one adapter, several shrink units
    _check_plan([0] * 200, [1] * 200, [8], False)           # same key in every lane of a wave
    _check_plan(list(range(64)) * 2, [1] * 128, [8] * 64, True)
    # benchmark configurations
    from workloads import make_workload
    for idx in (1, 3, 4):
        wl = make_workload(idx)
        _check_plan(wl.req_adapter, wl.req_ntok, wl.ranks, idx % 2 == 0)


def test_plan_device_reports_errors_in_status_word():
    import torch
    from gpu_common import ctx, rt, B
    c = ctx()
    dev = c.device
    t = lambda a: torch.tensor(a, dtype=torch.int32, device=dev)
    cases = [
        (([0, 5], [1, 1], [8, 8], 8, 2), B.LORA_ERR_BAD_ADAPTER_ID),
        (([0, 1], [1, -1], [8, 8], 8, 0), B.LORA_ERR_LENGTH_MISMATCH),
        (([0, 1], [1, 1], [8, 8], 8, 3), B.LORA_ERR_LENGTH_MISMATCH),
        (([0, 1], [1, 1], [8, 0], 8, 2), B.LORA_ERR_ADAPTER_NOT_RESIDENT),
        (([0, 1], [1, 1], [8, 16], 8, 2), B.LORA_ERR_RANK_TOO_LARGE),
        (([0, 1], [1, 1], [8, 12], 16, 2), B.LORA_ERR_SHAPE),
    ]
    cases.append((([0, 5, 1], [1, 1, -1], [8, 8], 8, 1), B.LORA_ERR_LENGTH_MISMATCH))  # two faults: the smaller code
    # the same kinds of fault in a batch of 150 requests, each in the last group of 64
    many = lambda bad_id, bad_len: ([0] * 140 + [bad_id] + [1] * 9, [1] * 145 + [bad_len] + [1] * 4)
    cases.append(((*many(7, 1), [8, 8], 8, 150), B.LORA_ERR_BAD_ADAPTER_ID))
    cases.append(((*many(1, -1), [8, 8], 8, 148), B.LORA_ERR_LENGTH_MISMATCH))
    cases.append(((*many(1, 1), [8, 8], 8, 151), B.LORA_ERR_LENGTH_MISMATCH))
    cases.append(((*many(1, 1), [8, 0], 8, 150), B.LORA_ERR_ADAPTER_NOT_RESIDENT))
    cases.append(((*many(1, 1), [8, 16], 8, 150), B.LORA_ERR_RANK_TOO_LARGE))
    for (ids, L, ranks, r_max, T), want in cases:
        for variant in (1, -1):  # other kernels, then the decode-sized one
            c.set_option("plan_variant", variant)
            pl = rt.plan_device(c, t(ids), t(L), t(ranks), r_max, T)
            status, n_seg = pl.status(c)
            assert status == want and n_seg == 0, (ids, L, ranks, status, variant)
        c.set_option("plan_variant", -1)
        # a failed plan makes the layer a no-op: Y keeps its contents, nothing faults
        X = torch.zeros((T, 64), dtype=torch.bfloat16, device=dev)
        W0 = torch.zeros((32, 64), dtype=torch.bfloat16, device=dev)
        A = [torch.zeros((max(r, 8), 64), dtype=torch.bfloat16, device=dev) for r in ranks]
        Bw = [torch.zeros((32, max(r, 8)), dtype=torch.bfloat16, device=dev) for r in ranks]
        table = rt.AdapterTable(A, Bw, [1.0] * len(ranks), dev)
        Y = torch.full((T, 32), 7.0, dtype=torch.bfloat16, device=dev)
        if T > 0:
            rt.linear(c, pl, X, W0, table, Y=Y)
            torch.cuda.synchronize()
            assert bool((Y == 7.0).all())
