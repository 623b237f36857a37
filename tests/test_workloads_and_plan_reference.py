"""The seeded input generator and the reference segment table."""
import numpy as np
import pytest

from oracle import plan_reference
from workloads import bf16_bits_from_f32, f32_from_bf16_bits, make_workload


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0, 3.1415926], np.float32)
    b = bf16_bits_from_f32(f)
    back = f32_from_bf16_bits(b)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: goes to the even mantissa (1.0)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.0 + 2 ** -7)
    # 1 + 3*2^-8 is a tie between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    assert back[3] == np.float32(1.0 + 2 ** -6)
    assert back[4] == -2.5 and back[5] == 0.0
    assert abs(back[6] - f[6]) <= 2 ** -8 * abs(f[6])
    # representable values survive
    assert np.array_equal(bf16_bits_from_f32(back), b)


def test_config_shapes_and_determinism():
    want = {0: (128, 16, 4, "f32"), 1: (64, 64, 32, "bf16"), 3: (1216, 196, 100, "bf16"), 4: (2048, 512, 512, "bf16")}
    for idx, (T, R, n_ad, dt) in want.items():
        wl = make_workload(idx)
        assert (wl.T, wl.n_req, wl.n_adapters, wl.dtype) == (T, R, n_ad, dt)
        wl2 = make_workload(idx)
        assert np.array_equal(wl.req_adapter, wl2.req_adapter) and np.array_equal(wl.req_ntok, wl2.req_ntok)
    wl = make_workload(2)
    assert wl.n_req == 16 and wl.req_ntok.min() >= 128 and wl.req_ntok.max() <= 1024
    wl = make_workload(4)
    assert wl.req_ntok.min() >= 1 and wl.req_adapter.min() >= 0 and wl.req_adapter.max() < 512
    # bounded Zipf: id 0 is the most frequent
    assert np.bincount(wl.req_adapter).argmax() == 0
    wl = make_workload(3)
    assert set(np.unique(wl.ranks)) <= {8, 16, 32, 64}
    assert np.allclose(wl.scales * wl.ranks, 16.0)
    assert sorted(wl.req_ntok.tolist())[-4:] == [256] * 4
    a = make_workload(1).A(5)
    assert a.shape == (16, 4096) and a.dtype == np.uint16
    assert np.array_equal(a, make_workload(1).A(5))
    assert not np.array_equal(a, make_workload(1).A(6))
    std = f32_from_bf16_bits(a).std()
    assert abs(std - 1 / 64) / (1 / 64) < 0.02


def _brute_plan(req_adapter, req_ntok, ranks):
    n_ad = len(ranks)
    rows = []
    t = 0
    for a, L in zip(req_adapter, req_ntok):
        for _ in range(L):
            rows.append((n_ad if a < 0 else a, t))
            t += 1
    rows.sort()  # (key, original row): ties broken by original position = stable
    perm = [t for _, t in rows]
    segs, indptr = [], []
    for slot, (k, _) in enumerate(rows):
        if not segs or segs[-1] != k:
            segs.append(k)
            indptr.append(slot)
    indptr.append(len(rows))
    return perm, [(-1 if k == n_ad else k) for k in segs], indptr


@pytest.mark.parametrize("seed", range(6))
def test_plan_reference_against_brute_force(seed):
    rng = np.random.default_rng(seed)
    n_ad = int(rng.integers(1, 7))
    R = int(rng.integers(0, 12))
    ranks = rng.choice([8, 16, 32], size=n_ad)
    ids = rng.integers(-1, n_ad, size=R)
    L = rng.integers(0, 5, size=R)
    ref = plan_reference(ids, L, ranks)
    perm, segs, indptr = _brute_plan(ids.tolist(), L.tolist(), ranks.tolist())
    assert ref["perm"].tolist() == perm
    assert ref["seg_adapter"].tolist() == segs
    assert ref["seg_indptr"].tolist() == indptr
    assert ref["n_seg"] == len(segs)
    want_rank = [0 if a < 0 else int(ranks[a]) for a in segs]
    assert ref["seg_rank"].tolist() == want_rank
    assert ref["seg_ext"].tolist() == [0] + np.cumsum(want_rank).astype(int).tolist()
    for slot in range(len(perm)):
        s = ref["row_seg"][slot]
        assert indptr[s] <= slot < indptr[s + 1]
