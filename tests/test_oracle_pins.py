"""Pins of the CPU oracle against what the definition and the mathematics fix.

The layer (paper sections 2.2 / 4.4 / 5: backbone and adapter products computed
separately, then summed) has an exact definition, so every pin below is either
exact or a re-association bound:
  P1 zero-B            == base product, bit for bit
  P2 one adapter       == X (W0 + s A B) with the merged matrix formed in fp64
  P3 permutation       of requests permutes output row blocks, bit for bit
  P4 batch of one      == the same rows inside any batch, bit for bit
  P5 brute force       exact integer arithmetic on tiny shapes
  P6 linearity         in s and in X
  P7 rank-one          closed form with unit-vector adapters
  P8 output RMS        closed form of the benchmark distributions
  P9 library           fp64 matmul of the same three products
  P10 worked example   a three-row layer derived by hand (tests/golden/worked_example.json)
"""
import itertools

import numpy as np
import pytest

from oracle import oracle_linear, oracle_workload
from workloads import make_custom, make_workload, to_f64


def _wl(dtype="bf16", seed=7, K=64, N=48, ranks=(8, 16, 8), scales=(2.0, 0.5, 1.0),
        req_adapter=(1, 0, -1, 2, 1, 0), req_ntok=(3, 1, 2, 4, 0, 5), **kw):
    return make_custom(seed=seed, dtype=dtype, K=K, N=N, ranks=ranks, scales=scales,
                       req_adapter=req_adapter, req_ntok=req_ntok, **kw)


def _tensors(wl):
    A = [wl.A(a) for a in range(wl.n_adapters)]
    B = [wl.B(a) for a in range(wl.n_adapters)]
    return wl.X(), wl.W0(), A, B


def _base_sequential(X, W0):
    """sum over k in ascending order, one rounded product at a time (fp64)."""
    x, w = to_f64(X), to_f64(W0)
    acc = np.zeros((x.shape[0], w.shape[0]))
    for k in range(x.shape[1]):
        acc = acc + x[:, k, None] * w[None, :, k]
    return acc


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_p1_zero_b_is_base_product_bitwise(dtype):
    wl = _wl(dtype)
    X, W0, A, B = _tensors(wl)
    Bz = [np.zeros_like(b) for b in B]
    Y = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, Bz, wl.ranks, wl.scales)
    assert np.array_equal(Y, _base_sequential(X, W0))
    # and the no-adapter id gives the same thing
    Yn = oracle_linear(X, W0, np.full_like(wl.req_adapter, -1), wl.req_ntok, A, B, wl.ranks, wl.scales)
    assert np.array_equal(Yn, Y)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_p2_single_adapter_equals_merged(dtype):
    wl = _wl(dtype, req_adapter=(1, 1, 1), req_ntok=(4, 1, 6))
    X, W0, A, B = _tensors(wl)
    Y = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, wl.scales)
    # merged weight in the formula's orientation: W[k,n] = W0[k,n] + s * sum_j A[k,j] B[j,n]
    Wm = to_f64(W0).T + float(wl.scales[1]) * (to_f64(A[1]).T @ to_f64(B[1]).T)
    Ym = to_f64(X) @ Wm
    rms = np.sqrt((Ym ** 2).mean())
    assert np.abs(Y - Ym).max() <= 1e-12 * rms


def test_p3_p4_permutation_and_batch_independence_bitwise():
    wl = _wl("bf16", seed=11)
    X, W0, A, B = _tensors(wl)
    Y = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, wl.scales)
    off = np.concatenate([[0], np.cumsum(wl.req_ntok)])
    R = wl.n_req
    rng = np.random.default_rng(0)
    for _ in range(3):
        order = rng.permutation(R)
        Xp = np.concatenate([X[off[i]:off[i + 1]] for i in order])
        Yp = oracle_linear(Xp, W0, wl.req_adapter[order], wl.req_ntok[order], A, B, wl.ranks, wl.scales)
        want = np.concatenate([Y[off[i]:off[i + 1]] for i in order])
        assert np.array_equal(Yp, want)
    for i in range(R):  # every request alone
        Yi = oracle_linear(X[off[i]:off[i + 1]], W0, wl.req_adapter[i:i + 1], wl.req_ntok[i:i + 1],
                           A, B, wl.ranks, wl.scales)
        assert np.array_equal(Yi, Y[off[i]:off[i + 1]])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_p5_brute_force_exact_integers(dtype):
    # small integers and power-of-two scales: every product and sum is exact
    wl = make_custom(seed=3, dtype=dtype, K=16, N=8, ranks=(4, 2), scales=(2.0, 0.5),
                     req_adapter=(0, 1, -1, 0), req_ntok=(2, 3, 1, 2), integer_valued=True)
    X, W0, A, B = _tensors(wl)
    Y = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, wl.scales)
    xi = to_f64(X).astype(int).tolist()
    wi = to_f64(W0).astype(int).tolist()
    ai = [to_f64(a).astype(int).tolist() for a in A]
    bi = [to_f64(b).astype(int).tolist() for b in B]
    twice_scale = [4, 1]  # 2*s as integers
    t = 0
    for a, L in zip(wl.req_adapter.tolist(), wl.req_ntok.tolist()):
        for _ in range(L):
            for n in range(8):
                base = sum(xi[t][k] * wi[n][k] for k in range(16))
                lo2 = 0
                if a >= 0:
                    r = int(wl.ranks[a])
                    v = [sum(xi[t][k] * ai[a][j][k] for k in range(16)) for j in range(r)]
                    lo2 = twice_scale[a] * sum(v[j] * bi[a][n][j] for j in range(r))
                assert Y[t, n] * 2 == 2 * base + lo2, (t, n)
            t += 1
    assert t == wl.T


def test_p6_linearity_in_scale_and_input():
    wl = _wl("f32", seed=5)
    X, W0, A, B = _tensors(wl)
    ys = [oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks,
                        np.full(wl.n_adapters, s, np.float32)) for s in (0.0, 1.0, 2.0)]
    rms = np.sqrt((ys[2] ** 2).mean())
    assert np.abs((ys[2] - ys[1]) - (ys[1] - ys[0])).max() <= 1e-12 * rms
    X2 = make_custom(seed=6, dtype="f32", K=64, N=48, ranks=wl.ranks, scales=wl.scales,
                     req_adapter=wl.req_adapter, req_ntok=wl.req_ntok).X()
    Xs = (X.astype(np.float64) + X2.astype(np.float64)).astype(np.float32)
    exact = np.array_equal(Xs.astype(np.float64), X.astype(np.float64) + X2.astype(np.float64))
    y1 = ys[1]
    y2 = oracle_linear(X2, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, np.ones(wl.n_adapters, np.float32))
    y12 = oracle_linear(Xs, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, np.ones(wl.n_adapters, np.float32))
    tol = 1e-12 if exact else 1e-6  # the fp32 sum of inputs may round
    assert np.abs(y12 - (y1 + y2)).max() <= tol * rms


def test_p7_rank_one_unit_vectors():
    K, N, T = 32, 24, 5
    wl = make_custom(seed=9, dtype="f32", K=K, N=N, ranks=(8,), scales=(3.0,), req_adapter=(0,), req_ntok=(T,))
    X, W0 = wl.X(), wl.W0()
    k0, n0, j0 = 7, 13, 2
    A = np.zeros((8, K), np.float32)
    A[j0, k0] = 1.0  # A[k0, j0] = 1 in the formula's orientation
    B = np.zeros((N, 8), np.float32)
    B[n0, j0] = 1.0  # B[j0, n0] = 1
    Y = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, [A], [B], wl.ranks, wl.scales)
    base = _base_sequential(X, W0)
    want = base.copy()
    want[:, n0] = base[:, n0] + 3.0 * X[:, k0].astype(np.float64)
    assert np.array_equal(Y, want)
    # transposing either adapter operand would move the update elsewhere
    assert not np.array_equal(Y[:, n0], base[:, n0])
    mask = np.ones(N, bool)
    mask[n0] = False
    assert np.array_equal(Y[:, mask], base[:, mask])


def test_p8_output_rms_closed_form():
    # RMS(Y)^2 = K sigma_W^2 + s^2 r sigma_B^2 (K sigma_A^2), with sigma_A = 1/sqrt(K)
    for idx, tol_lora in ((0, 0.12), (1, 0.06)):  # config 0 has few adapter samples
        wl = make_workload(idx)
        K, r, s = wl.projections[0].K, int(wl.ranks[0]), float(wl.scales[0])
        want_lora = s * np.sqrt(r) * 0.02  # K sigma_A^2 = 1
        want = np.sqrt(K * 0.02 ** 2 + want_lora ** 2)
        assert abs(want - (0.339, 1.290)[idx]) < 2e-3 and abs(want_lora - (0.113, 0.160)[idx]) < 1e-3
        Y = oracle_workload(wl)
        rms = np.sqrt((Y ** 2).mean())
        assert abs(rms - want) / want < 0.03, (idx, rms)
        Yb = oracle_linear(wl.X(), wl.W0(), np.full_like(wl.req_adapter, -1), wl.req_ntok,
                           [None] * wl.n_adapters, [None] * wl.n_adapters, wl.ranks, wl.scales)
        lora_rms = np.sqrt(((Y - Yb) ** 2).mean())
        assert abs(lora_rms - want_lora) / want_lora < tol_lora, (idx, lora_rms)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_p9_library_matmul(dtype):
    wl = _wl(dtype, seed=21, K=96, N=40)
    X, W0, A, B = _tensors(wl)
    Y, V = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, wl.scales, return_v=True)
    x = to_f64(X)
    ra = wl.row_adapter()
    want = x @ to_f64(W0).T
    for a in range(wl.n_adapters):
        m = ra == a
        v = x[m] @ to_f64(A[a]).T
        want[m] += float(wl.scales[a]) * (v @ to_f64(B[a]).T)
        assert np.abs(V[m, :wl.ranks[a]] - v).max() <= 1e-12 * max(1.0, np.abs(v).max())
        assert np.all(V[m, wl.ranks[a]:] == 0)
    rms = np.sqrt((want ** 2).mean())
    assert np.abs(Y - want).max() <= 1e-12 * rms


def _worked_example(dtype):
    import json
    import os
    from workloads.bits import bf16_bits_from_f32
    fx = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")))
    conv = (lambda a: bf16_bits_from_f32(np.asarray(a, np.float32))) if dtype == "bf16" else (lambda a: np.asarray(a, np.float32))
    return fx, conv


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_p10_worked_example_derived_by_hand(dtype):
    fx, conv = _worked_example(dtype)
    Y = oracle_linear(conv(fx["X"]), conv(fx["W0"]), fx["req_adapter"], fx["req_ntok"], [conv(fx["A0"])], [conv(fx["B0"])],
                      np.asarray(fx["rank"], np.int32), np.asarray(fx["scale"], np.float32))
    assert np.array_equal(Y, np.asarray(fx["Y"], np.float64))


def test_row_subset_matches_full_and_errors():
    wl = _wl("bf16", seed=2)
    X, W0, A, B = _tensors(wl)
    Y = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, wl.scales)
    rows = np.array([14, 0, 3, 3, 9])
    Ys = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, wl.scales, rows=rows)
    assert np.array_equal(Ys, Y[rows])
    with pytest.raises(ValueError):  # id out of range is an error, never clamped
        oracle_linear(X, W0, np.array([3, 0, -1, 2, 1, 0]), wl.req_ntok, A, B, wl.ranks, wl.scales)
    with pytest.raises(ValueError):  # lengths must add up to the rows of X
        oracle_linear(X, W0, wl.req_adapter, wl.req_ntok + 1, A, B, wl.ranks, wl.scales)
    with pytest.raises(ValueError):
        oracle_linear(X, W0, wl.req_adapter, -wl.req_ntok, A, B, wl.ranks, wl.scales)


def test_empty_batch_and_zero_length_requests():
    wl = _wl("bf16", req_adapter=(0, 1), req_ntok=(0, 0))
    X, W0, A, B = _tensors(wl)
    Y = oracle_linear(X, W0, wl.req_adapter, wl.req_ntok, A, B, wl.ranks, wl.scales)
    assert Y.shape == (0, 48)
