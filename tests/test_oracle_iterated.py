"""Pins of the oracle's iterated (k-plane) compressor and k-plane linear (Sec. 4.2 of the paper, ablation over
the fidelity of Delta) against things other than itself: a hand-computed example, the closed form of the
optimal-scale residual, the half-normal closed form of the second scale, the 1-bit functions already pinned,
and library float64 routines."""
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _golden_kv(name):
    kv = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or "=" not in line:
                continue
            k, v = [s.strip() for s in line.split("=")]
            kv[k] = v
    return kv


def _signs(packed, inn):
    bits = np.unpackbits(np.ascontiguousarray(packed).view(np.uint8), axis=-1, bitorder="little")[..., :inn]
    return bits.astype(np.float64) * 2 - 1


def _pair(rng, out, inn, sigma=0.002):
    base = (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
    ft = (base.astype(np.float32) + rng.standard_normal((out, inn)).astype(np.float32) * sigma).astype(np.float16)
    return base, ft


def test_hand_computed_three_iterations(ref):
    g = _golden_kv("iterated_small.txt")
    base = np.full((1, 32), 0.5, dtype=np.float16)
    delta = np.tile(np.array([3, -1, 1, -3], dtype=np.float32) / 64, 8)
    ft = (base.astype(np.float32) + delta).astype(np.float16)
    packed, alpha, mean, rsq = ref.compress_iterated(base, ft, 3)
    for j in range(3):
        assert float(alpha[j]) == float(g[f"alpha_{j}"]) and mean[j] == float(g[f"alpha_{j}"])
        assert int(packed[j, 0, 0]) == int(g[f"word_{j}"], 16)
    for j in range(4):
        assert rsq[j] == float(g[f"rsq_{j}"])
    xs = {"ones": np.ones(32), "e0": np.eye(32)[0], "e1": np.eye(32)[1], "e3": np.eye(32)[3]}
    for name, xv in xs.items():
        x = xv.astype(np.float16)[None, :]
        y16, y32 = ref.linear_multitenant_kbit(x, base, [[packed[0], packed[1]]], alpha[None, :2], [0])
        assert float(y32[0, 0]) == float(g[f"y_{name}"]) == float(y16[0, 0]), name


def test_first_plane_is_the_one_bit_compressor(ref):
    rng = np.random.default_rng(11)
    base, ft = _pair(rng, 24, 160)
    p1, a1, m1 = ref.compress(base, ft)
    packed, alpha, mean, _ = ref.compress_iterated(base, ft, 3)
    assert np.array_equal(packed[0], p1) and float(alpha[0]) == a1 and mean[0] == m1
    # and iterating is the same as compressing against the materialised previous model, when that model is
    # exactly representable: take a base whose sum with +-alpha_0 stays in binary16 (coarse grid, alpha = 2^-6)
    base_c = (rng.integers(-8, 8, size=(4, 64)) / 16.0).astype(np.float16)
    d = rng.permutation(np.tile(np.array([3, -1, 1, -3], dtype=np.float32) / 128, 64)).reshape(4, 64)   # mean |d| = 2^-6
    ft_c = (base_c.astype(np.float32) + d).astype(np.float16)
    pk, al, _, _ = ref.compress_iterated(base_c, ft_c, 2)
    s0 = _signs(pk[0], 64)
    model1 = (base_c.astype(np.float64) + float(al[0]) * s0).astype(np.float16)
    assert np.array_equal(model1.astype(np.float64), base_c.astype(np.float64) + float(al[0]) * s0)   # exact
    p2, a2, _ = ref.compress(model1, ft_c)
    assert np.array_equal(pk[1], p2) and float(al[1]) == a2


def test_residual_follows_the_optimal_scale_closed_form(ref):
    """With a = mean|r| (Eq. 4), ||r - a Sign(r)||^2 = ||r||^2 - n a^2 (Eq. 3 expanded); with the scale rounded
    to binary16 the exact expression is ||r||^2 - 2 a sum|r| + n a^2.  Both are checked, from the oracle's planes
    and scales only, in float64 with numpy; the residual can never grow."""
    rng = np.random.default_rng(12)
    out, inn, k = 48, 256, 6
    base, ft = _pair(rng, out, inn)
    packed, alpha, mean, rsq = ref.compress_iterated(base, ft, k)
    n = out * inn
    r = ft.astype(np.float64) - base.astype(np.float64)
    for j in range(k):
        assert rsq[j] == pytest.approx(float(np.sum(r * r)), rel=1e-6)
        assert mean[j] == pytest.approx(float(np.mean(np.abs(r))), rel=1e-6)
        assert float(alpha[j]) == float(np.float16(np.float32(mean[j])))
        assert np.array_equal(_signs(packed[j], inn) > 0, r > 0) or np.mean((_signs(packed[j], inn) > 0) != (r > 0)) < 1e-3
        a = float(alpha[j])
        want_next = rsq[j] - 2 * a * mean[j] * n + n * a * a
        assert rsq[j + 1] == pytest.approx(want_next, rel=1e-4, abs=1e-12)
        assert rsq[j + 1] <= rsq[j] - n * mean[j] ** 2 * (1 - 1e-3) + 1e-12          # within rounding of the optimum
        r = r - a * _signs(packed[j], inn)
    assert np.all(np.diff(rsq) <= 0)
    # reconstruction: W_base + sum alpha_j S_j differs from W_fine by the last residual
    recon = base.astype(np.float64) + sum(float(alpha[j]) * _signs(packed[j], inn) for j in range(k))
    assert float(np.sum((ft.astype(np.float64) - recon) ** 2)) == pytest.approx(rsq[k], rel=1e-3, abs=1e-12)


def test_second_scale_matches_half_normal_closed_form(ref):
    """Gaussian delta of standard deviation s: alpha_0 = s sqrt(2/pi) = a s, and the next residual |z| - a has
    mean absolute value s (2 a (2 Phi(a) - 3/2) + 4 phi(a) - 2 phi(0)) = 0.48262 s."""
    rng = np.random.default_rng(13)
    out, inn, sigma = 256, 1024, 0.25
    base = np.zeros((out, inn), dtype=np.float16)
    ft = (rng.standard_normal((out, inn)) * sigma).astype(np.float16)
    _, alpha, mean, _ = ref.compress_iterated(base, ft, 2)
    a = math.sqrt(2 / math.pi)
    Phi = 0.5 * (1 + math.erf(a / math.sqrt(2)))
    phi = lambda z: math.exp(-z * z / 2) / math.sqrt(2 * math.pi)   # noqa: E731
    second = 2 * a * (2 * Phi - 1.5) + 4 * phi(a) - 2 * phi(0.0)
    from scipy.integrate import quad
    numeric = quad(lambda z: abs(z - a) * 2 * phi(z), 0, 12, points=[a])[0]      # E| |z| - a | by quadrature
    assert second == pytest.approx(numeric, abs=1e-9) and second == pytest.approx(0.48262, abs=1e-5)
    assert mean[0] / sigma == pytest.approx(a, rel=5e-3)
    assert mean[1] / sigma == pytest.approx(second, rel=5e-3)
    assert float(alpha[1]) == pytest.approx(mean[1], rel=2 ** -11)


def _dense_f64(x, base, planes_by_tenant, alphas, tok, inn):
    y = np.empty((x.shape[0], base.shape[0]), dtype=np.float64)
    for t, e in enumerate(tok):
        weff = base.astype(np.float64)
        for j, p in enumerate(planes_by_tenant[e]):
            weff = weff + float(alphas[e][j]) * _signs(p, inn)
        y[t] = weff @ x[t].astype(np.float64)
    return y


def test_kbit_linear_matches_dense_float64_matmul_and_one_bit_linear(ref):
    rng = np.random.default_rng(14)
    out, inn, k, nt = 40, 320, 3, 3
    base = (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
    planes, alphas = [], []
    for _ in range(nt):
        ft = (base.astype(np.float32) + rng.standard_normal((out, inn)).astype(np.float32) * 0.002).astype(np.float16)
        pk, al, _, _ = ref.compress_iterated(base, ft, k)
        planes.append([pk[j] for j in range(k)])
        alphas.append(al)
    alphas = np.array(alphas, dtype=np.float32)
    tok = [2, 0, 0, 1, 2]
    x = rng.standard_normal((len(tok), inn)).astype(np.float16)
    y16, y32 = ref.linear_multitenant_kbit(x, base, planes, alphas, tok)
    y64 = ref.linear_multitenant_kbit_f64(x, base, planes, alphas, tok)
    want = _dense_f64(x, base, planes, alphas, tok, inn)
    scale = np.max(np.abs(want))
    assert np.max(np.abs(y64 - want)) <= 1e-12 * scale
    assert np.max(np.abs(y32 - want)) <= 2e-5 * scale
    assert np.array_equal(y16, y32.astype(np.float16))
    # one plane: the 1-bit linear, bit for bit
    y16_1, y32_1 = ref.linear_multitenant_kbit(x, base, [[p[0]] for p in planes], alphas[:, :1], tok)
    z16, z32 = ref.linear_multitenant(x, base, [p[0] for p in planes], alphas[:, 0], tok)
    assert np.array_equal(y32_1, z32) and np.array_equal(y16_1, z16)
    # a plane with scale 0 changes nothing; swapping two planes together with their scales changes only rounding
    al0 = alphas.copy()
    al0[:, 2] = 0.0
    _, y32_two = ref.linear_multitenant_kbit(x, base, [p[:2] for p in planes], alphas[:, :2], tok)
    _, y32_z = ref.linear_multitenant_kbit(x, base, planes, al0, tok)
    assert np.array_equal(y32_two, y32_z)
    _, y32_sw = ref.linear_multitenant_kbit(x, base, [[p[1], p[0], p[2]] for p in planes], alphas[:, [1, 0, 2]], tok)
    assert np.max(np.abs(y32_sw - y32)) <= 2e-6 * scale
    # one-hot x reads W_base[n,c] + sum_j alpha_j s_j[n,c]
    e = np.zeros((1, inn), dtype=np.float16)
    e[0, 37] = 1.0
    _, y1 = ref.linear_multitenant_kbit(e, base, planes, alphas, [1])
    s = np.stack([_signs(planes[1][j], inn)[:, 37] for j in range(k)])
    want1 = base[:, 37].astype(np.float32)
    for j in range(k):
        want1 = want1 + np.float32(alphas[1, j]) * s[j].astype(np.float32)
    assert np.array_equal(y1[0], want1)


def test_kbit_argument_errors(ref):
    base = np.zeros((2, 32), dtype=np.float16)
    p = np.zeros((2, 1), dtype=np.uint32)
    with pytest.raises(IndexError):
        ref.linear_multitenant_kbit(np.zeros((1, 32), dtype=np.float16), base, [[p, p]], np.zeros((1, 2)), [1])
    with pytest.raises(ValueError):
        ref.compress_iterated(np.zeros((2, 48), dtype=np.float16), np.zeros((2, 48), dtype=np.float16), 2)
    with pytest.raises(ValueError):
        ref.compress_iterated(base, base, 0)
