"""Pins for the CPU oracle: what the paper and plain mathematics fix, not the oracle's own formulas.

Paper passages pinned here: Eq. 1-2 (sign quantiser, Sign(0) = -1), Eq. 3-4 (alpha = mean|Delta| is the
L2-optimal scale), Eq. 6 (base product + scaled sign product = product with the approximated weight),
Sec. 4.3 (a 1-bit delta is 1/16 of the fp16 matrix; rank-128 LoRA is byte-equal at 4096 x 4096).
"""
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- conversions
def test_f16_to_f32_matches_numpy_on_every_bit_pattern(ref):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([ref.f16_to_f32(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f32_to_f16_round_nearest_even_matches_numpy(ref):
    rng = np.random.default_rng(1)
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, 70000.0, -70000.0, float("inf"), float("-inf"),
            2.0**-24, 2.0**-25, 2.0**-25 * 1.0000001, 2.0**-26, 3 * 2.0**-25, 2.0**-14, 2.0**-14 - 2.0**-25,
            1.0 + 2.0**-11, 1.0 + 3 * 2.0**-11, 1.0 + 2.0**-11 + 2.0**-20, 2047.5, 2048.5, 2049.5, 1e-8, 6.1e-5]
    vals += list(rng.standard_normal(4000) * 0.02)
    vals += list(rng.standard_normal(2000) * 1e-5)
    vals += list(np.exp(rng.uniform(-20, 12, 4000)) * rng.choice([-1, 1], 4000))
    # every midpoint between adjacent positive binary16 values (ties), exactly representable in binary32
    h = np.arange(0, 0x7BFF, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals += list(((lo + hi) / 2)[::7])
    arr = np.array(vals, dtype=np.float32)
    want = arr.astype(np.float16).view(np.uint16)
    got = np.array([ref.f32_to_f16(float(v)) for v in arr], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_f64_to_f16_rounds_once_and_matches_numpy(ref):
    """The conversion the scale of Eq. 4 goes through: binary64 straight to binary16.  numpy's float64 -> float16 cast
    rounds once; values just beside a middle between two binary16 neighbours tell one rounding from two."""
    rng = np.random.default_rng(2)
    vals = [0.0, -0.0, 1.0, 65504.0, 65519.999999, 65520.0, 1e6, -1e6, float("inf"), float("-inf"), 2.0**-24, 2.0**-25,
            2.0**-25 * (1 + 2.0**-40), 2.0**-26, 3 * 2.0**-25, 2.0**-14, 2.0**-14 - 2.0**-25, 1e-300, 1.6e-3, 7.98e-4]
    vals += list(rng.standard_normal(4000) * 0.002)
    vals += list(np.exp(rng.uniform(-20, 12, 4000)) * rng.choice([-1, 1], 4000))
    h = np.arange(0, 0x7BFF, 5, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = (lo + hi) / 2
    ulp32 = np.spacing(mid.astype(np.float32)).astype(np.float64)
    # the middle itself (tie -> even), and a quarter of a binary32 step to either side: binary32 would swallow it
    vals += list(mid) + list(mid + ulp32 / 4) + list(mid - ulp32 / 4)
    arr = np.array(vals, dtype=np.float64)
    with np.errstate(over="ignore"):
        want = arr.astype(np.float16).view(np.uint16)
    got = np.array([ref.f64_to_f16(float(v)) for v in arr], dtype=np.uint16)
    assert np.array_equal(got, want)
    # and the two-step conversion really differs on those: the test would see a detour through binary32
    two_step = np.array([ref.f32_to_f16(float(np.float32(v))) for v in mid + ulp32 / 4], dtype=np.uint16)
    one_step = np.array([ref.f64_to_f16(float(v)) for v in mid + ulp32 / 4], dtype=np.uint16)
    assert (two_step != one_step).sum() > len(mid) // 3


def midpoint_scale_matrices():
    """A (base, fine-tuned) pair of 1 x 64 whose mean |Delta| is 1 + 2^-11 + 2^-29: a hair above the middle between the
    binary16 neighbours 1 and 1 + 2^-10.  One rounding gives 1 + 2^-10; by way of binary32 (which rounds the mean onto
    the middle, a tie) it would give 1."""
    base = np.zeros((1, 64), dtype=np.float16)
    ft = np.ones((1, 64), dtype=np.float16)
    ft[0, :32] = np.float16(1.0 + 2.0**-10)
    base[0, 63] = np.float16(-(2.0**-23))            # Delta = 1 + 2^-23, exact in binary32
    return base, ft


def test_scale_is_rounded_once_at_a_binary16_middle(ref):
    base, ft = midpoint_scale_matrices()
    packed, alpha, mean = ref.compress(base, ft)
    assert mean == 1.0 + 2.0**-11 + 2.0**-29                      # the binary64 mean is exact here
    assert float(np.float32(mean)) == 1.0 + 2.0**-11              # binary32 would put it ON the middle
    assert alpha == 1.0 + 2.0**-10                                # one rounding: up
    assert alpha == float(np.float64(mean).astype(np.float16))
    assert np.all(packed == 0xFFFFFFFF)


def test_f32_to_f16_nan_stays_nan(ref):
    h = ref.f32_to_f16(float("nan"))
    assert (h & 0x7C00) == 0x7C00 and (h & 0x3FF) != 0


# --------------------------------------------------------------------------- Eq. 2 + packing layout
def _golden_words():
    rows = []
    with open(os.path.join(GOLDEN, "pack_words.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, pat, word = [s.strip() for s in line.split("|")]
            rows.append((name, pat, int(word, 16)))
    return rows


@pytest.mark.parametrize("name,pat,word", _golden_words())
def test_pack_signs_hand_derived_words(ref, name, pat, word):
    val = {"p": 0.25, "n": -0.25, "z": 0.0, "m": -0.0}
    delta = np.array([[val[c] for c in pat]], dtype=np.float16)
    assert ref.pack_signs(delta)[0, 0] == word
    # the same pattern through compress: W_base = 0.5, W_fine = 0.5 + delta (exact in fp16)
    base = np.full((1, 32), 0.5, dtype=np.float16)
    ft = (base.astype(np.float32) + delta.astype(np.float32)).astype(np.float16)
    packed, _, _ = ref.compress(base, ft)
    assert packed[0, 0] == word


def test_sign_of_zero_is_minus_one_including_specials(ref):
    # Eq. 2: Sign(w) = -1 for w <= 0.  Subnormals keep their sign; +inf is positive; nan compares false.
    tiny = np.float16(2.0**-24)
    d = np.zeros((1, 32), dtype=np.float16)
    d[0, :8] = [0.0, -0.0, tiny, -tiny, np.inf, -np.inf, np.nan, 65504.0]
    word = int(ref.pack_signs(d)[0, 0])
    assert word == (1 << 2) | (1 << 4) | (1 << 7)
    s = ref.unpack_signs(np.array([[word]], dtype=np.uint32), 32)[0]
    assert s[0] == -1 and s[1] == -1 and s[2] == +1 and s[3] == -1 and s[5] == -1 and s[6] == -1


def test_pack_unpack_roundtrip_and_bruteforce_bits(ref):
    rng = np.random.default_rng(7)
    out, inn = 37, 96
    d = (rng.standard_normal((out, inn)) * 0.002).astype(np.float16)
    d[rng.random((out, inn)) < 0.1] = 0.0
    packed = ref.pack_signs(d)
    assert packed.shape == (out, inn // 32) and packed.dtype == np.uint32
    signs = ref.unpack_signs(packed, inn)
    assert np.array_equal(signs, np.where(d.astype(np.float32) > 0, 1, -1).astype(np.int8))
    # brute force, pure Python, element by element: bit j of word w is k = 32 w + j
    for n in range(0, out, 9):
        for k in range(inn):
            bit = (int(packed[n, k // 32]) >> (k % 32)) & 1
            assert bit == (1 if float(d[n, k]) > 0 else 0)
    # arbitrary bit patterns survive unpack -> pack
    words = rng.integers(0, 2**32, size=(5, 4), dtype=np.uint64).astype(np.uint32)
    s = ref.unpack_signs(words, 128)
    assert np.array_equal(ref.pack_signs(s.astype(np.float16)), words)


def test_compress_bit_is_wft_greater_than_wbase(ref):
    # the sign of the fp32 delta equals the plain comparison of the two fp16 inputs, also for
    # subnormal differences, equal entries, signed zeros and infinities
    rng = np.random.default_rng(11)
    out, inn = 16, 64
    base = (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
    ft = (base.astype(np.float32) + rng.standard_normal((out, inn)).astype(np.float32) * 0.002).astype(np.float16)
    ft[0, :4] = base[0, :4]                                   # zero delta
    base[1, :4] = [0.0, -0.0, 0.0, -0.0]
    ft[1, :4] = [-0.0, 0.0, 2.0**-24, -(2.0**-24)]
    base[2, :3] = [6.0e-8, 65504.0, -65504.0]
    ft[2, :3] = [1.2e-7, np.inf, -np.inf]
    packed, _, _ = ref.compress(base, ft)
    want = np.zeros((out, inn // 32), dtype=np.uint32)
    for n in range(out):
        for k in range(inn):
            if float(ft[n, k]) > float(base[n, k]):
                want[n, k // 32] |= np.uint32(1 << (k % 32))
    assert np.array_equal(packed, want)


def test_pack_rejects_in_not_multiple_of_32(ref):
    with pytest.raises(ValueError):
        ref.pack_signs(np.zeros((2, 48), dtype=np.float16))
    with pytest.raises(ValueError):
        ref.compress(np.zeros((2, 48), dtype=np.float16), np.zeros((2, 48), dtype=np.float16))


# --------------------------------------------------------------------------- Eq. 3-4: alpha
def _golden_kv(name):
    kv = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or "=" not in line:
                continue
            k, v = [s.strip() for s in line.split("=")]
            kv[k] = v
    return kv


def _worked_example():
    base = np.full((2, 32), 0.5, dtype=np.float16)
    ft = base.copy()
    ft[0, :16] = 0.75
    ft[0, 16:] = 0.25
    ft[1, 0::2] = 0.625
    return base, ft


def test_worked_example_alpha_words_and_outputs(ref):
    g = _golden_kv("eq4_alpha_small.txt")
    base, ft = _worked_example()
    packed, alpha, mean = ref.compress(base, ft)
    assert alpha == float(g["alpha"]) and mean == float(g["alpha"])
    assert int(packed[0, 0]) == int(g["word_row0"], 16)
    assert int(packed[1, 0]) == int(g["word_row1"], 16)
    xs = {
        "ones": np.ones(32), "e0": np.eye(32)[0], "e1": np.eye(32)[1],
        "firsthalf": np.concatenate([np.ones(16), np.zeros(16)]),
    }
    for name, xv in xs.items():
        x = xv.astype(np.float16)[None, :]
        y16, y32 = ref.linear_multitenant(x, base, [packed], [alpha], [0])
        for row in (0, 1):
            want = float(g[f"y_{name}_row{row}"])
            assert float(y32[0, row]) == want, (name, row)
            assert float(y16[0, row]) == want, (name, row)


def test_alpha_minimises_l2_error_bruteforce_scan(ref):
    # Eq. 3: || Delta - a * Sign(Delta) ||^2 as a function of a is minimal at a = mean|Delta| (Eq. 4).
    rng = np.random.default_rng(3)
    for out, inn in [(4, 32), (3, 64), (8, 32)]:
        base = (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
        ft = (base.astype(np.float32) + rng.standard_normal((out, inn)).astype(np.float32) * 0.002).astype(np.float16)
        ft[0, :3] = base[0, :3]  # zero deltas take Sign = -1; the optimum is unchanged by that (Eq. 3)
        packed, alpha, mean = ref.compress(base, ft)
        delta = ft.astype(np.float64) - base.astype(np.float64)
        s = ref.unpack_signs(packed, inn).astype(np.float64)
        grid = np.linspace(0.0, 4 * np.abs(delta).mean(), 40001)
        err = ((delta[None] - grid[:, None, None] * s[None]) ** 2).sum(axis=(1, 2))
        a_best = grid[int(np.argmin(err))]
        step = grid[1] - grid[0]
        assert abs(a_best - mean) <= step, (a_best, mean)
        # stationarity: d/da sum (|d| - a)^2 = 0  <=>  sum(|d| - a) = 0
        assert abs((np.abs(delta) - mean).sum()) < 1e-12
        # and the error at alpha is no worse than at neighbours
        e = lambda a: ((delta - a * s) ** 2).sum()
        assert e(mean) <= e(mean * 1.01) and e(mean) <= e(mean * 0.99)
        # alpha is that mean rounded once to binary16
        assert alpha == float(np.float16(mean))


def test_alpha_statistics_scaling_and_permutation(ref):
    rng = np.random.default_rng(5)
    out, inn = 256, 512
    base = np.zeros((out, inn), dtype=np.float16)
    d = (rng.standard_normal((out, inn)) * 0.002).astype(np.float16)
    _, alpha, mean = ref.compress(base, d)
    # E|N(0, sigma)| = sigma * sqrt(2/pi); fp16 rounding of the inputs does not bias the mean
    assert abs(mean - 0.002 * math.sqrt(2 / math.pi)) < 4 * 0.002 * math.sqrt(1 - 2 / math.pi) / math.sqrt(out * inn)
    assert abs(alpha - mean) <= 2.0**-11 * mean
    # alpha(2 * Delta) = 2 * alpha(Delta): doubling is exact in binary16 here
    _, _, mean2 = ref.compress(base, (d.astype(np.float32) * 2).astype(np.float16))
    assert mean2 == 2 * mean
    # alpha(-Delta) = alpha(Delta)
    _, _, mean_neg = ref.compress(base, (-d).astype(np.float16))
    assert mean_neg == mean
    # permuting the entries does not change the mean beyond summation order
    perm = rng.permutation(out * inn)
    _, _, mean_p = ref.compress(base, d.reshape(-1)[perm].reshape(out, inn))
    assert abs(mean_p - mean) <= 1e-12 * mean
    # infinities propagate, nothing is clamped
    d2 = d.copy()
    d2[0, 0] = np.inf
    _, alpha_inf, _ = ref.compress(base, d2)
    assert math.isinf(alpha_inf)


# --------------------------------------------------------------------------- Eq. 6: the linear
def _problem(rng, T, out, inn, n_tenants, sigma=0.002):
    base = (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
    packed, alphas = [], []
    for _ in range(n_tenants):
        ft = (base.astype(np.float32) + rng.standard_normal((out, inn)).astype(np.float32) * sigma).astype(np.float16)
        from oracle import ref as R
        p, a, _ = R.compress(base, ft)
        packed.append(p)
        alphas.append(a)
    x = rng.standard_normal((T, inn)).astype(np.float16)
    return base, packed, np.array(alphas, dtype=np.float32), x


def _dense_f64(ref, x, base, packed, alphas, tok):
    """Eq. 6 written with library routines: W_eff = W_base + alpha * S (float64), y = x @ W_eff^T."""
    T, inn = x.shape
    y = np.empty((T, base.shape[0]), dtype=np.float64)
    for t in range(T):
        bits = np.unpackbits(packed[tok[t]].view(np.uint8), axis=1, bitorder="little")[:, :inn]
        s = bits.astype(np.float64) * 2 - 1
        weff = base.astype(np.float64) + float(alphas[tok[t]]) * s
        y[t] = weff @ x[t].astype(np.float64)
    return y


def test_linear_matches_dense_float64_library_matmul(ref):
    rng = np.random.default_rng(13)
    T, out, inn, nt = 5, 24, 160, 3      # non-square, out != in != T so a transposed operand cannot pass
    base, packed, alphas, x = _problem(rng, T, out, inn, nt)
    tok = [2, 0, 1, 0, 2]
    want = _dense_f64(ref, x, base, packed, alphas, tok)
    y64 = ref.linear_multitenant_f64(x, base, packed, alphas, tok)
    assert np.allclose(y64, want, rtol=0, atol=1e-12)
    y16, y32 = ref.linear_multitenant(x, base, packed, alphas, tok)
    # binary32 sequential accumulation: |error| <= K * eps * sum|terms| (loose classical bound)
    bound = inn * 2.0**-24 * (np.abs(x.astype(np.float64)) @ (np.abs(base.astype(np.float64)) + alphas.max()).T)
    assert np.all(np.abs(y32 - want) <= bound)
    assert np.max(np.abs(y32 - want)) / np.max(np.abs(want)) < 1e-5
    # the binary16 output is the nearest binary16 to the binary32 value
    assert np.array_equal(y16.view(np.uint16), y32.astype(np.float16).view(np.uint16))


def test_linear_special_cases_reduce_to_library_routines(ref):
    rng = np.random.default_rng(17)
    T, out, inn = 3, 20, 96
    base, packed, alphas, x = _problem(rng, T, out, inn, 1)
    x64, b64 = x.astype(np.float64), base.astype(np.float64)
    ones = np.full((out, inn // 32), 0xFFFFFFFF, dtype=np.uint32)
    zeros = np.zeros((out, inn // 32), dtype=np.uint32)
    tok = [0] * T
    a = 0.0015625
    # alpha = 0: plain product with W_base
    y = ref.linear_multitenant_f64(x, base, packed, [0.0], tok)
    assert np.allclose(y, x64 @ b64.T, atol=1e-12, rtol=0)
    # all bits set: base + alpha * sum_k x ; all clear: base - alpha * sum_k x
    y = ref.linear_multitenant_f64(x, base, [ones], [a], tok)
    assert np.allclose(y, x64 @ b64.T + np.float32(a).astype(np.float64) * x64.sum(1, keepdims=True), atol=1e-12, rtol=0)
    y = ref.linear_multitenant_f64(x, base, [zeros], [a], tok)
    assert np.allclose(y, x64 @ b64.T - np.float32(a).astype(np.float64) * x64.sum(1, keepdims=True), atol=1e-12, rtol=0)
    # W_base = 0 and alpha = 1: a pure +-1 dot product
    s = ref.unpack_signs(packed[0], inn).astype(np.float64)
    y = ref.linear_multitenant_f64(x, np.zeros_like(base), packed, [1.0], tok)
    assert np.allclose(y, x64 @ s.T, atol=1e-12, rtol=0)
    # one-hot x: y[n] = W_base[n,k] + alpha * s[n,k], a single binary32 addition
    for k in (0, 31, 32, 95):
        xe = np.zeros((1, inn), dtype=np.float16)
        xe[0, k] = 1.0
        _, y32 = ref.linear_multitenant(xe, base, packed, alphas, [0])
        want = base[:, k].astype(np.float32) + np.float32(alphas[0]) * s[:, k].astype(np.float32)
        assert np.array_equal(y32[0], want)


def test_fused_equals_materialised_weight(ref):
    # Eq. 6: W_base X + Delta_hat X = (W_base + Delta_hat) X, up to binary32 re-association
    rng = np.random.default_rng(19)
    T, out, inn = 4, 33, 256
    base, packed, alphas, x = _problem(rng, T, out, inn, 2)
    for t in (0, 1):
        _, y32 = ref.linear_multitenant(x, base, packed, alphas, [t] * T)
        ym, yabs = ref.linear_materialised(x, base, packed[t], float(alphas[t]))
        assert np.all(np.abs(y32 - ym) <= 1e-5 * yabs + 1e-30)


def test_tenant_permutation_and_token_independence(ref):
    rng = np.random.default_rng(23)
    T, out, inn, nt = 6, 17, 128, 4
    base, packed, alphas, x = _problem(rng, T, out, inn, nt)
    tok = [3, 1, 1, 0, 3, 2]
    y16, y32 = ref.linear_multitenant(x, base, packed, alphas, tok)
    # renumbering tenants changes nothing
    perm = [2, 0, 3, 1]                       # new id -> old id
    inv = {old: new for new, old in enumerate(perm)}
    y16p, _ = ref.linear_multitenant(x, base, [packed[o] for o in perm], alphas[perm], [inv[t] for t in tok])
    assert np.array_equal(y16.view(np.uint16), y16p.view(np.uint16))
    # each token alone gives the same row
    for t in range(T):
        yt, _ = ref.linear_multitenant(x[t:t + 1], base, packed, alphas, [tok[t]])
        assert np.array_equal(yt.view(np.uint16)[0], y16.view(np.uint16)[t])
    # permuting the tokens permutes the rows
    order = [4, 2, 0, 5, 1, 3]
    yo, _ = ref.linear_multitenant(x[order], base, packed, alphas, [tok[i] for i in order])
    assert np.array_equal(yo.view(np.uint16), y16.view(np.uint16)[order])
    # T = 0 is legal and empty
    y0, _ = ref.linear_multitenant(x[:0], base, packed, alphas, [])
    assert y0.shape == (0, out)
    with pytest.raises(IndexError):
        ref.linear_multitenant(x[:1], base, packed, alphas, [nt])
    with pytest.raises(IndexError):
        ref.linear_multitenant(x[:1], base, packed, alphas, [-1])


def test_naive_baseline_is_a_plain_per_tenant_product(ref):
    rng = np.random.default_rng(29)
    T, out, inn, nt = 4, 12, 64, 2
    base, packed, alphas, x = _problem(rng, T, out, inn, nt)
    ws = [ref.materialise_f16(base, packed[t], float(alphas[t])) for t in range(nt)]
    s0 = ref.unpack_signs(packed[0], inn).astype(np.float32)
    assert np.array_equal(ws[0].view(np.uint16),
                          (base.astype(np.float32) + np.float32(alphas[0]) * s0).astype(np.float16).view(np.uint16))
    tok = [1, 0, 0, 1]
    _, y32 = ref.linear_naive(x, ws, tok)
    for t in range(T):
        want = ws[tok[t]].astype(np.float64) @ x[t].astype(np.float64)
        assert np.allclose(y32[t], want, rtol=0, atol=1e-4)


# --------------------------------------------------------------------------- Sec. 4.3 footprint
def test_footprint_arithmetic():
    out = inn = 4096
    packed_bytes = out * (inn // 32) * 4
    assert packed_bytes == out * inn // 8 == 2_097_152
    assert out * inn * 2 == 16 * packed_bytes            # "16x" in Sec. 4.3
    assert 2 * 4096 * 128 * 2 == packed_bytes            # rank-128 LoRA is byte-equal at 4096 x 4096
