"""Pins of the oracle's 8-bit round-to-nearest base (Sec. 4.2 of the paper, quantized base models): the quantiser
against the properties that define round-to-nearest with a per-row absmax scale and a hand example, the compressor
and the linear against the already pinned fp16-base functions on weights that the quantiser represents exactly,
and against float64 library routines."""
import numpy as np
import pytest


def _signs(packed, inn):
    bits = np.unpackbits(np.ascontiguousarray(packed).view(np.uint8), axis=-1, bitorder="little")[..., :inn]
    return bits.astype(np.float64) * 2 - 1


def test_quantiser_hand_example(ref):
    # row 0: absmax 127/64 -> scale 1/64 exactly, every entry a multiple of 1/64: exact integers, ties included
    w = np.zeros((3, 32), dtype=np.float16)
    w[0, :6] = np.array([127, -127, 1, -1, 63, 0.5], dtype=np.float32) / 64      # 0.5/64 -> q = 0.5 -> rounds to even: 0
    w[0, 6] = 1.5 / 64                                                           # q = 1.5 -> 2 (to even)
    w[0, 7] = 2.5 / 64                                                           # q = 2.5 -> 2 (to even)
    w[1, :] = 0                                                                  # all-zero row: scale 1, q 0
    w[2, 0], w[2, 1] = 1.0, -0.25                                                # absmax 1 -> scale 1/127
    q, scale = ref.quantize_rtn8(w)
    assert scale[0] == np.float32(127 / 64) / np.float32(127) == np.float32(1 / 64)
    assert list(q[0, :8]) == [127, -127, 1, -1, 63, 0, 2, 2] and not q[0, 8:].any()
    assert scale[1] == 1.0 and not q[1].any()
    assert scale[2] == np.float32(1.0) / np.float32(127.0)
    assert q[2, 0] == 127 and q[2, 1] == int(np.rint(np.float32(-0.25) / scale[2])) == -32


def test_quantiser_is_round_to_nearest_with_absmax_scale(ref):
    rng = np.random.default_rng(21)
    w = (rng.standard_normal((40, 256)) * 0.02).astype(np.float16)
    q, scale = ref.quantize_rtn8(w)
    w32 = w.astype(np.float32)
    amax = np.abs(w32).max(axis=1)
    assert np.array_equal(scale, amax / np.float32(127))
    assert q.min() >= -127 and q.max() <= 127 and np.all(np.abs(q).max(axis=1) == 127)
    # nearest: the error is at most half a step (plus the rounding of the division), and no neighbour is closer
    deq = scale[:, None].astype(np.float64) * q.astype(np.float64)
    err = np.abs(w32.astype(np.float64) - deq)
    assert np.all(err <= 0.5 * scale[:, None] * (1 + 1e-6))
    for d in (-1, 1):
        other = scale[:, None].astype(np.float64) * np.clip(q.astype(np.float64) + d, -127, 127)
        assert np.all(err <= np.abs(w32.astype(np.float64) - other) * (1 + 1e-6) + 1e-12)
    # idempotent: quantising the dequantised weights (where fp16 holds them exactly) gives the same integers
    w2 = (np.float32(2.0 ** -9) * rng.integers(-127, 128, size=(8, 64))).astype(np.float16)
    w2[:, 0] = 127 * 2.0 ** -9
    q2, s2 = ref.quantize_rtn8(w2)
    assert np.all(s2 == np.float32(2.0 ** -9)) and np.array_equal(q2.astype(np.float32) * s2[:, None], w2.astype(np.float32))


def _exact_problem(rng, out, inn, n_tenants):
    """Base weights of the form 2^-9 * integer in [-127, 127] with 127 present in every row: the quantiser represents
    them exactly, so every q8 function must agree bit for bit with its fp16-base counterpart."""
    base = (np.float32(2.0 ** -9) * rng.integers(-127, 128, size=(out, inn))).astype(np.float16)
    base[:, 0] = 127 * 2.0 ** -9
    fts = [(base.astype(np.float32) + rng.standard_normal((out, inn)).astype(np.float32) * 0.002).astype(np.float16)
           for _ in range(n_tenants)]
    return base, fts


def test_q8_functions_equal_fp16_base_functions_on_exactly_representable_weights(ref):
    rng = np.random.default_rng(22)
    out, inn, nt = 24, 160, 3
    base, fts = _exact_problem(rng, out, inn, nt)
    q, scale = ref.quantize_rtn8(base)
    assert np.array_equal(scale[:, None] * q.astype(np.float32), base.astype(np.float32))
    packed, alphas = [], []
    for ft in fts:
        p8, a8, m8 = ref.compress_q8(q, scale, ft)
        p16, a16, m16 = ref.compress(base, ft)
        assert np.array_equal(p8, p16) and a8 == a16 and m8 == m16
        packed.append(p8)
        alphas.append(a8)
    tok = [2, 0, 1, 1]
    x = rng.standard_normal((len(tok), inn)).astype(np.float16)
    y16_q, y32_q = ref.linear_multitenant_q8(x, q, scale, packed, alphas, tok)
    y16, y32 = ref.linear_multitenant(x, base, packed, alphas, tok)
    assert np.array_equal(y32_q, y32) and np.array_equal(y16_q, y16)


def test_q8_compress_and_linear_against_float64_library_routines(ref):
    rng = np.random.default_rng(23)
    out, inn, nt = 40, 320, 3
    base = (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
    q, scale = ref.quantize_rtn8(base)
    deq = scale[:, None].astype(np.float64) * q.astype(np.float64)
    packed, alphas = [], []
    for _ in range(nt):
        ft = (base.astype(np.float32) + rng.standard_normal((out, inn)).astype(np.float32) * 0.002).astype(np.float16)
        p, a, mean = ref.compress_q8(q, scale, ft)
        d = ft.astype(np.float64) - deq
        bits = _signs(p, inn) > 0
        assert np.mean(bits != (d > 0)) < 1e-3 and np.all(bits[np.abs(d) > 1e-6] == (d > 0)[np.abs(d) > 1e-6])
        assert mean == pytest.approx(float(np.mean(np.abs(d))), rel=1e-5)
        assert a == float(np.float16(np.float32(mean)))
        packed.append(p)
        alphas.append(a)
    tok = [1, 2, 0, 2, 2]
    x = rng.standard_normal((len(tok), inn)).astype(np.float16)
    y16, y32 = ref.linear_multitenant_q8(x, q, scale, packed, alphas, tok)
    y64 = ref.linear_multitenant_q8_f64(x, q, scale, packed, alphas, tok)
    want = np.stack([(deq + float(alphas[e]) * _signs(packed[e], inn)) @ x[t].astype(np.float64) for t, e in enumerate(tok)])
    top = np.max(np.abs(want))
    assert np.max(np.abs(y64 - want)) <= 1e-12 * top
    assert np.max(np.abs(y32 - want)) <= 2e-5 * top
    assert np.array_equal(y16, y32.astype(np.float16))
    with pytest.raises(IndexError):
        ref.linear_multitenant_q8(x[:1], q, scale, packed, alphas, [3])
