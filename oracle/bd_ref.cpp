// CPU oracle for the BitDelta hot path (arxiv 2402.10193).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
// GPU library is checked against.  Nothing in the product path may include,
// link or call it; only the tests, the smoke check and the benchmark's
// cpu_baseline leg do.  It shares no source with the HIP code: the fp16
// conversions, the bit layout and every loop below are written out here on
// their own.
//
// What it computes, and where the paper defines it:
//   * weight delta            Delta = W_fine - W_base                (Sec. 3.1)
//   * 1-bit quantiser         Sign(d) = +1 if d > 0 else -1           (Eq. 2)
//   * scale                   alpha = mean |Delta_ij|                 (Eq. 4)
//   * serving decomposition   X'_i = W_base X_i + alpha_i Sign(Delta_i) X_i
//                                                                     (Eq. 6)
//   * iterated compression   the compressor applied again with the compressed
//                             model as the base: k sign planes, k scales
//                                        (Sec. 4.2, ablation over the fidelity of Delta)
//   * quantised base         8-bit round-to-nearest base weights under the same deltas
//                                        (Sec. 4.2, "Quantized base models", Table 5)
// Readings where the paper is silent (all listed in the design notes):
//   * weights are [out, in] row-major, the reduction runs along `in`;
//   * 32 signs per uint32 along `in`, least significant bit first,
//     bit = 1 means +1 (Eq. 2's "d > 0"), so zero and negative map to bit 0;
//   * Delta is formed in IEEE binary32 from the binary16 inputs;
//   * alpha is summed in binary64, divided by out*in, rounded ONCE (binary64 ->
//     binary16, nearest even; not by way of binary32) and carried as a float;
//   * the two products of Eq. 6 are accumulated separately in binary32 in
//     ascending k, alpha is applied to the finished +-1 sum in binary32, and the
//     result is rounded once (nearest even) to binary16.  A binary64 variant
//     exists to bound the oracle's own rounding noise.
//
//   * iterated compression: the residual W_fine - (W_base + sum_i alpha_i S_i)
//     is carried in binary32 (one rounding per iteration: r <- r - alpha * s),
//     never re-rounded to binary16; every alpha_j is rounded to binary16 like
//     the first; the k-plane linear accumulates each plane's +-1 sum separately
//     in binary32 and adds alpha_j * sum_j to the base product in ascending j.
//   * 8-bit RTN base: one scale per output row, s_n = max_k |W[n,k]| / 127 in binary32 (1 for an
//     all-zero row), q = clamp(round-to-nearest-even(W / s_n), -127, 127); the base the deltas
//     are taken against and the linear multiplies is s_n * q in binary32 (never re-rounded to
//     binary16); activations, fine-tuned weights and alpha stay as they are.
//
// Parity pins live in tests/test_oracle_*.py (closed forms, brute force,
// library special cases, hand-written words).  No function here is unpinned.

#include <cstdint>
#include <cstring>
#include <cmath>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// binary16 -> binary32, exact.  Written from the IEEE 754 layout:
// 1 sign, 5 exponent (bias 15), 10 fraction bits.
inline float half_bits_to_float(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t expo = (h >> 10) & 0x1Fu;
    const uint32_t frac = h & 0x3FFu;
    uint32_t bits;
    if (expo == 0) {
        if (frac == 0) {
            bits = sign;  // +-0
        } else {
            // subnormal: value = frac * 2^-24; normalise into binary32
            int shift = 0;
            uint32_t f = frac;
            while ((f & 0x400u) == 0) { f <<= 1; ++shift; }
            f &= 0x3FFu;
            bits = sign | ((uint32_t)(127 - 15 - shift + 1) << 23) | (f << 13);
        }
    } else if (expo == 31) {
        bits = sign | 0x7F800000u | (frac << 13);  // inf / nan (payload kept)
    } else {
        bits = sign | ((expo + (127 - 15)) << 23) | (frac << 13);
    }
    float out;
    std::memcpy(&out, &bits, 4);
    return out;
}

// binary32 -> binary16, round to nearest, ties to even.
inline uint16_t float_to_half_bits(float v) {
    uint32_t bits;
    std::memcpy(&bits, &v, 4);
    const uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    const uint32_t absbits = bits & 0x7FFFFFFFu;
    if (absbits >= 0x7F800000u) {  // inf or nan
        if (absbits == 0x7F800000u) return (uint16_t)(sign | 0x7C00u);
        uint16_t payload = (uint16_t)((absbits >> 13) & 0x3FFu);
        return (uint16_t)(sign | 0x7C00u | payload | 0x200u);  // quiet nan
    }
    const int e32 = (int)(absbits >> 23);          // biased binary32 exponent
    const uint32_t m32 = absbits & 0x7FFFFFu;
    const int e = e32 - 127;                       // unbiased
    if (e >= 16) return (uint16_t)(sign | 0x7C00u);  // overflows even before rounding
    if (e >= -14) {
        // normal binary16 range: keep 10 fraction bits, round on the 13 dropped
        uint32_t mant = m32 >> 13;
        const uint32_t rest = m32 & 0x1FFFu;
        uint32_t half = ((uint32_t)(e + 15) << 10) | mant;
        if (rest > 0x1000u || (rest == 0x1000u && (mant & 1u))) ++half;  // may carry into exponent / inf
        return (uint16_t)(sign | half);
    }
    if (e < -25) return sign;  // below half of the smallest subnormal: rounds to zero
    // subnormal result: value = m * 2^-24 with m in [0, 1024]
    const uint32_t full = m32 | 0x800000u;          // 24-bit significand, value = full * 2^(e-23)
    const int drop = (-24) - (e - 23);              // bits to drop so the unit is 2^-24  (14..25)
    const uint32_t mant = full >> drop;
    const uint32_t rest = full & ((1u << drop) - 1u);
    const uint32_t halfway = 1u << (drop - 1);
    uint32_t half = mant;
    if (rest > halfway || (rest == halfway && (mant & 1u))) ++half;
    return (uint16_t)(sign | half);
}

// binary64 -> binary16, ONE rounding to nearest even, written out from the IEEE layout (not by way of binary32:
// a value a hair above the middle between two binary16 neighbours would first round onto that middle and then,
// as a tie, to the even neighbour).
inline uint16_t double_to_half_bits(double v) {
    uint64_t bits;
    std::memcpy(&bits, &v, sizeof(bits));
    const uint16_t sign = (uint16_t)((bits >> 48) & 0x8000u);
    const uint64_t absbits = bits & 0x7FFFFFFFFFFFFFFFull;
    if (absbits >= 0x7FF0000000000000ull)   // Inf or NaN
        return (uint16_t)(sign | 0x7C00u | ((absbits > 0x7FF0000000000000ull) ? 0x0200u : 0u));
    const int e = (int)(absbits >> 52) - 1023;          // unbiased (binary64 subnormals: far below binary16's range)
    const uint64_t frac = absbits & 0xFFFFFFFFFFFFFull;  // 52 bits
    if (e >= 16) return (uint16_t)(sign | 0x7C00u);
    if (e >= -14) {
        uint32_t mant = (uint32_t)(frac >> 42);          // 10 bits kept
        const uint64_t rest = frac & ((1ull << 42) - 1), halfway = 1ull << 41;
        uint32_t half = ((uint32_t)(e + 15) << 10) | mant;
        if (rest > halfway || (rest == halfway && (mant & 1u))) ++half;   // may carry into the exponent / to Inf
        return (uint16_t)(sign | half);
    }
    if (e < -25) return sign;                            // below half of the smallest subnormal (2^-25 itself: see below)
    // subnormal result, unit 2^-24: value = (2^52 + frac) * 2^(e-52)
    const uint64_t full = frac | (1ull << 52);
    const int drop = (-24) - (e - 52);                   // 42 + (-14 - e) : 43..53
    const uint64_t mant = full >> drop, rest = full & ((1ull << drop) - 1), halfway = 1ull << (drop - 1);
    uint32_t half = (uint32_t)mant;
    if (rest > halfway || (rest == halfway && (mant & 1ull))) ++half;
    return (uint16_t)(sign | half);
}

inline int sign_of_bit(const uint32_t* row_words, int64_t k) {
    return ((row_words[k >> 5] >> (k & 31)) & 1u) ? +1 : -1;
}

}  // namespace

extern "C" {

// ---- conversions, exported so tests can pin them against a library -------
float bd_ref_f16_to_f32(uint16_t h) { return half_bits_to_float(h); }
uint16_t bd_ref_f32_to_f16(float v) { return float_to_half_bits(v); }
uint16_t bd_ref_f64_to_f16(double v) { return double_to_half_bits(v); }

int bd_ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

// ---- Eq. 2 applied to an explicit delta matrix ----------------------------
// delta_f16 [out, in] binary16 bits -> packed [out, in/32].  Returns 0, or -1
// when `in` is not a multiple of 32.
int bd_ref_pack_signs(const uint16_t* delta_f16, int64_t out, int64_t in, uint32_t* packed) {
    if (in % 32 != 0) return -1;
    const int64_t words = in / 32;
    for (int64_t n = 0; n < out; ++n) {
        for (int64_t w = 0; w < words; ++w) {
            uint32_t word = 0;
            for (int j = 0; j < 32; ++j) {
                const float d = half_bits_to_float(delta_f16[n * in + w * 32 + j]);
                if (d > 0.0f) word |= (1u << j);
            }
            packed[n * words + w] = word;
        }
    }
    return 0;
}

// packed [out, in/32] -> signs [out, in] as int8 (+1 / -1)
int bd_ref_unpack_signs(const uint32_t* packed, int64_t out, int64_t in, int8_t* signs) {
    if (in % 32 != 0) return -1;
    const int64_t words = in / 32;
    for (int64_t n = 0; n < out; ++n)
        for (int64_t k = 0; k < in; ++k)
            signs[n * in + k] = (int8_t)sign_of_bit(packed + n * words, k);
    return 0;
}

// ---- Sec. 3.1: delta, sign bits (Eq. 2), alpha (Eq. 4) --------------------
// alpha_f16_as_float: the scale rounded once to binary16, returned as float.
// alpha_unrounded:    the binary64 mean before that rounding (may be null).
int bd_ref_compress(const uint16_t* w_base_f16, const uint16_t* w_ft_f16, int64_t out, int64_t in,
                    uint32_t* packed, float* alpha_f16_as_float, double* alpha_unrounded) {
    if (in % 32 != 0) return -1;
    const int64_t words = in / 32;
    std::vector<double> row_sum((size_t)out, 0.0);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        double s = 0.0;
        for (int64_t w = 0; w < words; ++w) {
            uint32_t word = 0;
            for (int j = 0; j < 32; ++j) {
                const int64_t idx = n * in + w * 32 + j;
                const float d = half_bits_to_float(w_ft_f16[idx]) - half_bits_to_float(w_base_f16[idx]);
                if (d > 0.0f) word |= (1u << j);
                s += (double)std::fabs(d);
            }
            packed[n * words + w] = word;
        }
        row_sum[(size_t)n] = s;
    }
    double total = 0.0;
    for (int64_t n = 0; n < out; ++n) total += row_sum[(size_t)n];
    const double mean = (out > 0 && in > 0) ? total / ((double)out * (double)in) : 0.0;
    if (alpha_unrounded) *alpha_unrounded = mean;
    if (alpha_f16_as_float) *alpha_f16_as_float = half_bits_to_float(double_to_half_bits(mean));
    return 0;
}

// ---- Eq. 6, fused form ------------------------------------------------------
// x_f16 [T, in], w_base_f16 [out, in], packed_by_tenant[n_tenants] -> each
// [out, in/32], alpha_by_tenant[n_tenants], tenant_of_token[T].
// y_f16 [T, out] (may be null) gets the binary16 result, y_f32 [T, out] (may be
// null) the binary32 value before the final rounding.
// Returns 0; -1 bad shape; -2 tenant id out of range.
int bd_ref_linear_multitenant(const uint16_t* x_f16, const uint16_t* w_base_f16,
                              const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                              const int32_t* tenant_of_token, uint16_t* y_f16, float* y_f32,
                              int64_t T, int64_t out, int64_t in, int32_t n_tenants) {
    if (in % 32 != 0) return -1;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return -2;
    const int64_t words = in / 32;
    std::vector<float> xf((size_t)(T * in));
    for (int64_t i = 0; i < T * in; ++i) xf[(size_t)i] = half_bits_to_float(x_f16[i]);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        for (int64_t t = 0; t < T; ++t) {
            const uint32_t* srow = packed_by_tenant[tenant_of_token[t]] + n * words;
            const float* xr = xf.data() + t * in;
            float acc_base = 0.0f;
            float acc_delta = 0.0f;
            for (int64_t k = 0; k < in; ++k) {
                const float xv = xr[k];
                acc_base += xv * half_bits_to_float(w_base_f16[n * in + k]);
                acc_delta += (sign_of_bit(srow, k) > 0) ? xv : -xv;
            }
            const float yv = acc_base + alpha_by_tenant[tenant_of_token[t]] * acc_delta;
            if (y_f32) y_f32[t * out + n] = yv;
            if (y_f16) y_f16[t * out + n] = float_to_half_bits(yv);
        }
    }
    return 0;
}

// Same definition with binary64 accumulation and no output rounding: bounds
// the binary32 oracle's own error.
int bd_ref_linear_multitenant_f64(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                  const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                  const int32_t* tenant_of_token, double* y_f64,
                                  int64_t T, int64_t out, int64_t in, int32_t n_tenants) {
    if (in % 32 != 0) return -1;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return -2;
    const int64_t words = in / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        for (int64_t t = 0; t < T; ++t) {
            const uint32_t* srow = packed_by_tenant[tenant_of_token[t]] + n * words;
            double acc_base = 0.0, acc_delta = 0.0;
            for (int64_t k = 0; k < in; ++k) {
                const double xv = (double)half_bits_to_float(x_f16[t * in + k]);
                acc_base += xv * (double)half_bits_to_float(w_base_f16[n * in + k]);
                acc_delta += (double)sign_of_bit(srow, k) * xv;
            }
            y_f64[t * out + n] = acc_base + (double)alpha_by_tenant[tenant_of_token[t]] * acc_delta;
        }
    }
    return 0;
}

// ---- Sec. 4.2 (fidelity of Delta): the compressor iterated k times ----------
// Iteration j treats W_base + sum_{i<j} alpha_i S_i as the base model: its delta is the residual
//   r_0 = f32(W_fine) - f32(W_base),   r_{j+1} = r_j - alpha_j * Sign(r_j)      (binary32)
// and it emits plane j = sign bits of r_j (Eq. 2) and alpha_j = mean |r_j| (Eq. 4, binary64 sum,
// one rounding to binary16).  packed: [k][out][in/32]; alpha, alpha_unrounded: [k];
// residual_sq (may be null): [k+1], sum of r_j^2 in binary64 before each iteration and after the last.
int bd_ref_compress_iterated(const uint16_t* w_base_f16, const uint16_t* w_ft_f16, int64_t out, int64_t in,
                             int32_t k, uint32_t* packed, float* alpha_f16_as_float, double* alpha_unrounded,
                             double* residual_sq) {
    if (in % 32 != 0 || k < 1) return -1;
    const int64_t words = in / 32, count = out * in;
    std::vector<float> r((size_t)count);
    for (int64_t i = 0; i < count; ++i) r[(size_t)i] = half_bits_to_float(w_ft_f16[i]) - half_bits_to_float(w_base_f16[i]);
    std::vector<double> row_abs((size_t)out), row_sq((size_t)out);
    for (int32_t j = 0; j <= k; ++j) {
#pragma omp parallel for schedule(static)
        for (int64_t n = 0; n < out; ++n) {
            double sa = 0.0, sq = 0.0;
            for (int64_t c = 0; c < in; ++c) {
                const double v = (double)r[(size_t)(n * in + c)];
                sa += std::fabs(v);
                sq += v * v;
            }
            row_abs[(size_t)n] = sa;
            row_sq[(size_t)n] = sq;
        }
        double total_abs = 0.0, total_sq = 0.0;
        for (int64_t n = 0; n < out; ++n) {
            total_abs += row_abs[(size_t)n];
            total_sq += row_sq[(size_t)n];
        }
        if (residual_sq) residual_sq[j] = total_sq;
        if (j == k) break;
        const double mean = count > 0 ? total_abs / (double)count : 0.0;
        const float a = half_bits_to_float(double_to_half_bits(mean));
        if (alpha_unrounded) alpha_unrounded[j] = mean;
        alpha_f16_as_float[j] = a;
        uint32_t* plane = packed + (int64_t)j * out * words;
#pragma omp parallel for schedule(static)
        for (int64_t n = 0; n < out; ++n) {
            for (int64_t w = 0; w < words; ++w) {
                uint32_t word = 0;
                for (int b = 0; b < 32; ++b) {
                    float& v = r[(size_t)(n * in + w * 32 + b)];
                    const bool plus = v > 0.0f;
                    if (plus) word |= (1u << b);
                    v = plus ? v - a : v + a;          // r - alpha * (+-1)
                }
                plane[n * words + w] = word;
            }
        }
    }
    return 0;
}

// ---- Eq. 6 with k sign planes per tenant -------------------------------------
//   y[t,n] = sum_k x W_base  +  sum_{j<k} alpha_{e,j} * (sum_k x s_{e,j}),   e = tenant(t)
// planes[e * k + j]: [out, in/32]; alpha[e * k + j].  Every sum over the reduction index is binary32,
// ascending; the planes are added to the base product in ascending j; one rounding to binary16.
int bd_ref_linear_multitenant_kbit(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                   const uint32_t* const* planes, const float* alpha,
                                   const int32_t* tenant_of_token, uint16_t* y_f16, float* y_f32,
                                   int64_t T, int64_t out, int64_t in, int32_t n_tenants, int32_t k) {
    if (in % 32 != 0 || k < 1) return -1;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return -2;
    const int64_t words = in / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        for (int64_t t = 0; t < T; ++t) {
            const int64_t e = tenant_of_token[t];
            float y = 0.0f;
            for (int64_t c = 0; c < in; ++c)
                y += half_bits_to_float(x_f16[t * in + c]) * half_bits_to_float(w_base_f16[n * in + c]);
            for (int32_t j = 0; j < k; ++j) {
                const uint32_t* srow = planes[e * k + j] + n * words;
                float acc = 0.0f;
                for (int64_t c = 0; c < in; ++c) {
                    const float xv = half_bits_to_float(x_f16[t * in + c]);
                    acc += sign_of_bit(srow, c) > 0 ? xv : -xv;
                }
                y += alpha[e * k + j] * acc;
            }
            if (y_f32) y_f32[t * out + n] = y;
            if (y_f16) y_f16[t * out + n] = float_to_half_bits(y);
        }
    }
    return 0;
}

// binary64 accumulation, no output rounding
int bd_ref_linear_multitenant_kbit_f64(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                       const uint32_t* const* planes, const float* alpha,
                                       const int32_t* tenant_of_token, double* y_f64,
                                       int64_t T, int64_t out, int64_t in, int32_t n_tenants, int32_t k) {
    if (in % 32 != 0 || k < 1) return -1;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return -2;
    const int64_t words = in / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        for (int64_t t = 0; t < T; ++t) {
            const int64_t e = tenant_of_token[t];
            double y = 0.0;
            for (int64_t c = 0; c < in; ++c)
                y += (double)half_bits_to_float(x_f16[t * in + c]) * (double)half_bits_to_float(w_base_f16[n * in + c]);
            for (int32_t j = 0; j < k; ++j) {
                const uint32_t* srow = planes[e * k + j] + n * words;
                double acc = 0.0;
                for (int64_t c = 0; c < in; ++c)
                    acc += (double)sign_of_bit(srow, c) * (double)half_bits_to_float(x_f16[t * in + c]);
                y += (double)alpha[e * k + j] * acc;
            }
            y_f64[t * out + n] = y;
        }
    }
    return 0;
}

// ---- Sec. 4.2 (quantized base models): 8-bit round-to-nearest base ----------
// q [out, in] int8, scale [out] binary32.
int bd_ref_quantize_rtn8(const uint16_t* w_f16, int64_t out, int64_t in, int8_t* q, float* scale) {
    for (int64_t n = 0; n < out; ++n) {
        float amax = 0.0f;
        for (int64_t c = 0; c < in; ++c) {
            const float a = std::fabs(half_bits_to_float(w_f16[n * in + c]));
            if (a > amax) amax = a;          // NaN never compares greater: it does not enter the scale
        }
        const float s = amax > 0.0f ? amax / 127.0f : 1.0f;
        scale[n] = s;
        for (int64_t c = 0; c < in; ++c) {
            float v = std::nearbyintf(half_bits_to_float(w_f16[n * in + c]) / s);   // default rounding mode: to nearest even
            if (!(v >= -127.0f)) v = -127.0f;   // also catches NaN
            if (v > 127.0f) v = 127.0f;
            q[n * in + c] = (int8_t)v;
        }
    }
    return 0;
}

// The compressor of Sec. 3.1 against a quantised base: Delta = f32(W_fine) - scale[n] * q[n,k]  (binary32)
int bd_ref_compress_q8(const int8_t* q, const float* scale, const uint16_t* w_ft_f16, int64_t out, int64_t in,
                       uint32_t* packed, float* alpha_f16_as_float, double* alpha_unrounded) {
    if (in % 32 != 0) return -1;
    const int64_t words = in / 32;
    std::vector<double> row_sum((size_t)out, 0.0);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        double s = 0.0;
        for (int64_t w = 0; w < words; ++w) {
            uint32_t word = 0;
            for (int j = 0; j < 32; ++j) {
                const int64_t idx = n * in + w * 32 + j;
                const float base = scale[n] * (float)q[idx];
                const float d = half_bits_to_float(w_ft_f16[idx]) - base;
                if (d > 0.0f) word |= (1u << j);
                s += (double)std::fabs(d);
            }
            packed[n * words + w] = word;
        }
        row_sum[(size_t)n] = s;
    }
    double total = 0.0;
    for (int64_t n = 0; n < out; ++n) total += row_sum[(size_t)n];
    const double mean = (out > 0 && in > 0) ? total / ((double)out * (double)in) : 0.0;
    if (alpha_unrounded) *alpha_unrounded = mean;
    if (alpha_f16_as_float) *alpha_f16_as_float = half_bits_to_float(double_to_half_bits(mean));
    return 0;
}

// Eq. 6 with the quantised base: y = sum_k x * (scale[n] * q[n,k]) + alpha * sum_k x * s, binary32, ascending k.
int bd_ref_linear_multitenant_q8(const uint16_t* x_f16, const int8_t* q, const float* scale,
                                 const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                 const int32_t* tenant_of_token, uint16_t* y_f16, float* y_f32,
                                 int64_t T, int64_t out, int64_t in, int32_t n_tenants) {
    if (in % 32 != 0) return -1;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return -2;
    const int64_t words = in / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        for (int64_t t = 0; t < T; ++t) {
            const uint32_t* srow = packed_by_tenant[tenant_of_token[t]] + n * words;
            float acc_base = 0.0f, acc_delta = 0.0f;
            for (int64_t c = 0; c < in; ++c) {
                const float xv = half_bits_to_float(x_f16[t * in + c]);
                acc_base += xv * (scale[n] * (float)q[n * in + c]);
                acc_delta += sign_of_bit(srow, c) > 0 ? xv : -xv;
            }
            const float y = acc_base + alpha_by_tenant[tenant_of_token[t]] * acc_delta;
            if (y_f32) y_f32[t * out + n] = y;
            if (y_f16) y_f16[t * out + n] = float_to_half_bits(y);
        }
    }
    return 0;
}

int bd_ref_linear_multitenant_q8_f64(const uint16_t* x_f16, const int8_t* q, const float* scale,
                                     const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                     const int32_t* tenant_of_token, double* y_f64,
                                     int64_t T, int64_t out, int64_t in, int32_t n_tenants) {
    if (in % 32 != 0) return -1;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return -2;
    const int64_t words = in / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        for (int64_t t = 0; t < T; ++t) {
            const uint32_t* srow = packed_by_tenant[tenant_of_token[t]] + n * words;
            double acc_base = 0.0, acc_delta = 0.0;
            for (int64_t c = 0; c < in; ++c) {
                const double xv = (double)half_bits_to_float(x_f16[t * in + c]);
                acc_base += xv * ((double)scale[n] * (double)q[n * in + c]);
                acc_delta += (double)sign_of_bit(srow, c) * xv;
            }
            y_f64[t * out + n] = acc_base + (double)alpha_by_tenant[tenant_of_token[t]] * acc_delta;
        }
    }
    return 0;
}

// ---- Eq. 6, left-hand side: the approximated fine-tuned weight, materialised
// W_eff[n,k] = f32(W_base[n,k]) + alpha * s[n,k]  (binary32, not rounded to
// binary16), y = sum_k x * W_eff in binary32, ascending k.  One tenant.
int bd_ref_linear_materialised(const uint16_t* x_f16, const uint16_t* w_base_f16, const uint32_t* packed,
                               float alpha, float* y_f32, float* abs_dot_f32,
                               int64_t T, int64_t out, int64_t in) {
    if (in % 32 != 0) return -1;
    const int64_t words = in / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        std::vector<float> weff((size_t)in);
        for (int64_t k = 0; k < in; ++k)
            weff[(size_t)k] = half_bits_to_float(w_base_f16[n * in + k]) + alpha * (float)sign_of_bit(packed + n * words, k);
        for (int64_t t = 0; t < T; ++t) {
            float acc = 0.0f, aabs = 0.0f;
            for (int64_t k = 0; k < in; ++k) {
                const float p = half_bits_to_float(x_f16[t * in + k]) * weff[(size_t)k];
                acc += p;
                aabs += std::fabs(p);
            }
            y_f32[t * out + n] = acc;
            if (abs_dot_f32) abs_dot_f32[t * out + n] = aabs;
        }
    }
    return 0;
}

// The naive system the paper compares with: every tenant keeps its own full
// binary16 matrix and tokens are multiplied by their tenant's matrix (Sec. 4.3).
// w_by_tenant[n_tenants] -> each [out, in] binary16.
int bd_ref_linear_naive(const uint16_t* x_f16, const uint16_t* const* w_by_tenant,
                        const int32_t* tenant_of_token, uint16_t* y_f16, float* y_f32,
                        int64_t T, int64_t out, int64_t in, int32_t n_tenants) {
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n) {
        for (int64_t t = 0; t < T; ++t) {
            const uint16_t* wrow = w_by_tenant[tenant_of_token[t]] + n * in;
            float acc = 0.0f;
            for (int64_t k = 0; k < in; ++k)
                acc += half_bits_to_float(x_f16[t * in + k]) * half_bits_to_float(wrow[k]);
            if (y_f32) y_f32[t * out + n] = acc;
            if (y_f16) y_f16[t * out + n] = float_to_half_bits(acc);
        }
    }
    return 0;
}

// W_t = f16( f32(W_base) + alpha * s )  -- the per-tenant matrix the naive
// baseline stores when it is fed BitDelta's approximation instead of W_fine.
int bd_ref_materialise_f16(const uint16_t* w_base_f16, const uint32_t* packed, float alpha,
                           uint16_t* w_out_f16, int64_t out, int64_t in) {
    if (in % 32 != 0) return -1;
    const int64_t words = in / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < out; ++n)
        for (int64_t k = 0; k < in; ++k)
            w_out_f16[n * in + k] = float_to_half_bits(
                half_bits_to_float(w_base_f16[n * in + k]) + alpha * (float)sign_of_bit(packed + n * words, k));
    return 0;
}

}  // extern "C"
