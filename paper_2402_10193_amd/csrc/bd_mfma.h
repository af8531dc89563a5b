// Pieces shared by the matrix-core decode kernels: the sign-word -> fp16 operand expansion, the
// LDS staging geometry of x and a few small helpers.
#pragma once

#include "bd_device.h"

namespace bd {

constexpr int kStepK = 512;            // reduction elements one wavefront consumes per step
constexpr int kXsRowBytes = 1040;      // 512 fp16 of one column + 16 B pad: row stride = 4 * odd banks
constexpr int kXsWaveBytes = 16 * kXsRowBytes;
constexpr int kMaxWaves = 8;

// ---- sign word -> fp16 operands ------------------------------------------------------------
// Register j (0..15) of a word carries the elements k = j (low half) and k = j + 16 (high
// half); MFMA slice m uses registers 4m .. 4m+3.
//
// kPlain:    each half is +1.0 or -1.0: shift the (inverted) bit pair onto the two fp16 sign
//            bits, then one and-or.  Two vector instructions per pair.
// kMantissa: the bit is left in the fp16 *mantissa*: with the exponent chosen per bit position
//            p (2..9) as 2^(9-p), the half reads 2^(9-p) + b/2, so the product sum becomes
//            sum_k 2^(9-p(k)) x_k + (1/2) sum_k b_k x_k.  The first term does not depend on the
//            row or the tenant: it is produced once per step by one more MFMA whose A operand
//            holds the constants 2^(11-p) + 1, giving H = sum_k (2^(11-p(k)) + 1) x_k, and
//            sum_k s_k x_k = 4 acc - H exactly in real arithmetic.  Only two shifts per word are
//            needed, so the expansion costs 18 instead of 32 vector instructions per 32 signs.
//            Price: acc carries terms up to 2^7 |x|, i.e. 7 of the 24 accumulator bits.
enum UnpackMode { kPlain = 0, kMantissa = 1 };

// Constants of the expansion, held in registers the compiler cannot fold back into literals
// (a literal operand would split every and-or into two instructions on this ISA).
template <int MODE>
struct ExpandConsts;

__device__ __forceinline__ uint32_t opaque_s(uint32_t v) {
    asm("" : "+s"(v));
    return v;
}
__device__ __forceinline__ uint32_t opaque_v(uint32_t v) {
    asm("" : "+v"(v));
    return v;
}

template <>
struct ExpandConsts<kPlain> {
    uint32_t mask, one;
    __device__ __forceinline__ ExpandConsts() : mask(opaque_s(0x80008000u)), one(opaque_v(0x3C003C00u)) {}
};

template <>
struct ExpandConsts<kMantissa> {
    uint32_t mask[8];   // bit p (2..9) of both halves
    uint32_t expo[8];   // fp16 2^(9-p) in both halves
    uint32_t hreg[8];   // fp16 2^(11-p) + 1 in both halves: the A operand of the H product
    __device__ __forceinline__ ExpandConsts() {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int p = i + 2;
            mask[i] = opaque_s(0x00010001u << p);
            expo[i] = opaque_v((uint32_t)((24 - p) << 10) * 0x00010001u);
            hreg[i] = opaque_v(hconst(p));
        }
    }
    // fp16 bits of 2^(11-p) + 1 in both halves: exponent field 26-p, mantissa bit p-1
    __device__ __forceinline__ static constexpr uint32_t hconst(int p) {
        return (uint32_t)(((26 - p) << 10) | (1u << (p - 1))) * 0x00010001u;
    }
};

// Per word state (what has to stay live while the four slices of a word are consumed).
template <int MODE>
struct WordState;

template <>
struct WordState<kPlain> {
    uint32_t nw;
    __device__ __forceinline__ void set(uint32_t word) { nw = ~word; }
    __device__ __forceinline__ uint32_t reg(int j, const ExpandConsts<kPlain>& k) const {
        return ((nw << (15 - j)) & k.mask) | k.one;
    }
};

template <>
struct WordState<kMantissa> {
    uint32_t ta, tb;
    __device__ __forceinline__ void set(uint32_t word) {
        ta = word << 2;   // bits 0..7 / 16..23 -> mantissa positions 2..9 of the low / high half
        tb = word >> 6;   // bits 8..15 / 24..31 -> the same positions
    }
    __device__ __forceinline__ uint32_t reg(int j, const ExpandConsts<kMantissa>& k) const {
        const uint32_t t = (j < 8) ? ta : tb;
        return (t & k.mask[j & 7]) | k.expo[j & 7];
    }
};

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    const u32x4 v = {a, b, c, d};
    return __builtin_bit_cast(half8, v);
}

// s_waitcnt immediate that waits only for the vector-memory counter (gfx9 encoding: vmcnt in
// bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
__device__ __forceinline__ constexpr int vmcnt_only(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }

__device__ __forceinline__ void lds_wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// All global loads are "uniform 64-bit base + 32-bit lane offset", the form that needs one
// address register per lane; the host guarantees every tensor is below 4 GiB.
__device__ __forceinline__ u32x4 load16_stream(const void* base, uint32_t lane_off) {
    return *(const u32x4*)((const unsigned char*)base + lane_off);
}

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

}  // namespace bd
