// Matrix-core decode kernel for the multi-tenant linear of Eq. 6 of the paper:
//     y[t, n] = sum_k x[t,k] W_base[n,k]  +  alpha_e * sum_k x[t,k] s_e[n,k],   e = tenant(t).
//
// Shape of the work.  At decode every token has its own tenant, so each packed sign word is
// used exactly once: the sign stream cannot be amortised over tokens and the kernel has to
// turn ~1 sign element per byte-of-base-weight into a multiply-add operand while the weights
// stream from HBM.  The vector ALU alone cannot do that at HBM speed on this chip, so the
// multiply-adds of both products go to v_mfma_f32_16x16x32_f16 and the vector ALU is left with
// nothing but the bit -> fp16 expansion (one and-or per pair of signs, see SignExpander).
//
// Decomposition.  A workgroup owns 16 consecutive output rows and all of K; its wavefronts
// split K in steps of 512.  In the MFMA the 16 A rows are the output rows, the 16 B columns
// are the tokens of one column tile (tokens sorted by tenant) and lane (r, g) = (lane % 16,
// lane / 16) supplies 8 reduction elements.  Because a contraction does not care in which
// order k is visited, every operand is loaded in the layout its memory wants:
//   base   lane (r,g), slice v: W[n0+r][k0 + 32v + 8g .. +8]   (64 contiguous bytes per row and load)
//   signs  lane (r,g): the four words covering k0 + 128g .. +128 of row n0+r (one 128-bit load)
//   x      staged once per step and wavefront in LDS, read back in either order.
// A delta "job" is one tenant's run of columns in a tile; its MFMA result is only valid in
// those columns, which are selected once per pass.  Jobs are processed in passes of 8/4/2/1 so
// that every pass is straight-line code.  Partial sums of the wavefronts are added in a fixed
// order through LDS, so results are deterministic and y is written exactly once.
#include "bd_device.h"
#include "bd_launch.h"

namespace bd {

constexpr int kStepK = 512;            // reduction elements one wavefront consumes per step
constexpr int kXsBlockBytes = 264;     // 128 fp16 of one column + 8 B pad (2 banks)
constexpr int kXsRowBytes = 1072;      // 4 blocks + 16 B pad: row stride = 4 * odd banks
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

__device__ __forceinline__ void lds_wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// All global loads are "uniform 64-bit base + 32-bit lane offset", the form that needs one
// address register per lane; the host guarantees every tensor is below 4 GiB.
__device__ __forceinline__ u32x4 load16(const void* base, uint32_t lane_off) {
    return *(const u32x4*)((const unsigned char*)base + lane_off);
}
__device__ __forceinline__ u32x4 load16_stream(const void* base, uint32_t lane_off) {
    return __builtin_nontemporal_load((const u32x4*)((const unsigned char*)base + lane_off));
}

struct LaneCtx {
    const uint16_t* x;
    const uint16_t* w;
    const uint32_t* const* packed_by_tenant;
    int64_t in;
    uint32_t woff;                         // byte offset of W[row][8 g]
    uint32_t soff;                         // byte offset of packed[row][4 g]
    uint32_t xoff;                         // byte offset 16 * lane inside a 512-element chunk of x
    unsigned char* xs;                     // this wavefront's LDS region
    unsigned char* xs_wr;                  // + column * kXsRowBytes
    const unsigned char* xs_base_rd;       // + (v/4)*264 + (v%4)*64
    const unsigned char* xs_delta_rd;      // + u*64 + m*8 (+32)
    int g, wave, n_waves, n_steps, n_tiles;
};

// x of one column tile, 512 reduction elements from k0 -> this wavefront's LDS region.
// Two batches of eight columns keep the transient registers at 32.  Columns beyond T and
// elements beyond `in` are written as zeros, so whatever the weight registers hold there
// multiplies zero.
__device__ __forceinline__ void stage_x(const LaneCtx& cx, const DecodeMeta& meta, int tile, int64_t k0, bool full,
                                        uint32_t xoff) {
    const bool kvalid = full || (k0 + (xoff >> 1) < cx.in);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        u32x4 v[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int col = tile * 16 + half * 8 + c;
            v[c] = u32x4{0u, 0u, 0u, 0u};
            if (col < meta.T) {
                const uint16_t* colbase = cx.x + (int64_t)meta.token_of_col[col] * cx.in + k0;
                if (kvalid) v[c] = load16(colbase, xoff);
            }
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) *(u32x4*)(cx.xs_wr + (half * 8 + c) * kXsRowBytes) = v[c];
        __builtin_amdgcn_sched_barrier(0);
    }
}

// One pass: JP delta jobs of column tile `tile` over all of this wavefront's steps.  A BASE
// pass also streams W (once per call) and builds the base product of tile 0, and of tile 1
// when there is one.  In mantissa mode every pass rebuilds the H term of its tile (one MFMA
// per slice, the same value each time), which keeps the pass free of flags.
template <int JP, int MODE, bool BASE>
__device__ __forceinline__ void run_pass(const LaneCtx& cx, const DecodeMeta& meta, const ExpandConsts<MODE>& kc,
                                         int tile, int job0, float4v (&accb)[2], float4v& accb1, float4v& acch,
                                         float4v (&acc)[JP]) {
    const uint32_t* sptr[JP];
#pragma unroll
    for (int j = 0; j < JP; ++j) {
        acc[j] = float4v{0.f, 0.f, 0.f, 0.f};
        sptr[j] = cx.packed_by_tenant[meta.job_tenant[job0 + j]];
    }
    acch = float4v{0.f, 0.f, 0.f, 0.f};
    for (int step = cx.wave; step < cx.n_steps; step += cx.n_waves) {
        const int64_t k0 = (int64_t)step * kStepK;
        const bool full = k0 + kStepK <= cx.in;
        // Lane offsets are re-read through an empty asm every step: otherwise the compiler hoists
        // "uniform base + lane offset" of every load out of the loop as 64-bit register pairs.
        uint32_t woff = cx.woff, soff = cx.soff, xoff = cx.xoff;
        asm volatile("" : "+v"(woff), "+v"(soff), "+v"(xoff));
        // ---- long-latency loads first: base slices and sign words
        u32x4 wreg[BASE ? 16 : 1];
        if constexpr (BASE) {
            const uint16_t* wk = cx.w + k0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                wreg[v] = u32x4{0u, 0u, 0u, 0u};
                if (full || k0 + 32 * v < cx.in) wreg[v] = load16_stream(wk + 32 * v, woff);
            }
        }
        u32x4 sreg[JP];
        const bool svalid = full || (k0 + 128 * cx.g < cx.in);
#pragma unroll
        for (int j = 0; j < JP; ++j) {
            sreg[j] = u32x4{0u, 0u, 0u, 0u};
            if (svalid) sreg[j] = load16_stream(sptr[j] + (k0 >> 5), soff);
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- x of this tile and step -> LDS
        stage_x(cx, meta, tile, k0, full, xoff);
        lds_wave_sync();

        if constexpr (BASE) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const half8 b = *(const half8*)(cx.xs_base_rd + (v >> 2) * kXsBlockBytes + (v & 3) * 64);
                accb[v & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, wreg[v]), b, accb[v & 1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            WordState<MODE> ws[JP];
#pragma unroll
            for (int j = 0; j < JP; ++j) ws[j].set(sreg[j][u]);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const u32x2 lo = *(const u32x2*)(cx.xs_delta_rd + u * 64 + m * 8);
                const u32x2 hi = *(const u32x2*)(cx.xs_delta_rd + u * 64 + m * 8 + 32);
                const half8 bd = as_half8(__builtin_amdgcn_perm(hi[0], lo[0], 0x05040100u),
                                          __builtin_amdgcn_perm(hi[0], lo[0], 0x07060302u),
                                          __builtin_amdgcn_perm(hi[1], lo[1], 0x05040100u),
                                          __builtin_amdgcn_perm(hi[1], lo[1], 0x07060302u));
                if constexpr (MODE == kMantissa) {
                    const int pb = (m & 1) * 4 + 2;
                    const half8 hop = as_half8(kc.hreg[pb - 2], kc.hreg[pb - 1], kc.hreg[pb], kc.hreg[pb + 1]);
                    acch = __builtin_amdgcn_mfma_f32_16x16x32_f16(hop, bd, acch, 0, 0, 0);
                }
#pragma unroll
                for (int j = 0; j < JP; ++j) {
                    const half8 a = as_half8(ws[j].reg(4 * m, kc), ws[j].reg(4 * m + 1, kc), ws[j].reg(4 * m + 2, kc),
                                             ws[j].reg(4 * m + 3, kc));
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bd, acc[j], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);   // keep the expansion of one slice next to its MFMAs
            }
        }
        // ---- second column tile's base product while this step's W is still in registers
        if constexpr (BASE) {
            if (cx.n_tiles > 1) {
                __builtin_amdgcn_wave_barrier();
                stage_x(cx, meta, 1, k0, full, xoff);
                lds_wave_sync();
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const half8 b = *(const half8*)(cx.xs_base_rd + (v >> 2) * kXsBlockBytes + (v & 3) * 64);
                    accb1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, wreg[v]), b, accb1, 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();   // the next step's staging must not overtake these reads
    }
}

// Keep, per lane, the result of the job that owns this lane's column.
template <int JP>
__device__ __forceinline__ void select_columns(const DecodeMeta& meta, const float* __restrict__ alpha_by_tenant, int job0,
                                               int c, const float4v (&acc)[JP], float4v& dsel, float& alpha_c) {
#pragma unroll
    for (int j = 0; j < JP; ++j) {
        const bool mine = c >= meta.job_col_begin[job0 + j] && c < meta.job_col_end[job0 + j];
        const float a = alpha_by_tenant[meta.job_tenant[job0 + j]];
        dsel = mine ? acc[j] : dsel;
        alpha_c = mine ? a : alpha_c;
    }
}

template <int JP, int MODE>
__device__ __forceinline__ void pass_and_select(const LaneCtx& cx, const DecodeMeta& meta, const ExpandConsts<MODE>& kc,
                                                const float* __restrict__ alpha_by_tenant, int tile, int job0, bool base,
                                                int c, float4v (&accb)[2], float4v& accb1, float4v& acch, float4v& dsel,
                                                float& alpha_c) {
    float4v acc[JP];
    if (base) run_pass<JP, MODE, true>(cx, meta, kc, tile, job0, accb, accb1, acch, acc);
    else run_pass<JP, MODE, false>(cx, meta, kc, tile, job0, accb, accb1, acch, acc);
    select_columns<JP>(meta, alpha_by_tenant, job0, c, acc, dsel, alpha_c);
}

template <int MODE>
__global__ __launch_bounds__(kMaxWaves * kWave) void linear_decode_mfma_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
    const uint32_t* const* __restrict__ packed_by_tenant, const float* __restrict__ alpha_by_tenant,
    const DecodeMeta meta, uint16_t* __restrict__ y, const int64_t out, const int64_t in) {
    extern __shared__ __align__(16) unsigned char smem[];
    LaneCtx cx;
    const int lane = threadIdx.x & (kWave - 1);
    cx.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, and the compiler knows it
    cx.n_waves = blockDim.x >> 6;
    const int c = lane & 15;          // A row (output row) for loads, B/D column (token) for MFMA results
    cx.g = lane >> 4;
    cx.xs = smem + cx.wave * kXsWaveBytes;
    const int64_t n0 = (int64_t)blockIdx.x * 16;
    const int64_t nrow = (n0 + c < out) ? n0 + c : out - 1;   // clamp: padded rows repeat the last row
    cx.n_steps = (int)((in + kStepK - 1) / kStepK);
    cx.n_tiles = (meta.T + 15) >> 4;
    cx.in = in;
    cx.x = x;
    cx.w = w;
    cx.packed_by_tenant = packed_by_tenant;
    cx.woff = (uint32_t)((nrow * in + 8 * cx.g) * 2);
    cx.soff = (uint32_t)((nrow * (in >> 5) + 4 * cx.g) * 4);
    cx.xoff = (uint32_t)(16 * lane);
    cx.xs_wr = cx.xs + (lane >> 4) * kXsBlockBytes + (lane & 15) * 16;
    cx.xs_base_rd = cx.xs + c * kXsRowBytes + cx.g * 16;
    cx.xs_delta_rd = cx.xs + c * kXsRowBytes + cx.g * kXsBlockBytes;
    const ExpandConsts<MODE> kc;

    float4v ypart0 = {0.f, 0.f, 0.f, 0.f}, ypart1 = {0.f, 0.f, 0.f, 0.f};
    float4v accb1 = {0.f, 0.f, 0.f, 0.f};   // base product of the second column tile, built during the first pass

    int job = 0;
    for (int tile = 0; tile < cx.n_tiles; ++tile) {
        int job_end = job;
        while (job_end < meta.n_jobs && meta.job_tile[job_end] == tile) ++job_end;
        float4v accb[2] = {float4v{0.f, 0.f, 0.f, 0.f}, float4v{0.f, 0.f, 0.f, 0.f}};
        float4v acch = {0.f, 0.f, 0.f, 0.f};
        float4v dsel = {0.f, 0.f, 0.f, 0.f};
        float alpha_c = 0.f;
        bool base = (tile == 0);     // W streams exactly once, in the first pass of the first tile
        while (job < job_end) {      // the host guarantees at least one job per tile
            const int left = job_end - job;
            if (left >= 8) {
                pass_and_select<8, MODE>(cx, meta, kc, alpha_by_tenant, tile, job, base, c, accb, accb1, acch, dsel, alpha_c);
                job += 8;
            } else if (left >= 4) {
                pass_and_select<4, MODE>(cx, meta, kc, alpha_by_tenant, tile, job, base, c, accb, accb1, acch, dsel, alpha_c);
                job += 4;
            } else if (left >= 2) {
                pass_and_select<2, MODE>(cx, meta, kc, alpha_by_tenant, tile, job, base, c, accb, accb1, acch, dsel, alpha_c);
                job += 2;
            } else {
                pass_and_select<1, MODE>(cx, meta, kc, alpha_by_tenant, tile, job, base, c, accb, accb1, acch, dsel, alpha_c);
                job += 1;
            }
            base = false;
        }
        float4v bsum = accb[0] + accb[1];
        if (tile == 1) bsum = accb1;
        float4v d = dsel;
        if constexpr (MODE == kMantissa) d = 4.0f * dsel - acch;
        if (tile == 0) ypart0 = bsum + alpha_c * d;
        else ypart1 = bsum + alpha_c * d;
    }

    // ---- add the wavefronts' partial tiles in a fixed order and write y once
    __syncthreads();   // every wavefront is done with its staging region
    float* red = (float*)cx.xs;   // [tile][col][row] of this wavefront
    *(float4v*)(red + c * 16 + 4 * cx.g) = ypart0;
    if (cx.n_tiles > 1) *(float4v*)(red + 256 + c * 16 + 4 * cx.g) = ypart1;
    __syncthreads();
    for (int idx = threadIdx.x; idx < cx.n_tiles * 256; idx += blockDim.x) {
        const int tile = idx >> 8, col = (idx >> 4) & 15, row = idx & 15;
        const int gcol = tile * 16 + col;
        if (gcol < meta.T && n0 + row < out) {
            float s = 0.f;
            for (int wv = 0; wv < cx.n_waves; ++wv)
                s += *(const float*)(smem + wv * kXsWaveBytes + (tile * 256 + col * 16 + row) * 4);
            y[(int64_t)meta.token_of_col[gcol] * out + n0 + row] = f2h_rne(s);
        }
    }
}

bool decode_mfma_variant_known(int variant) { return variant == 2 || variant == 3; }

template <int MODE>
static hipError_t launch_one(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                             const float* alpha_by_tenant, const DecodeMeta& meta, uint16_t* y, int64_t out, int64_t in,
                             hipStream_t st) {
    const int n_steps = (int)((in + kStepK - 1) / kStepK);
    const int n_waves = n_steps < kMaxWaves ? n_steps : kMaxWaves;
    const size_t lds = (size_t)n_waves * kXsWaveBytes;
    auto kernel = linear_decode_mfma_kernel<MODE>;
    static bool attr_set = false;   // raising the dynamic LDS limit is idempotent; a race only repeats it
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           kMaxWaves * kXsWaveBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)((out + 15) / 16)), dim3(n_waves * kWave), lds, st, x, w,
                       packed_by_tenant, alpha_by_tenant, meta, y, out, in);
    return hipGetLastError();
}

// variant 2 = plain +-1 expansion, variant 3 = mantissa expansion.
// Requires in % 128 == 0 and every tensor (W, x, each packed delta) below 4 GiB.
hipError_t launch_linear_decode_mfma(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                     const float* alpha_by_tenant, const DecodeMeta& meta, uint16_t* y, int64_t out,
                                     int64_t in, int variant, hipStream_t st) {
    switch (variant) {
        case 2: return launch_one<kPlain>(x, w, packed_by_tenant, alpha_by_tenant, meta, y, out, in, st);
        case 3: return launch_one<kMantissa>(x, w, packed_by_tenant, alpha_by_tenant, meta, y, out, in, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace bd
