// Decode kernel of the multi-tenant linear (Eq. 6 of the paper) over the tiled serving layout:
//     y[t, n] = sum_k x[t,k] W_base[n,k]  +  alpha_e * sum_k x[t,k] s_e[n,k],   e = tenant(t).
//
// At decode every token has its own tenant, so a packed sign word is used exactly once and
// the kernel is a pure stream: per byte of base weight it must turn B/16 sign bits into
// multiply-add operands.  Both products run on v_mfma_f32_16x16x32_f16 (A = 16 output rows x
// 32 k, B = 32 k x 16 token columns, tokens sorted by tenant); a delta "job" is one tenant's
// signs against all 16 columns, of which only that tenant's columns are kept.
//
// Sign expansion.  A byte of 8 signs becomes the 8 fp16 values +-1.0 (one 128-bit MFMA operand
// register group) by ONE look-up in LDS: the table has 256 entries x 16 B, replicated 16 times
// so that lane l reads copy l % 16 and a group of 16 lanes never shares a bank.  The address
// is built by one v_perm_b32 (sign byte -> address bits 8..15, lane copy -> bits 4..7), so the
// vector ALU spends one instruction per 8 signs; the LDS read port does the rest, next to the
// matrix pipe.  (Expanding with and-or instructions costs >= 8 per 8 signs and, at one token per
// tenant, makes the vector ALU the bottleneck long before HBM.)
//
// Decomposition.  A workgroup owns 16 output rows; its wavefronts split the k tiles into
// contiguous ranges.  Per tile a wavefront needs 8 KiB of base (8 loads), 512 B of signs per
// job (one 64-bit load per lane) and the 16 x 256 block of x, which each lane loads straight
// from global memory (L2 hits) in B-operand order: no staging, no barrier in the loop.
// Everything of step s+1 is requested while step s is being multiplied: W[v] right after its
// MFMA, the signs of job j right after their addresses are formed, x into a second register
// set.  Partial sums of the wavefronts are added in a fixed order through LDS; y is written once.
#include <type_traits>

#include "bd_device.h"
#include "bd_tiled.h"

namespace bd {

namespace {

constexpr int kLutBytes = 256 * 16 * 16;          // 256 entries x 16 copies x 16 B
constexpr int kRedBytesPerWave = 16 * 16 * 4;     // one 16 x 16 fp32 tile
constexpr int kMaxWavesTiled = 8;

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef const u32x4 __attribute__((address_space(3)))* lds_u32x4_ptr;

__device__ __forceinline__ u32x4 ldg16_stream(const unsigned char* base, uint32_t off) {
    return __builtin_nontemporal_load((const u32x4*)(base + off));
}
__device__ __forceinline__ u32x2 ldg8_stream(const unsigned char* base, uint32_t off) {
    return __builtin_nontemporal_load((const u32x2*)(base + off));
}
__device__ __forceinline__ u32x4 ldg16(const unsigned char* base, uint32_t off) {
    return *(const u32x4*)(base + off);
}

// The eight operands of one job's tile: byte v of the lane's sign words -> table entry.
// `lanebits` = 16 * (lane % 16) in byte 0; the selector puts sign byte (v % 4) of word v / 4
// into byte 1 and zeros above: address = 256 * byte + 16 * copy (the table starts at LDS address 0).
__device__ __forceinline__ void lut_issue(const u32x2 s, const uint32_t lanebits, u32x4 (&a)[8]) {
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const uint32_t addr = __builtin_amdgcn_perm(s[v >> 2], lanebits, 0x0C0C0000u | ((4u + (v & 3)) << 8));
        a[v] = *(lds_u32x4_ptr)(uintptr_t)addr;
    }
}

}  // namespace

template <int NJ>
__global__ __launch_bounds__(kMaxWavesTiled * kWave) void linear_decode_tiled_kernel(const TiledArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];   // [0, 64 KiB): table; then one fp32 tile per wavefront
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    const int c = lane & 15;   // A row (output row) for loads, B/D column (token) for MFMA operands and results
    const int g = lane >> 4;

    // which matrix of the launch this workgroup belongs to
    int m = 0, rb = blockIdx.x;
    if (a.n_mats > 1 && rb >= a.rb_end[0]) m = 1;
    if (a.n_mats > 2 && rb >= a.rb_end[1]) m = 2;
    if (m > 0) rb -= a.rb_end[m - 1];
    const int KT = a.KT;
    const int kb = wave * KT / nw, ke = (wave + 1) * KT / nw;   // this wavefront's k tiles
    const int steps = ke - kb;

    const unsigned char* wt = (const unsigned char*)a.wt[m];
    const unsigned char* xg = (const unsigned char*)a.x;
    const unsigned char* sp[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) sp[j] = (const unsigned char*)a.signs[m][j];
    uint32_t woff = (uint32_t)(rb * KT + kb) * (uint32_t)kTileBaseBytes + (uint32_t)lane * 16u;
    uint32_t soff = (uint32_t)(rb * KT + kb) * (uint32_t)kTileSignBytes + (uint32_t)lane * 8u;

    // this lane's column: token row of x, owning job, scale
    int tok = a.col_token[0], myjob = -1, tenant = 0;
#pragma unroll
    for (int i = 0; i < kTiledMaxTokens; ++i) {
        tok = (c == i && i < a.T) ? a.col_token[i] : tok;
        myjob = (c == i && i < a.T) ? a.col_job[i] : myjob;
        tenant = (c == i && i < a.T) ? a.col_tenant[i] : tenant;
    }
    // columns beyond T read token col_token[0]'s x (valid memory); their results are never stored
    uint32_t xoff = (uint32_t)tok * (uint32_t)a.in * 2u + (uint32_t)g * 16u + (uint32_t)kb * (uint32_t)(kTileK * 2);
    const int k_ragged = (a.in % kTileK != 0) ? KT - 1 : -1;   // the tile that reaches beyond `in`, if any

    auto load_x = [&](u32x4 (&xr)[8], const int kt, const uint32_t off) {
        if (kt != k_ragged) {
#pragma unroll
            for (int v = 0; v < 8; ++v) xr[v] = ldg16(xg, off + v * 64);
        } else {
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                xr[v] = u32x4{0u, 0u, 0u, 0u};
                if (kt * kTileK + 32 * v + 8 * g < a.in) xr[v] = ldg16(xg, off + v * 64);
            }
        }
    };

    // ---- requests of the first step, in the order they are consumed
    u32x4 wr[8], xc[8];
    u32x2 sr[NJ];
    if (steps > 0) {
#pragma unroll
        for (int v = 0; v < 8; ++v) wr[v] = ldg16_stream(wt, woff + v * 1024);
        load_x(xc, kb, xoff);
#pragma unroll
        for (int j = 0; j < NJ; ++j) sr[j] = ldg8_stream(sp[j], soff);
    } else {
#pragma unroll
        for (int v = 0; v < 8; ++v) wr[v] = xc[v] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < NJ; ++j) sr[j] = u32x2{0u, 0u};
    }
    const float alpha_c = a.alpha[m][tenant];

    // ---- the table: entry b, copy cp at 256 b + 16 cp; element e = bit e of b ? +1.0 : -1.0
    for (int idx = threadIdx.x; idx < 256 * 16; idx += blockDim.x) {
        const uint32_t b = (uint32_t)idx >> 4;
        u32x4 e;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            e[i] = 0xBC00BC00u ^ (((b >> (2 * i)) & 1u) << 15) ^ (((b >> (2 * i + 1)) & 1u) << 31);
        *(u32x4*)(smem + idx * 16) = e;
    }
    __syncthreads();
    const uint32_t lanebits = (uint32_t)c << 4;

    float4v accb = {0.f, 0.f, 0.f, 0.f}, dsel = {0.f, 0.f, 0.f, 0.f};

    // One step = one tile.  MORE: there is a next tile, request it while this one is multiplied.
    auto step = [&](auto more_tag, const int kt) {
        constexpr bool MORE = decltype(more_tag)::value;
        // ---- base product; W[v] of the next tile goes into the register group just read
        if constexpr (MORE) woff += kTileBaseBytes;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            accb = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, wr[v]), __builtin_bit_cast(half8, xc[v]),
                                                          accb, 0, 0, 0);
            if constexpr (MORE) wr[v] = ldg16_stream(wt, woff + v * 1024);
        }
        u32x4 xn[8];
        if constexpr (MORE) {
            xoff += kTileK * 2;
            load_x(xn, kt + 1, xoff);
            soff += kTileSignBytes;
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- delta jobs: table look-ups of job j+1 are in flight while job j is multiplied
        u32x4 cur[8], nxt[8];
        float4v sel = {0.f, 0.f, 0.f, 0.f};   // the job owning this lane's column, this tile
        lut_issue(sr[0], lanebits, cur);
        if constexpr (MORE) sr[0] = ldg8_stream(sp[0], soff);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (j + 1 < NJ) {
                lut_issue(sr[j + 1], lanebits, nxt);
                if constexpr (MORE) sr[j + 1] = ldg8_stream(sp[j + 1], soff);
            }
            float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int v = 0; v < 8; ++v)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, cur[v]),
                                                             __builtin_bit_cast(half8, xc[v]), acc, 0, 0, 0);
            const bool mine = (myjob == j);
#pragma unroll
            for (int i = 0; i < 4; ++i) sel[i] = mine ? acc[i] : sel[i];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int v = 0; v < 8; ++v) cur[v] = nxt[v];
        }
        dsel += sel;
        if constexpr (MORE) {
#pragma unroll
            for (int v = 0; v < 8; ++v) xc[v] = xn[v];
        }
    };
    for (int s = 0; s + 1 < steps; ++s) step(std::true_type{}, kb + s);
    if (steps > 0) step(std::false_type{}, ke - 1);

    // ---- add the wavefronts' partial tiles in a fixed order and write y once
    float* red = (float*)(smem + kLutBytes);
    {
        float4v r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = accb[i] + alpha_c * dsel[i];
        *(float4v*)(red + wave * 256 + c * 16 + 4 * g) = r;   // [column][row]
    }
    __syncthreads();
    const int n0 = rb * kTileRows;
    const int out = a.out[m];
    uint16_t* y = a.y[m];
    for (int idx = threadIdx.x; idx < 256; idx += blockDim.x) {
        const int col = idx >> 4, row = idx & 15;
        if (col < a.T && n0 + row < out) {
            float s = 0.f;
            for (int wv = 0; wv < nw; ++wv) s += red[wv * 256 + idx];
            y[(int64_t)a.col_token[col] * out + n0 + row] = f2h_rne(s);
        }
    }
}

template <int NJ>
static hipError_t launch_nj(const TiledArgs& args, int n_waves, unsigned grid, hipStream_t st) {
    auto kernel = linear_decode_tiled_kernel<NJ>;
    const size_t lds = (size_t)kLutBytes + (size_t)kMaxWavesTiled * kRedBytesPerWave;
    static bool attr_set = false;   // raising the dynamic LDS limit is idempotent; a race only repeats it
    if (!attr_set) {
        hipFuncAttributes fa;
        hipError_t e = hipFuncGetAttributes(&fa, (const void*)kernel);
        if (e != hipSuccess) return e;
        if (fa.sharedSizeBytes != 0) return hipErrorInvalidValue;   // the table must start at LDS address 0
        e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(n_waves * kWave), lds, st, args);
    return hipGetLastError();
}

hipError_t launch_linear_decode_tiled(const TiledArgs& args, int n_jobs, hipStream_t st) {
    if (n_jobs < 1 || n_jobs > kTiledMaxJobs || args.n_mats < 1 || args.n_mats > kTiledMaxMats) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)args.rb_end[args.n_mats - 1];
    // One workgroup of 8 wavefronts per compute unit while the grid fits in one round; beyond
    // that, workgroups of 4 so that two are resident per unit and one's epilogue overlaps the
    // other's stream.  Never more wavefronts than k tiles.
    static int cus = 0;   // compute units of the current device, asked once
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            cus = v;
        else
            cus = 256;
    }
    int n_waves = grid <= (unsigned)cus ? 8 : 4;
    while (n_waves > 1 && n_waves > args.KT) n_waves >>= 1;
    if (n_jobs <= 4) return launch_nj<4>(args, n_waves, grid, st);
    if (n_jobs <= 8) return launch_nj<8>(args, n_waves, grid, st);
    return launch_nj<16>(args, n_waves, grid, st);
}

}  // namespace bd
