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
//   x      staged once per step and wavefront in LDS (direct global->LDS loads), read back in either order.
// A delta "job" is one tenant's run of columns in a tile; its MFMA result is only valid in
// those columns, which are selected once per pass.  Jobs are processed in passes of 8/4/2/1 so
// that every pass is straight-line code.  Partial sums of the wavefronts are added in a fixed
// order through LDS, so results are deterministic and y is written exactly once.
#include <type_traits>

#include "bd_device.h"
#include "bd_launch.h"
#include "bd_mfma.h"

namespace bd {

#ifdef BD_EXPERIMENT_STAMPS
// experiment only: shader-clock stamps of the first workgroups' wavefronts
__device__ unsigned long long bd_stamps[64 * 8 * 16];
#define BD_STAMP(i)                                                                                   \
    do {                                                                                              \
        if (blockIdx.x < 64 && (threadIdx.x & 63) == 0)                                               \
            bd_stamps[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 16 + (i)] = __builtin_readcyclecounter(); \
    } while (0)
#else
#define BD_STAMP(i) do { } while (0)
#endif

struct LaneCtx {
    const uint16_t* x;
    const uint16_t* w;
    const uint32_t* const* packed_by_tenant;
    int in;                                // reduction length (below 2^31)
    uint32_t woff;                         // byte offset of W[row][8 g]
    uint32_t soff;                         // byte offset of packed[row][4 g]
    uint32_t xoff;                         // byte offset 16 * lane inside a 512-element chunk of x
    unsigned char* xs;                     // this wavefront's LDS region: [16 columns][kXsRowBytes]
    const unsigned char* xs_base_rd;       // + 64 v
    const unsigned char* xs_delta_rd;      // + 64 u + 8 m (+32)
    int lane, g, wave, n_waves, n_steps;
};

// x of one column tile, 512 reduction elements from k0 -> this wavefront's LDS region, by
// direct global->LDS loads (no registers; lane l's 16 bytes land at row + 16 l).  Rows of
// columns beyond T are never written and stay zero from the start of the kernel; elements
// beyond `in` are written as zeros, so whatever the weight registers hold there multiplies 0.
template <bool FULL>
__device__ __forceinline__ void stage_x(const LaneCtx& cx, const DecodeMeta& meta, int tile, int k0, uint32_t xoff) {
    const bool kvalid = FULL || (k0 + (int)(xoff >> 1) < cx.in);
#pragma unroll
    for (int c = 0; c < 16; ++c) {
        const int col = tile * 16 + c;
        if (col < meta.T) {
            const unsigned char* colbase = (const unsigned char*)(cx.x + (int64_t)meta.token_of_col[col] * cx.in + k0);
            unsigned char* row = cx.xs + c * kXsRowBytes;
            if constexpr (FULL) {
                __builtin_amdgcn_global_load_lds((gptr_t)(colbase + xoff), (lptr_t)row, 16, 0, 0);
            } else {
                if (kvalid) __builtin_amdgcn_global_load_lds((gptr_t)(colbase + xoff), (lptr_t)row, 16, 0, 0);
                else *(u32x4*)(row + xoff) = u32x4{0u, 0u, 0u, 0u};
            }
        }
    }
}

// The JG delta jobs in slots [slot0, slot0 + JG) of a tile, one step: expand their sign words and
// multiply them with the staged x.  Padding slots re-read the first job's words and are never
// selected.  On return `sel` holds, per lane, the partial sum of the job
// that owns the lane's column (unchanged if none of these jobs does).
// The B operand (x) of delta slice (u, m): elements (4m+q, 4m+q+16), q = 0..3, of word u of
// this lane's 128-element block, as four fp16 pairs.
struct DeltaB {
    u32x2 lo, hi;
    __device__ __forceinline__ void read(const LaneCtx& cx, int u, int m) {
        lo = *(const u32x2*)(cx.xs_delta_rd + u * 64 + m * 8);
        hi = *(const u32x2*)(cx.xs_delta_rd + u * 64 + m * 8 + 32);
    }
    __device__ __forceinline__ half8 operand() const {
        return as_half8(__builtin_amdgcn_perm(hi[0], lo[0], 0x05040100u), __builtin_amdgcn_perm(hi[0], lo[0], 0x07060302u),
                        __builtin_amdgcn_perm(hi[1], lo[1], 0x05040100u), __builtin_amdgcn_perm(hi[1], lo[1], 0x07060302u));
    }
};

template <int JG, int MODE>
__device__ __forceinline__ void delta_group(const LaneCtx& cx, const DecodeMeta& meta, const ExpandConsts<MODE>& kc,
                                            int tile, int slot0, int c, const u32x4 (&sreg)[JG], float4v& sel) {
    float4v acc[JG];
#pragma unroll
    for (int j = 0; j < JG; ++j) acc[j] = float4v{0.f, 0.f, 0.f, 0.f};
    DeltaB nxt;
    nxt.read(cx, 0, 0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        WordState<MODE> ws[JG];
#pragma unroll
        for (int j = 0; j < JG; ++j) ws[j].set(sreg[j][u]);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const half8 bd = nxt.operand();
            if (u * 4 + m + 1 < 16) nxt.read(cx, (u * 4 + m + 1) >> 2, (u * 4 + m + 1) & 3);   // LDS latency hides under this slice
#pragma unroll
            for (int j = 0; j < JG; ++j) {
                const half8 a = as_half8(ws[j].reg(4 * m, kc), ws[j].reg(4 * m + 1, kc), ws[j].reg(4 * m + 2, kc),
                                         ws[j].reg(4 * m + 3, kc));
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bd, acc[j], 0, 0, 0);
            }
            // Issue order inside the slice: the expansion of job j+1 (4 and-or) goes between the
            // MFMAs of jobs j and j+1, so the vector ALU and the matrix pipe run at the same time
            // even with a single wavefront on the SIMD.
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // next slice's LDS reads
            __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);   // perms + expansion of job 0
#pragma unroll
            for (int j = 0; j + 1 < JG; ++j) {
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);   // expansion of job j+1 ...
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // ... ahead of the MFMA of job j
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_barrier(0);   // keep the expansion of one slice next to its MFMAs
        }
    }
#pragma unroll
    for (int j = 0; j < JG; ++j) {
        const bool mine = (c >= meta.slot_col_begin[tile][slot0 + j]) & (c < meta.slot_col_end[tile][slot0 + j]);
#pragma unroll
        for (int i = 0; i < 4; ++i) sel[i] = mine ? acc[j][i] : sel[i];
    }
}

// H = sum_k (2^(11-p(k)) + 1) x_k of one step (mantissa mode only): the same four B operands
// per word as the delta product, against a constant A operand.
__device__ __forceinline__ void h_term(const LaneCtx& cx, const ExpandConsts<kMantissa>& kc, float4v& acch) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        DeltaB b[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) b[m].read(cx, u, m);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int pb = (m & 1) * 4;
            const half8 hop = as_half8(kc.hreg[pb], kc.hreg[pb + 1], kc.hreg[pb + 2], kc.hreg[pb + 3]);
            acch = __builtin_amdgcn_mfma_f32_16x16x32_f16(hop, b[m].operand(), acch, 0, 0, 0);
        }
    }
}

// NG groups of JG job slots per column tile: (1,4) up to 4 jobs, (1,8) up to 8, (2,8) up to 16.
template <int MODE, int TILES, int NG, int JG>
__global__ __launch_bounds__(kMaxWaves * kWave) void linear_decode_mfma_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
    const uint32_t* const* __restrict__ packed_by_tenant, const float* __restrict__ alpha_by_tenant,
    const DecodeMeta meta, uint16_t* __restrict__ y, const int64_t out, const int64_t in64) {
    const int in = (int)in64;
    extern __shared__ __align__(16) unsigned char smem[];
    LaneCtx cx;
    const int lane = threadIdx.x & (kWave - 1);
    cx.lane = lane;
    BD_STAMP(0);
    cx.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, and the compiler knows it
    cx.n_waves = blockDim.x >> 6;
    const int c = lane & 15;          // A row (output row) for loads, B/D column (token) for MFMA results
    cx.g = lane >> 4;
    cx.xs = smem + cx.wave * kXsWaveBytes;
    const int64_t n0 = (int64_t)blockIdx.x * 16;
    const int64_t nrow = (n0 + c < out) ? n0 + c : out - 1;   // clamp: padded rows repeat the last row
    cx.n_steps = (int)((in + kStepK - 1) / kStepK);
    cx.in = in;
    cx.x = x;
    cx.w = w;
    cx.packed_by_tenant = packed_by_tenant;
    cx.woff = (uint32_t)((nrow * in64 + 8 * cx.g) * 2);
    cx.soff = (uint32_t)((nrow * (in64 >> 5) + 4 * cx.g) * 4);
    cx.xoff = (uint32_t)(16 * lane);
    cx.xs_base_rd = cx.xs + c * kXsRowBytes + cx.g * 16;
    cx.xs_delta_rd = cx.xs + c * kXsRowBytes + cx.g * 256;
    const ExpandConsts<MODE> kc;

    // zero this wavefront's staging rows once: rows of absent columns are never written again
#pragma unroll
    for (int i = 0; i < kXsWaveBytes / (kWave * 16); ++i) *(u32x4*)(cx.xs + (i * kWave + lane) * 16) = u32x4{0u, 0u, 0u, 0u};
    if (lane < (kXsWaveBytes % (kWave * 16)) / 16)
        *(u32x4*)(cx.xs + ((kXsWaveBytes / (kWave * 16)) * kWave + lane) * 16) = u32x4{0u, 0u, 0u, 0u};

    // per tile: the packed-delta pointer of every job slot and this lane's scale = alpha of the
    // tenant owning its column.  The slot tenants arrive with the kernel arguments (fixed slots,
    // constant indices).  Lane j of `slot_ptr_*` fetches the pointer of slot j with ONE vector load
    // (sixteen dependent scalar loads would serialise for microseconds); the step loop reads the
    // lanes back as uniform values.  The alpha load is issued here and first used in the epilogue.
    int n_jobs_tile[TILES];
    uint32_t slot_ptr_lo[TILES], slot_ptr_hi[TILES];
    float alpha_c[TILES];
#pragma unroll
    for (int tile = 0; tile < TILES; ++tile) {
        n_jobs_tile[tile] = meta.tile_job_end[tile] - meta.tile_job_begin[tile];
        int my_tenant = 0, lane_tenant = 0;
#pragma unroll
        for (int j = 0; j < NG * JG; ++j) {
            const int t = meta.slot_tenant[tile][j];
            lane_tenant = (lane == j) ? t : lane_tenant;
            const bool mine = (c >= meta.slot_col_begin[tile][j]) & (c < meta.slot_col_end[tile][j]);
            my_tenant = mine ? t : my_tenant;
        }
        const uint64_t p = (uint64_t)packed_by_tenant[lane_tenant];   // lanes >= NG*JG fetch slot-0-like tenant 0: valid, unused
        slot_ptr_lo[tile] = (uint32_t)p;
        slot_ptr_hi[tile] = (uint32_t)(p >> 32);
        alpha_c[tile] = (tile * 16 + c < meta.T) ? alpha_by_tenant[my_tenant] : 0.f;
    }

    BD_STAMP(9);
    float4v accb[TILES], acch[TILES], dsel[TILES];
#pragma unroll
    for (int tile = 0; tile < TILES; ++tile) accb[tile] = acch[tile] = dsel[tile] = float4v{0.f, 0.f, 0.f, 0.f};

    // One step of this wavefront: 512 reduction elements from k0.  FULL steps carry no guards at
    // all; the (at most one) ragged last step of the matrix takes the guarded instantiation.
    auto do_step = [&](auto full_tag, const int k0) {
        constexpr bool FULL = decltype(full_tag)::value;
        // Lane offsets are re-read through an empty asm every step: otherwise the compiler hoists
        // "uniform base + lane offset" of every load out of the loop as 64-bit register pairs.
        uint32_t woff = cx.woff, soff = cx.soff, xoff = cx.xoff;
        asm volatile("" : "+v"(woff), "+v"(soff), "+v"(xoff));
        const bool svalid = FULL || (k0 + 128 * cx.g < in);

        // ---- issue order = arrival order: x (L2 hits, straight into LDS), the sign words (their
        // expansion is the bulk of the work), W last (its 16 MFMAs per tile are the short tail)
        lds_wave_sync();                         // the previous step's LDS reads are done
        BD_STAMP(10);
        stage_x<FULL>(cx, meta, 0, k0, xoff);
        __builtin_amdgcn_sched_barrier(0);
        BD_STAMP(11);
        u32x4 sreg[NG][JG];
        auto load_signs = [&](const int tile) {
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
#pragma unroll
                for (int j = 0; j < JG; ++j) {
                    const uint64_t pj = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)slot_ptr_lo[tile], gi * JG + j) |
                                        ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)slot_ptr_hi[tile], gi * JG + j) << 32);
                    const uint32_t* sp = (const uint32_t*)pj + (k0 >> 5);
                    if constexpr (FULL) {
                        sreg[gi][j] = load16_stream(sp, soff);
                    } else {
                        sreg[gi][j] = u32x4{0u, 0u, 0u, 0u};
                        if (svalid) sreg[gi][j] = load16_stream(sp, soff);
                    }
                }
            }
        };
        load_signs(0);
        BD_STAMP(12);
        u32x4 wreg[16];
        {
            const uint16_t* wk = w + k0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                if constexpr (FULL) {
                    wreg[v] = load16_stream(wk + 32 * v, woff);
                } else {
                    wreg[v] = u32x4{0u, 0u, 0u, 0u};
                    if (k0 + 32 * v < in) wreg[v] = load16_stream(wk + 32 * v, woff);
                }
            }
        }
        BD_STAMP(1);
        __builtin_amdgcn_sched_barrier(0);
        // The direct-to-LDS loads are older than the NG*JG + 16 register loads above and memory
        // loads return in order: "at most that many outstanding" means x has landed.  (The guarded
        // instantiation may have skipped loads, so it waits for everything.)
        if constexpr (FULL) __builtin_amdgcn_s_waitcnt(vmcnt_only(NG * JG + 16));
        else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
#pragma unroll
        for (int tile = 0; tile < TILES; ++tile) {
            if (tile > 0) {
                // second column tile: new sign words, and its x over the same LDS rows
                lds_wave_sync();
                stage_x<FULL>(cx, meta, tile, k0, xoff);
                __builtin_amdgcn_sched_barrier(0);
                load_signs(tile);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (FULL) __builtin_amdgcn_s_waitcnt(vmcnt_only(NG * JG));
                else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
            }
            lds_wave_sync();
            BD_STAMP(2);
            if constexpr (MODE == kMantissa) {
                h_term(cx, kc, acch[tile]);
                __builtin_amdgcn_sched_barrier(0);
            }
            BD_STAMP(3);
            // ---- delta jobs, one group of JG at a time; keep the job owning this lane's column
            float4v sel = {0.f, 0.f, 0.f, 0.f};
#ifdef BD_EXPERIMENT_NO_DELTA_MATH
            {   // experiment only: consume the sign words without expanding them
                uint32_t fold = 0;
#pragma unroll
                for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                    for (int j = 0; j < JG; ++j) fold ^= sreg[gi][j][0] ^ sreg[gi][j][1] ^ sreg[gi][j][2] ^ sreg[gi][j][3];
                sel[0] = (fold == 0x12345u) ? 1.f : 0.f;
            }
#else
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
                if (gi == 0 || gi * JG < n_jobs_tile[tile])
                    delta_group<JG, MODE>(cx, meta, kc, tile, gi * JG, c, sreg[gi], sel);
            }
#endif
            dsel[tile] += sel;
            BD_STAMP(4);
            // ---- base product of this tile, four B operands in flight
#pragma unroll
            for (int vb = 0; vb < 16; vb += 4) {
                half8 b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) b[i] = *(const half8*)(cx.xs_base_rd + (vb + i) * 64);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    accb[tile] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, wreg[vb + i]), b[i], accb[tile], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            BD_STAMP(5);
        }
    };
    const int n_full = in / kStepK;
    for (int step = cx.wave; step < n_full; step += cx.n_waves) do_step(std::true_type{}, step * kStepK);
    if (n_full < cx.n_steps && (n_full % cx.n_waves) == cx.wave) do_step(std::false_type{}, n_full * kStepK);

    // ---- add the wavefronts' partial tiles in a fixed order and write y once
    BD_STAMP(6);
    __syncthreads();   // every wavefront is done with its staging region
    BD_STAMP(7);
    float* red = (float*)cx.xs;   // [tile][col][row] of this wavefront
#pragma unroll
    for (int tile = 0; tile < TILES; ++tile) {
        float4v d = dsel[tile];
        if constexpr (MODE == kMantissa) d = 4.0f * dsel[tile] - acch[tile];
        *(float4v*)(red + tile * 256 + c * 16 + 4 * cx.g) = accb[tile] + alpha_c[tile] * d;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < TILES * 256; idx += blockDim.x) {
        const int tile = idx >> 8, col = (idx >> 4) & 15, row = idx & 15;
        const int gcol = tile * 16 + col;
        if (gcol < meta.T && n0 + row < out) {
            float s = 0.f;
            for (int wv = 0; wv < cx.n_waves; ++wv)
                s += *(const float*)(smem + wv * kXsWaveBytes + (tile * 256 + col * 16 + row) * 4);
            y[(int64_t)meta.token_of_col[gcol] * out + n0 + row] = f2h_rne(s);
        }
    }
    BD_STAMP(8);
}

#ifdef BD_EXPERIMENT_STAMPS
extern "C" int bd_debug_read_stamps(unsigned long long* host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(bd_stamps), sizeof(unsigned long long) * n);
}
#endif

bool decode_mfma_variant_known(int variant) { return variant == 2 || variant == 3; }

template <int MODE, int TILES, int NG, int JG>
static hipError_t launch_one(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                             const float* alpha_by_tenant, const DecodeMeta& meta, uint16_t* y, int64_t out, int64_t in,
                             hipStream_t st) {
    const int n_steps = (int)((in + kStepK - 1) / kStepK);
    const int n_waves = n_steps < kMaxWaves ? n_steps : kMaxWaves;
    const size_t lds = (size_t)n_waves * kXsWaveBytes;
    auto kernel = linear_decode_mfma_kernel<MODE, TILES, NG, JG>;
    static PerDeviceOnce lds_limit;   // one per instantiation
    const hipError_t ea = lds_limit.run([&] {
        return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxWaves * kXsWaveBytes);
    });
    if (ea != hipSuccess) return ea;
    hipLaunchKernelGGL(kernel, dim3((unsigned)((out + 15) / 16)), dim3(n_waves * kWave), lds, st, x, w,
                       packed_by_tenant, alpha_by_tenant, meta, y, out, in);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_mode(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                              const float* alpha_by_tenant, const DecodeMeta& meta, uint16_t* y, int64_t out, int64_t in,
                              hipStream_t st) {
    int max_jobs = 0, cur = 0;   // most jobs in one column tile
    for (int j = 0; j < meta.n_jobs; ++j) {
        cur = (j > 0 && meta.job_tile[j] == meta.job_tile[j - 1]) ? cur + 1 : 1;
        max_jobs = cur > max_jobs ? cur : max_jobs;
    }
#define BD_ARGS x, w, packed_by_tenant, alpha_by_tenant, meta, y, out, in, st
    if (meta.T <= 16) {
        if (max_jobs <= 4) return launch_one<MODE, 1, 1, 4>(BD_ARGS);
        if (max_jobs <= 8) return launch_one<MODE, 1, 1, 8>(BD_ARGS);
        return launch_one<MODE, 1, 2, 8>(BD_ARGS);
    }
    if (max_jobs <= 4) return launch_one<MODE, 2, 1, 4>(BD_ARGS);
    if (max_jobs <= 8) return launch_one<MODE, 2, 1, 8>(BD_ARGS);
    return launch_one<MODE, 2, 2, 8>(BD_ARGS);
#undef BD_ARGS
}

// variant 2 = plain +-1 expansion, variant 3 = mantissa expansion.
// Requires in % 128 == 0 and every tensor (W, x, each packed delta) below 4 GiB.
hipError_t launch_linear_decode_mfma(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                     const float* alpha_by_tenant, const DecodeMeta& meta, uint16_t* y, int64_t out,
                                     int64_t in, int variant, hipStream_t st) {
    switch (variant) {
        case 2: return launch_mode<kPlain>(x, w, packed_by_tenant, alpha_by_tenant, meta, y, out, in, st);
        case 3: return launch_mode<kMantissa>(x, w, packed_by_tenant, alpha_by_tenant, meta, y, out, in, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace bd
