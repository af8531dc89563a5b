// Prefill form of the multi-tenant linear (Eq. 6 of the paper; the batched W_INT1 A_FP16 product
// of Sec. 4.3 when every tenant brings many tokens):
//     y[t, n] = sum_k x[t,k] W_base[n,k]  +  alpha_e * sum_k x[t,k] s_e[n,k],   e = tenant(t).
//
// With hundreds of tokens per tenant both products are dense contractions, so this is a tiled
// matrix-core GEMM.  Tokens are sorted by tenant on the host and cut into M tiles of 128 rows
// that never mix tenants (the last tile of a tenant is padded with empty rows).  A workgroup
// (4 wavefronts, 2 x 2) owns one 128 x 128 tile of y and walks k in steps of 64 (32 for the last step of in % 64 == 32):
//   x tile   128 tokens x 64 k   fp16, gathered through the token permutation
//   W tile   128 rows   x 64 k   fp16
//   s tile   128 rows   x 64 k   two packed words per row, expanded to +-1.0 fp16 on the way into
//                                LDS: a nibble of signs -> 4 fp16 through a 16-entry table kept in 32
//                                copies (4 KB), lane l reading copy l % 32, so that the look-ups of
//                                the lanes served together never share a bank
// and every wavefront accumulates its 64 x 64 corner twice with v_mfma_f32_16x16x32_f16: x.W^T
// and x.s^T in separate binary32 accumulators, combined as acc_b + alpha * acc_d at the end (alpha
// multiplies the finished +-1 sum, as in the decode kernels).  Global loads of step k+1 are in
// registers while step k is multiplied.  An LDS row holds the 8 16-byte chunks of its 64 k in the order
// chunk ^ ((row / 2) % 8): the 16 lanes that LDS serves together then touch all 64 banks once, both when
// they write one chunk of 16 consecutive rows or 8 chunks of 2 rows (staging) and when they read one chunk
// of 16 consecutive rows (operands).
//
// PLANES (Sec. 4.2 of the paper, fidelity of the delta: k sign planes per tenant with scales alpha_j): the sign tile
// then holds d[n,k] = sum_j alpha_j s_j[n,k], added up in fp16 in ascending j while the signs are expanded (s_j = +-1,
// so alpha_j s_j is exact and every addition rounds once), and the combine is acc_b + acc_d.  The one rounding of d to
// fp16 per weight is what a materialised fine-tuned weight would carry too; it is 2^-11 of the delta term.
// Q8 (Sec. 4.2, quantized base models): W is the row-major int8 q of the 8-bit base; a byte u = q + 128 next to the
// constant 0x64 is the fp16 number 1024 + u, minus 1152 gives q exactly, the base accumulator holds sum_k x q and
// the row's scale multiplies the finished sum.
#include "bd_device.h"
#include "bd_launch.h"

namespace bd {

namespace {

constexpr int kPfRowBytes = kPrefillK * 2;                 // 128
constexpr int kPfTileBytes = kPrefillTile * kPfRowBytes;   // 16384
static_assert(kPrefillK == 64, "the chunk swizzle assumes 8 chunks per row");

__device__ __forceinline__ int pf_off(const int row, const int chunk) {
    return row * kPfRowBytes + ((chunk ^ ((row >> 1) & 7)) << 4);
}
constexpr int kPfChunks = kPrefillK / 8;                   // 16-byte chunks per tile row
constexpr int kPfPerThread = kPrefillTile * kPfChunks / 256;
constexpr int kPfLutBytes = 16 * 32 * 8;                   // [nibble][copy] of 4 fp16
constexpr int kPfPanel = 8;                                // N tiles per column panel of the launch order
constexpr int kPfChunk = 64;                               // consecutive tiles one XCD works on together (32 CUs x 2 workgroups)
constexpr int kPfXcds = 8;

}  // namespace

// Copies up to 960 ints that arrive in the kernel arguments to device memory: the token
// permutation reaches the GPU without a host-to-device copy call (asynchronous, capturable).
__global__ __launch_bounds__(256) void prefill_meta_kernel(const PrefillMetaChunk c, int32_t* __restrict__ dst, const int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) dst[i] = c.v[i];
}

// The same tables written from runs: triple r = (first index, first value, n) stands for n values first, first + 1, ...
// (n > 0) or -n copies of the value (n < 0).  A batch whose tokens arrive grouped by tenant is a handful of runs.
__global__ __launch_bounds__(256) void prefill_meta_runs_kernel(const PrefillMetaChunk c, int32_t* __restrict__ dst, const int n_runs) {
    for (int r = 0; r < n_runs; ++r) {
        const int first = c.v[3 * r], value = c.v[3 * r + 1], n = c.v[3 * r + 2];
        const int count = n < 0 ? -n : n;
        for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < count; i += gridDim.x * blockDim.x)
            dst[first + i] = n > 0 ? value + i : value;
    }
}

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
constexpr int kPfMaxPlanes = 8;

template <bool PLANES, bool Q8>
__global__ __launch_bounds__(256, 2) void linear_prefill_kernel(
    const uint16_t* __restrict__ x, const void* __restrict__ w_any, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, const float* __restrict__ wscale, const int32_t* __restrict__ row_token,
    const int32_t* __restrict__ tile_tenant, uint16_t* __restrict__ y, const int64_t out, const int64_t in,
    const int n_mtiles, const int n_ntiles, const int k_planes) {
    __shared__ __align__(16) unsigned char lds[3 * kPfTileBytes + kPfLutBytes];
    unsigned char* const xs = lds;
    unsigned char* const ws = lds + kPfTileBytes;
    unsigned char* const ss = lds + 2 * kPfTileBytes;
    unsigned char* const lut = lds + 3 * kPfTileBytes;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 15, g = lane >> 4;
    // Launch order -> tile.  Workgroup ids go round-robin over the 8 XCDs, each with an L2 of its own; the
    // workgroups an XCD runs together (ids L, L+8, ...) should form a compact block of tiles so that every x
    // and W slice it fetches serves 8 of them.  Tiles are numbered panel by panel (8 N tiles wide, row-major
    // inside), cut into chunks of 64 = 8 x 8 tiles, and chunk c goes to XCD c % 8.
    int mt, nt;
    {
        const int L = blockIdx.x, xcd = L % kPfXcds, slot = L / kPfXcds;
        const int chunk = (slot / kPfChunk) * kPfXcds + xcd;
        const int t = chunk * kPfChunk + slot % kPfChunk;
        if (t >= n_mtiles * n_ntiles) return;   // the grid is padded to whole rounds of chunks
        const int per_panel = n_mtiles * kPfPanel;
        const int panel = t / per_panel, tp = t - panel * per_panel;
        const int width = n_ntiles - panel * kPfPanel < kPfPanel ? n_ntiles - panel * kPfPanel : kPfPanel;
        mt = tp / width;
        nt = panel * kPfPanel + tp % width;
    }
    const int64_t n0 = (int64_t)nt * kPrefillTile;
    const int tenant = tile_tenant[mt];
    constexpr int NP = PLANES ? kPfMaxPlanes : 1;
    const int np = PLANES ? k_planes : 1;
    const float alpha = PLANES ? 1.f : alpha_by_tenant[tenant];
    const int64_t words_per_row = in >> 5;
    constexpr int kWBytes = Q8 ? 1 : 2;   // bytes per base weight
    const unsigned char* const w = (const unsigned char*)w_any;

    // nibble -> 4 fp16 (+1.0 where the bit is set, else -1.0), element e = bit e; entry [nibble][copy]
    {
        const uint32_t b = (uint32_t)tid >> 4;
        uint2 e;
        e.x = 0xBC00BC00u ^ ((b & 1u) << 15) ^ (((b >> 1) & 1u) << 31);
        e.y = 0xBC00BC00u ^ (((b >> 2) & 1u) << 15) ^ (((b >> 3) & 1u) << 31);
        *(uint2*)(lut + b * 256 + (tid & 15) * 8) = e;
        *(uint2*)(lut + b * 256 + 128 + (tid & 15) * 8) = e;
    }
    const uint32_t lut_lane = (uint32_t)(tid & 31) * 8u;

    // what this thread fetches per step: four 16-byte chunks of x, four of W, (threads < 128) the sign words of one row
    const unsigned char* xsrc[kPfPerThread];
    const unsigned char* wsrc[kPfPerThread];
    bool xok[kPfPerThread];
    int soff_lds[kPfPerThread], kofs[kPfPerThread];
#pragma unroll
    for (int i = 0; i < kPfPerThread; ++i) {
        const int q = tid + 256 * i, row = q / kPfChunks, c8 = q % kPfChunks;
        const int tok = row_token[mt * kPrefillTile + row];
        xok[i] = tok >= 0;
        xsrc[i] = (const unsigned char*)(x + (int64_t)(tok >= 0 ? tok : 0) * in) + c8 * 16;
        const int64_t wrow = n0 + row < out ? n0 + row : out - 1;   // rows beyond out repeat the last row; never stored
        wsrc[i] = w + wrow * in * kWBytes + c8 * 8 * kWBytes;
        soff_lds[i] = pf_off(row, c8);
        kofs[i] = c8 * 8;
    }
    const int64_t srow = n0 + (tid & 127) < out ? n0 + (tid & 127) : out - 1;
    // the planes' pointers and scales are the same for the whole workgroup (scalars); the row's offset is the lane's
    const uint32_t* ssrc[NP];
    uint32_t alpha2[NP];   // PLANES: the bits of (alpha_j, alpha_j) in fp16 -- the scales are fp16 numbers carried as float
    const int64_t srow_off = srow * words_per_row;
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const int jj = j < np ? j : 0;
        ssrc[j] = packed_by_tenant[PLANES ? tenant * np + jj : tenant];
        const _Float16 a = PLANES ? (_Float16)alpha_by_tenant[tenant * np + jj] : (_Float16)1.f;
        alpha2[j] = __builtin_amdgcn_readfirstlane(__builtin_bit_cast(uint32_t, half2v{a, a}));   // a scalar register
    }

    u32x4 xg[kPfPerThread], wg[kPfPerThread];   // Q8: a chunk of W is 8 bytes, in wg[i][0..1]
    uint32_t sw[kPrefillK / 32];   // one plane: the row's words of the next step; several planes are fetched when they are staged
    // elements beyond `in` (second half of the last step when in % 64 == 32) are fetched as zeros
    auto fetch = [&](const int64_t k0) {
#pragma unroll
        for (int i = 0; i < kPfPerThread; ++i) {
            const bool kin = k0 + kofs[i] < in;
            xg[i] = wg[i] = u32x4{0u, 0u, 0u, 0u};
            if (xok[i] && kin) xg[i] = *(const u32x4*)(xsrc[i] + k0 * 2);
            if (kin) {
                if constexpr (Q8) {
                    const u32x2 b = *(const u32x2*)(wsrc[i] + k0);
                    wg[i][0] = b[0];
                    wg[i][1] = b[1];
                } else {
                    wg[i] = *(const u32x4*)(wsrc[i] + k0 * 2);
                }
            }
        }
        if constexpr (!PLANES) {
            if (tid < 128) {
#pragma unroll
                for (int h = 0; h < kPrefillK / 32; ++h)
                    sw[h] = (k0 >> 5) + h < words_per_row ? ssrc[0][srow_off + (k0 >> 5) + h] : 0u;
            }
        }
    };
    // 4 bytes q (two's complement) -> 4 fp16 numbers q
    auto q8_pair = [](const uint32_t b4, const uint32_t sel) {
        const uint32_t u = __builtin_amdgcn_perm(0x64646464u, b4 ^ 0x80808080u, sel);   // two fp16: 1024 + (q + 128)
        const half2v v = __builtin_bit_cast(half2v, u) - half2v{(_Float16)1152.f, (_Float16)1152.f};
        return __builtin_bit_cast(uint32_t, v);
    };
    auto stage = [&](const int64_t k0) {
#pragma unroll
        for (int i = 0; i < kPfPerThread; ++i) {
            *(u32x4*)(xs + soff_lds[i]) = xg[i];
            if constexpr (Q8) {
                // (a chunk fetched as zeros, beyond `in`, comes out as zeros: 1024 + 128 - 1152)
                *(u32x4*)(ws + soff_lds[i]) = u32x4{q8_pair(wg[i][0], 0x04010400u), q8_pair(wg[i][0], 0x04030402u),
                                                     q8_pair(wg[i][1], 0x04010400u), q8_pair(wg[i][1], 0x04030402u)};
            } else {
                *(u32x4*)(ws + soff_lds[i]) = wg[i];
            }
        }
        if constexpr (PLANES) {
            const int h = tid >> 7, row = tid & 127;
            // +-alpha_j = alpha_j's magnitude bits under the table entry's sign bits (alpha_j >= 0): one v_bfi_b32 per pair
            auto signed_alpha = [](const uint32_t entry, const uint32_t a) {
                return __builtin_bit_cast(half2v, (a & 0x7FFF7FFFu) | (entry & 0x80008000u));
            };
            // every thread one word per plane (row tid % 128, word tid / 128 of the step), fetched here: the registers
            // of a prefetch for eight planes are not there
            const int64_t wi = (k0 >> 5) + h;
            uint32_t pw[NP];
#pragma unroll
            for (int j = 0; j < NP; ++j) pw[j] = (j < np && wi < words_per_row) ? ssrc[j][srow_off + wi] : 0u;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                half2v d[4];
#pragma unroll
                for (int j = 0; j < NP; ++j)
                    if (j < np) {
                        const uint32_t byte = (pw[j] >> (8 * q)) & 0xFFu;
                        const uint2 lo = *(const uint2*)(lut + (byte & 15u) * 256u + lut_lane);
                        const uint2 hi = *(const uint2*)(lut + (byte >> 4) * 256u + lut_lane);
                        const half2v t0 = signed_alpha(lo.x, alpha2[j]), t1 = signed_alpha(lo.y, alpha2[j]);
                        const half2v t2 = signed_alpha(hi.x, alpha2[j]), t3 = signed_alpha(hi.y, alpha2[j]);
                        d[0] = j == 0 ? t0 : d[0] + t0;
                        d[1] = j == 0 ? t1 : d[1] + t1;
                        d[2] = j == 0 ? t2 : d[2] + t2;
                        d[3] = j == 0 ? t3 : d[3] + t3;
                    }
                *(u32x4*)(ss + pf_off(row, 4 * h + q)) =
                    u32x4{__builtin_bit_cast(uint32_t, d[0]), __builtin_bit_cast(uint32_t, d[1]),
                          __builtin_bit_cast(uint32_t, d[2]), __builtin_bit_cast(uint32_t, d[3])};
            }
        } else if (tid < 128) {
#pragma unroll
            for (int h = 0; h < kPrefillK / 32; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t byte = (sw[h] >> (8 * q)) & 0xFFu;
                    const uint2 lo = *(const uint2*)(lut + (byte & 15u) * 256u + lut_lane);
                    const uint2 hi = *(const uint2*)(lut + (byte >> 4) * 256u + lut_lane);
                    *(u32x4*)(ss + pf_off(tid, 4 * h + q)) = u32x4{lo.x, lo.y, hi.x, hi.y};
                }
        }
    };

    float4v accb[4][4], accd[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) accb[i][j] = accd[i][j] = float4v{0.f, 0.f, 0.f, 0.f};

    fetch(0);
    __syncthreads();   // the table is complete
    for (int64_t k0 = 0; k0 < in; k0 += kPrefillK) {
        stage(k0);
        __syncthreads();
        if (k0 + kPrefillK < in) fetch(k0 + kPrefillK);
#pragma unroll
        for (int h = 0; h < kPrefillK / 32; ++h) {
            half8 a[4], bw[4], bs[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = *(const half8*)(xs + pf_off(wm * 64 + i * 16 + r, 4 * h + g));
                bw[i] = *(const half8*)(ws + pf_off(wn * 64 + i * 16 + r, 4 * h + g));
                bs[i] = *(const half8*)(ss + pf_off(wn * 64 + i * 16 + r, 4 * h + g));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    accb[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], bw[j], accb[i][j], 0, 0, 0);
                    accd[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], bs[j], accd[i][j], 0, 0, 0);
                }
        }
        __syncthreads();   // everybody is done reading this step's tiles
    }

    // D[row 4 g + q][col r] of sub-tile (i, j): token row wm*64 + 16 i + 4 g + q, output feature n0 + wn*64 + 16 j + r
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int tok = row_token[mt * kPrefillTile + wm * 64 + i * 16 + 4 * g + q];
            if (tok < 0) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t n = n0 + wn * 64 + j * 16 + r;
                if (n < out) {
                    const float base = Q8 ? wscale[n] * accb[i][j][q] : accb[i][j][q];
                    y[(int64_t)tok * out + n] = f2h_rne(base + alpha * accd[i][j][q]);
                }
            }
        }
    }
}

hipError_t launch_prefill_meta(const PrefillMetaChunk& chunk, int32_t* dst, int n, hipStream_t st) {
    hipLaunchKernelGGL(prefill_meta_kernel, dim3(1), dim3(256), 0, st, chunk, dst, n);
    return hipGetLastError();
}

hipError_t launch_prefill_meta_runs(const PrefillMetaChunk& chunk, int32_t* dst, int n_runs, hipStream_t st) {
    hipLaunchKernelGGL(prefill_meta_runs_kernel, dim3(8), dim3(256), 0, st, chunk, dst, n_runs);
    return hipGetLastError();
}

// k_planes = 0: one plane per tenant, tables indexed by tenant; k_planes >= 1: tables indexed by tenant * k_planes + plane.
// wscale != nullptr: w is the row-major int8 base and wscale its per-row scales.
hipError_t launch_linear_prefill(const uint16_t* x, const void* w, const uint32_t* const* packed_by_tenant,
                                 const float* alpha_by_tenant, const float* wscale, const int32_t* row_token,
                                 const int32_t* tile_tenant, int n_mtiles, uint16_t* y, int64_t out, int64_t in,
                                 int k_planes, hipStream_t st) {
    const int n_ntiles = (int)((out + kPrefillTile - 1) / kPrefillTile);
    const int64_t tiles = (int64_t)n_mtiles * n_ntiles;
    if (tiles < 1 || tiles > (int64_t)1 << 30 || k_planes < 0 || k_planes > kPfMaxPlanes) return hipErrorInvalidValue;
    const int64_t round = (int64_t)kPfChunk * kPfXcds;                      // one chunk for every XCD
    const unsigned grid = (unsigned)((tiles + round - 1) / round * round);   // surplus workgroups return at once
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, st, x, w, packed_by_tenant, alpha_by_tenant, wscale, row_token,
                           tile_tenant, y, out, in, n_mtiles, n_ntiles, k_planes);
        return hipGetLastError();
    };
    if (k_planes > 0) return wscale ? go(linear_prefill_kernel<true, true>) : go(linear_prefill_kernel<true, false>);
    return wscale ? go(linear_prefill_kernel<false, true>) : go(linear_prefill_kernel<false, false>);
}

}  // namespace bd
