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

__global__ __launch_bounds__(256, 2) void linear_prefill_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, const int32_t* __restrict__ row_token, const int32_t* __restrict__ tile_tenant,
    uint16_t* __restrict__ y, const int64_t out, const int64_t in, const int n_mtiles, const int n_ntiles) {
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
    const uint32_t* __restrict__ packed = packed_by_tenant[tenant];
    const float alpha = alpha_by_tenant[tenant];
    const int64_t words_per_row = in >> 5;

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
        wsrc[i] = (const unsigned char*)(w + wrow * in) + c8 * 16;
        soff_lds[i] = pf_off(row, c8);
        kofs[i] = c8 * 8;
    }
    const int64_t srow = n0 + (tid & 127) < out ? n0 + (tid & 127) : out - 1;
    const uint32_t* ssrc = packed + srow * words_per_row;

    u32x4 xg[kPfPerThread], wg[kPfPerThread];
    uint32_t sw[kPrefillK / 32];
    // elements beyond `in` (second half of the last step when in % 64 == 32) are fetched as zeros
    auto fetch = [&](const int64_t k0) {
#pragma unroll
        for (int i = 0; i < kPfPerThread; ++i) {
            const bool kin = k0 + kofs[i] < in;
            xg[i] = wg[i] = u32x4{0u, 0u, 0u, 0u};
            if (xok[i] && kin) xg[i] = *(const u32x4*)(xsrc[i] + k0 * 2);
            if (kin) wg[i] = *(const u32x4*)(wsrc[i] + k0 * 2);
        }
        if (tid < 128) {
#pragma unroll
            for (int h = 0; h < kPrefillK / 32; ++h) sw[h] = (k0 >> 5) + h < words_per_row ? ssrc[(k0 >> 5) + h] : 0u;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < kPfPerThread; ++i) {
            *(u32x4*)(xs + soff_lds[i]) = xg[i];
            *(u32x4*)(ws + soff_lds[i]) = wg[i];
        }
        if (tid < 128) {
#pragma unroll
            for (int h = 0; h < kPrefillK / 32; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                {
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
        stage();
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
                if (n < out) y[(int64_t)tok * out + n] = f2h_rne(accb[i][j][q] + alpha * accd[i][j][q]);
            }
        }
    }
}

hipError_t launch_prefill_meta(const PrefillMetaChunk& chunk, int32_t* dst, int n, hipStream_t st) {
    hipLaunchKernelGGL(prefill_meta_kernel, dim3(1), dim3(256), 0, st, chunk, dst, n);
    return hipGetLastError();
}

hipError_t launch_linear_prefill(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                 const float* alpha_by_tenant, const int32_t* row_token, const int32_t* tile_tenant,
                                 int n_mtiles, uint16_t* y, int64_t out, int64_t in, hipStream_t st) {
    const int n_ntiles = (int)((out + kPrefillTile - 1) / kPrefillTile);
    const int64_t tiles = (int64_t)n_mtiles * n_ntiles;
    if (tiles < 1 || tiles > (int64_t)1 << 30) return hipErrorInvalidValue;
    const int64_t round = (int64_t)kPfChunk * kPfXcds;                      // one chunk for every XCD
    const unsigned grid = (unsigned)((tiles + round - 1) / round * round);   // surplus workgroups return at once
    hipLaunchKernelGGL(linear_prefill_kernel, dim3(grid), dim3(256), 0, st, x, w, packed_by_tenant, alpha_by_tenant,
                       row_token, tile_tenant, y, out, in, n_mtiles, n_ntiles);
    return hipGetLastError();
}

}  // namespace bd
