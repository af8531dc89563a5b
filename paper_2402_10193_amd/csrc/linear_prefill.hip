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
//                                LDS (four 16-byte entries of a 256-entry byte table per word)
// and every wavefront accumulates its 64 x 64 corner twice with v_mfma_f32_16x16x32_f16: x.W^T
// and x.s^T in separate binary32 accumulators, combined as acc_b + alpha * acc_d at the end (alpha
// multiplies the finished +-1 sum, as in the decode kernels).  Global loads of step k+1 are in
// registers while step k is multiplied; LDS rows are padded to 144 bytes so that the 16-byte
// operand reads of 16 lanes fall into 16 different bank groups.
#include "bd_device.h"
#include "bd_launch.h"

namespace bd {

namespace {

constexpr int kPfRowBytes = kPrefillK * 2 + 16;            // 144
constexpr int kPfTileBytes = kPrefillTile * kPfRowBytes;   // 18432
constexpr int kPfChunks = kPrefillK / 8;                   // 16-byte chunks per tile row
constexpr int kPfPerThread = kPrefillTile * kPfChunks / 256;
constexpr int kPfLutBytes = 256 * 16;

}  // namespace

// Copies up to 960 ints that arrive in the kernel arguments to device memory: the token
// permutation reaches the GPU without a host-to-device copy call (asynchronous, capturable).
__global__ __launch_bounds__(256) void prefill_meta_kernel(const PrefillMetaChunk c, int32_t* __restrict__ dst, const int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) dst[i] = c.v[i];
}

__global__ __launch_bounds__(256, 2) void linear_prefill_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, const int32_t* __restrict__ row_token, const int32_t* __restrict__ tile_tenant,
    uint16_t* __restrict__ y, const int64_t out, const int64_t in) {
    __shared__ __align__(16) unsigned char lds[3 * kPfTileBytes + kPfLutBytes];
    unsigned char* const xs = lds;
    unsigned char* const ws = lds + kPfTileBytes;
    unsigned char* const ss = lds + 2 * kPfTileBytes;
    unsigned char* const lut = lds + 3 * kPfTileBytes;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 15, g = lane >> 4;
    const int64_t n0 = (int64_t)blockIdx.x * kPrefillTile;
    const int mt = blockIdx.y;
    const int tenant = tile_tenant[mt];
    const uint32_t* __restrict__ packed = packed_by_tenant[tenant];
    const float alpha = alpha_by_tenant[tenant];
    const int64_t words_per_row = in >> 5;

    // byte -> 8 fp16 (+1.0 where the bit is set, else -1.0), element e = bit e
    {
        const uint32_t b = (uint32_t)tid;
        u32x4 e;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            e[i] = 0xBC00BC00u ^ (((b >> (2 * i)) & 1u) << 15) ^ (((b >> (2 * i + 1)) & 1u) << 31);
        *(u32x4*)(lut + tid * 16) = e;
    }

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
        soff_lds[i] = row * kPfRowBytes + c8 * 16;
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
                    *(u32x4*)(ss + tid * kPfRowBytes + h * 64 + q * 16) = *(const u32x4*)(lut + ((sw[h] >> (8 * q)) & 0xFFu) * 16);
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
                a[i] = *(const half8*)(xs + (wm * 64 + i * 16 + r) * kPfRowBytes + h * 64 + g * 16);
                bw[i] = *(const half8*)(ws + (wn * 64 + i * 16 + r) * kPfRowBytes + h * 64 + g * 16);
                bs[i] = *(const half8*)(ss + (wn * 64 + i * 16 + r) * kPfRowBytes + h * 64 + g * 16);
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
    const unsigned gx = (unsigned)((out + kPrefillTile - 1) / kPrefillTile);
    hipLaunchKernelGGL(linear_prefill_kernel, dim3(gx, (unsigned)n_mtiles), dim3(256), 0, st, x, w, packed_by_tenant,
                       alpha_by_tenant, row_token, tile_tenant, y, out, in);
    return hipGetLastError();
}

}  // namespace bd
