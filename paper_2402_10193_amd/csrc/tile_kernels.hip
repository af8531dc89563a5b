// Row-major -> tiled serving layout (see bd_tiled.h).  Offline, like the compressor: run once
// per base matrix and once per (tenant, matrix) delta.
#include "bd_device.h"
#include "bd_tiled.h"

namespace bd {

// One thread per 16-byte unit of the tiled base: unit ((rb KT + kt) 8 + v) 64 + l holds
// W[16 rb + l % 16][256 kt + 32 v + 8 (l / 16) .. + 8].
__global__ __launch_bounds__(256) void tile_base_kernel(const uint16_t* __restrict__ w, u32x4* __restrict__ wt,
                                                         const int64_t out, const int64_t in, const int64_t KT,
                                                         const int64_t n_units) {
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < n_units; u += (int64_t)gridDim.x * blockDim.x) {
        const int l = (int)(u & 63), v = (int)((u >> 6) & 7);
        const int64_t tile = u >> 9, kt = tile % KT, rb = tile / KT;
        const int64_t row = rb * kTileRows + (l & 15), k = kt * kTileK + 32 * v + 8 * (l >> 4);
        u32x4 val = {0u, 0u, 0u, 0u};
        if (row < out && k < in) val = *(const u32x4*)(w + row * in + k);   // in % 8 == 0: the 8 elements are all inside
        wt[u] = val;
    }
}

// One thread per lane slot of the tiled signs: slot (rb KT + kt) 64 + l holds 8 bytes, byte v =
// bits 8 g .. 8 g + 7 of packed word 8 kt + v of row 16 rb + l % 16   (g = l / 16).
__global__ __launch_bounds__(256) void tile_signs_kernel(const uint32_t* __restrict__ packed, u32x2* __restrict__ st,
                                                          const int64_t out, const int64_t in, const int64_t KT,
                                                          const int64_t n_slots) {
    const int64_t words_per_row = in >> 5;
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < n_slots; u += (int64_t)gridDim.x * blockDim.x) {
        const int l = (int)(u & 63);
        const int64_t tile = u >> 6, kt = tile % KT, rb = tile / KT;
        const int64_t row = rb * kTileRows + (l & 15);
        const int sh = 8 * (l >> 4);
        u32x2 val = {0u, 0u};
        if (row < out) {
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                const int64_t wi = kt * 8 + v;
                const uint32_t byte = wi < words_per_row ? ((packed[row * words_per_row + wi] >> sh) & 0xFFu) : 0u;
                val[v >> 2] |= byte << (8 * (v & 3));
            }
        }
        st[u] = val;
    }
}

// One 16-byte unit of the 8-bit base layout per thread: unit u = ((tile * 4 + i) * 64 + l), bytes [h][e] =
// 128 + q[16 rb + l % 16][256 kt + 32 (2 i + h) + 8 (l / 16) + e]; 128 (q = 0) outside the matrix.
__global__ __launch_bounds__(256) void tile_base_q8_kernel(const int8_t* __restrict__ q, u32x4* __restrict__ wq,
                                                            const int64_t out, const int64_t in, const int64_t KT,
                                                            const int64_t n_units) {
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < n_units; u += (int64_t)gridDim.x * blockDim.x) {
        const int l = (int)(u & 63), i = (int)((u >> 6) & 3);
        const int64_t tile = u >> 8, kt = tile % KT, rb = tile / KT;
        const int64_t row = rb * kTileRows + (l & 15);
        u32x4 val = {0x80808080u, 0x80808080u, 0x80808080u, 0x80808080u};
        if (row < out) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int64_t k0 = kt * kTileK + 32 * (2 * i + h) + 8 * (l >> 4);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t byte = k0 + e < in ? (uint32_t)(uint8_t)(q[row * in + k0 + e] + 128) : 128u;
                    const int pos = 8 * h + e;
                    val[pos >> 2] = (val[pos >> 2] & ~(0xFFu << (8 * (pos & 3)))) | (byte << (8 * (pos & 3)));
                }
            }
        }
        wq[u] = val;
    }
}

// scales of the rows of every row block, zero beyond `out`
__global__ __launch_bounds__(256) void tile_scales_kernel(const float* __restrict__ scale, float* __restrict__ dst,
                                                           const int64_t out, const int64_t n_padded) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_padded; i += (int64_t)gridDim.x * blockDim.x)
        dst[i] = i < out ? scale[i] : 0.0f;
}

__global__ __launch_bounds__(256) void fill_zero_u16_kernel(uint16_t* __restrict__ p, const int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

static unsigned grid_for(int64_t n, int block) {
    int64_t g = (n + block - 1) / block;
    return (unsigned)(g < 1 ? 1 : (g > 65536 ? 65536 : g));
}

hipError_t launch_tile_base(const uint16_t* w, int64_t out, int64_t in, uint16_t* wt, hipStream_t st) {
    const int64_t KT = tiled_k_tiles(in), n_units = tiled_row_blocks(out) * KT * (kTileBaseBytes / 16);
    hipLaunchKernelGGL(tile_base_kernel, dim3(grid_for(n_units, 256)), dim3(256), 0, st, w, (u32x4*)wt, out, in, KT, n_units);
    return hipGetLastError();
}

hipError_t launch_tile_signs(const uint32_t* packed, int64_t out, int64_t in, uint32_t* st_out, hipStream_t st) {
    const int64_t KT = tiled_k_tiles(in), n_slots = tiled_row_blocks(out) * KT * 64;
    hipLaunchKernelGGL(tile_signs_kernel, dim3(grid_for(n_slots, 256)), dim3(256), 0, st, packed, (u32x2*)st_out, out, in, KT,
                       n_slots);
    return hipGetLastError();
}

// p[0 .. n) = 0 (a kernel rather than a memset node: safe to capture into a HIP graph)
hipError_t launch_fill_zero_u16(uint16_t* p, int64_t n, hipStream_t st) {
    if (n > 0) hipLaunchKernelGGL(fill_zero_u16_kernel, dim3(grid_for(n, 256)), dim3(256), 0, st, p, n);
    return hipGetLastError();
}

hipError_t launch_tile_base_q8(const int8_t* q, const float* scale, int64_t out, int64_t in, unsigned char* wq, hipStream_t st) {
    const int64_t KT = tiled_k_tiles(in), RB = tiled_row_blocks(out), n_units = RB * KT * (kTileBaseQ8Bytes / 16);
    if (n_units > 0)
        hipLaunchKernelGGL(tile_base_q8_kernel, dim3(grid_for(n_units, 256)), dim3(256), 0, st, q, (u32x4*)wq, out, in, KT, n_units);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(tile_scales_kernel, dim3(grid_for(RB * kTileRows, 256)), dim3(256), 0, st, scale,
                       (float*)(wq + RB * KT * kTileBaseQ8Bytes), out, RB * kTileRows);
    return hipGetLastError();
}

}  // namespace bd
