// Plain vector-ALU form of the multi-tenant linear (Eq. 6 of the paper).
//
// One wavefront owns one output row n and a chunk of up to kTok tokens.  Each lane walks the
// reduction dimension in steps of 512 elements, 8 consecutive fp16 per 128-bit load; the sign
// bits of those 8 elements are one byte of the tenant's packed row.  Both sums are kept in
// binary32 and folded across the wavefront at the end.  The kernel is the simple, general
// fallback (any token count, any token order) and the reference point the matrix-core kernels
// are measured against; it re-reads the base row once per token chunk.
#include "bd_device.h"
#include "bd_launch.h"

namespace bd {

constexpr int kRowWaveThreads = 256;
constexpr int kRowsPerBlock = kRowWaveThreads / kWave;
constexpr int kTok = 4;

__global__ __launch_bounds__(kRowWaveThreads) void linear_rowwave_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, DecodeMeta meta, uint16_t* __restrict__ y, int64_t out, int64_t in) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t n = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.x / kWave;
    const int t0 = blockIdx.y * kTok;
    if (n >= out) return;   // whole wavefront leaves together

    const uint8_t* srow[kTok];
    float alpha[kTok];
    const uint16_t* xrow[kTok];
#pragma unroll
    for (int j = 0; j < kTok; ++j) {
        const int t = (t0 + j < meta.T) ? t0 + j : meta.T - 1;   // clamp: duplicates are computed and dropped
        const int tenant = meta.tenant_of_token[t];
        srow[j] = (const uint8_t*)packed_by_tenant[tenant] + n * (in / 8);
        alpha[j] = alpha_by_tenant[tenant];
        xrow[j] = x + (int64_t)t * in;
    }
    const uint16_t* wrow = w + n * in;

    float acc_b[kTok], acc_d[kTok];
#pragma unroll
    for (int j = 0; j < kTok; ++j) acc_b[j] = acc_d[j] = 0.0f;

    for (int64_t k = (int64_t)lane * 8; k < in; k += kWave * 8) {
        const u32x4 wv = *(const u32x4*)(wrow + k);
        float wf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) wf[e] = h2f((uint16_t)(wv[e >> 1] >> (16 * (e & 1))));
#pragma unroll
        for (int j = 0; j < kTok; ++j) {
            const u32x4 xv = *(const u32x4*)(xrow[j] + k);
            const uint32_t bits = srow[j][k >> 3];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float xf = h2f((uint16_t)(xv[e >> 1] >> (16 * (e & 1))));
                acc_b[j] = __builtin_fmaf(xf, wf[e], acc_b[j]);
                acc_d[j] += ((bits >> e) & 1u) ? xf : -xf;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kTok; ++j) {
        const float b = wave_sum(acc_b[j]);
        const float d = wave_sum(acc_d[j]);
        if (lane == 0 && t0 + j < meta.T) y[(int64_t)(t0 + j) * out + n] = f2h_rne(b + alpha[j] * d);
    }
}

hipError_t launch_linear_rowwave(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                 const float* alpha_by_tenant, const DecodeMeta& meta, uint16_t* y, int64_t out,
                                 int64_t in, hipStream_t st) {
    const dim3 grid((unsigned)((out + kRowsPerBlock - 1) / kRowsPerBlock), (unsigned)((meta.T + kTok - 1) / kTok));
    hipLaunchKernelGGL(linear_rowwave_kernel, grid, dim3(kRowWaveThreads), 0, st, x, w, packed_by_tenant,
                       alpha_by_tenant, meta, y, out, in);
    return hipGetLastError();
}

}  // namespace bd
