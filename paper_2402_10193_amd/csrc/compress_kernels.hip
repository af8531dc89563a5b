// Offline compressor kernels (Sec. 3.1 of the paper): delta, sign bits (Eq. 2), mean |delta| (Eq. 4).
//
// Both kernels are pure streams: every lane reads 8 consecutive fp16 (one 128-bit load per
// matrix), forms one byte of sign bits, and four neighbouring lanes merge their bytes into one
// uint32 word with two cross-lane ORs.  HBM traffic is 4 B read + 1/8 B written per element for
// the compressor, 2 B + 1/8 B for the packer.
#include "bd_device.h"
#include "bd_launch.h"

namespace bd {

constexpr int kCompressThreads = 256;

__device__ __forceinline__ uint32_t merge_quad_bytes(uint32_t byte, int lane) {
    uint32_t v = byte << (8 * (lane & 3));
    v |= __shfl_xor(v, 1, kWave);
    v |= __shfl_xor(v, 2, kWave);
    return v;
}

// delta [n_vec * 8] fp16 -> packed [n_vec / 4] words.  n_vec is a multiple of 4.
__global__ __launch_bounds__(kCompressThreads) void pack_signs_kernel(
    const u32x4* __restrict__ delta, uint32_t* __restrict__ packed, int64_t n_vec) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t stride = (int64_t)gridDim.x * kCompressThreads;
    for (int64_t i = (int64_t)blockIdx.x * kCompressThreads + threadIdx.x; i < n_vec; i += stride) {
        const u32x4 d = __builtin_nontemporal_load(delta + i);
        const uint32_t w[4] = {d[0], d[1], d[2], d[3]};
        uint32_t byte = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v = h2f((uint16_t)(w[e >> 1] >> (16 * (e & 1))));
            byte |= (v > 0.0f ? 1u : 0u) << e;
        }
        const uint32_t word = merge_quad_bytes(byte, lane);
        if ((lane & 3) == 0) packed[i >> 2] = word;
    }
}

// base, ft [n_vec * 8] fp16 -> packed [n_vec / 4], partial[gridDim.x] = this block's sum |delta|.
// Iterated compression (Sec. 4.2, fidelity of Delta): with n_prev > 0 the element's delta is first
// carried through the n_prev earlier iterations, r <- r - alpha_i * Sign(r) in binary32, so that
// plane n_prev is the sign of the residual left by the planes before it.
// NPREV is a template parameter and the update a select, not a branch: with the number of earlier planes a
// run-time value the loop body was a hundred scalar branches per 8 elements, and the stream ran at half its rate.
template <int NPREV>
__global__ __launch_bounds__(kCompressThreads) void compress_kernel(
    const u32x4* __restrict__ base, const u32x4* __restrict__ ft, uint32_t* __restrict__ packed,
    double* __restrict__ partial, int64_t n_vec, const float* __restrict__ alpha_prev) {
    __shared__ double wave_part[kCompressThreads / kWave];
    float ap[NPREV > 0 ? NPREV : 1];
#pragma unroll
    for (int i = 0; i < NPREV; ++i) ap[i] = alpha_prev[i];
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t stride = (int64_t)gridDim.x * kCompressThreads;
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kCompressThreads + threadIdx.x; i < n_vec; i += stride) {
        const u32x4 b = __builtin_nontemporal_load(base + i);
        const u32x4 f = __builtin_nontemporal_load(ft + i);
        const uint32_t bw[4] = {b[0], b[1], b[2], b[3]};
        const uint32_t fw[4] = {f[0], f[1], f[2], f[3]};
        uint32_t byte = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float vb = h2f((uint16_t)(bw[e >> 1] >> (16 * (e & 1))));
            const float vf = h2f((uint16_t)(fw[e >> 1] >> (16 * (e & 1))));
            float d = vf - vb;                      // the delta of Sec. 3.1, IEEE binary32
#pragma unroll
            for (int i = 0; i < NPREV; ++i) d += d > 0.0f ? -ap[i] : ap[i];   // d - a and d + (-a) are the same binary32 number
            byte |= (d > 0.0f ? 1u : 0u) << e;      // Eq. 2: +1 only for d > 0
            s += (double)__builtin_fabsf(d);
        }
        const uint32_t word = merge_quad_bytes(byte, lane);
        if ((lane & 3) == 0) packed[i >> 2] = word;
    }
    s = wave_sum(s);
    if (lane == 0) wave_part[threadIdx.x / kWave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kCompressThreads / kWave; ++w) t += wave_part[w];
        partial[blockIdx.x] = t;
    }
}

// ---- 8-bit round-to-nearest base (Sec. 4.2 of the paper, quantized base models) ----
// One workgroup per output row: scale = max |w| / 127 in binary32 (1 for an all-zero row; NaN never enters
// the maximum), q = clamp(round-to-nearest-even(w / scale), -127, 127) with an IEEE division.
__global__ __launch_bounds__(kCompressThreads) void quantize_rtn8_kernel(const uint16_t* __restrict__ w, int8_t* __restrict__ q,
                                                                          float* __restrict__ scale, const int64_t in) {
    __shared__ float wave_max[kCompressThreads / kWave];
    const uint16_t* row = w + (int64_t)blockIdx.x * in;
    int8_t* qrow = q + (int64_t)blockIdx.x * in;
    float amax = 0.0f;
    for (int64_t c = threadIdx.x; c < in; c += kCompressThreads) {
        const float a = __builtin_fabsf(h2f(row[c]));
        if (a > amax) amax = a;
    }
#pragma unroll
    for (int off = kWave / 2; off >= 1; off >>= 1) {
        const float o = __shfl_xor(amax, off, kWave);
        if (o > amax) amax = o;
    }
    if ((threadIdx.x & (kWave - 1)) == 0) wave_max[threadIdx.x / kWave] = amax;
    __syncthreads();
    amax = wave_max[0];
#pragma unroll
    for (int i = 1; i < kCompressThreads / kWave; ++i)
        if (wave_max[i] > amax) amax = wave_max[i];
    const float s = amax > 0.0f ? amax / 127.0f : 1.0f;
    if (threadIdx.x == 0) scale[blockIdx.x] = s;
    for (int64_t c = threadIdx.x; c < in; c += kCompressThreads) {
        float v = __builtin_rintf(h2f(row[c]) / s);
        if (!(v >= -127.0f)) v = -127.0f;   // also catches NaN
        if (v > 127.0f) v = 127.0f;
        qrow[c] = (int8_t)v;
    }
}

// The compressor against the quantised base: delta = f32(w_ft) - scale[n] * q[n,k].  Every lane takes 8
// consecutive elements of one row (in % 32 == 0), four lanes merge their bytes into one word.
__global__ __launch_bounds__(kCompressThreads) void compress_q8_kernel(
    const u32x2* __restrict__ q, const float* __restrict__ scale, const u32x4* __restrict__ ft,
    uint32_t* __restrict__ packed, double* __restrict__ partial, const int64_t n_vec, const int64_t vec_per_row) {
    __shared__ double wave_part[kCompressThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t stride = (int64_t)gridDim.x * kCompressThreads;
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kCompressThreads + threadIdx.x; i < n_vec; i += stride) {
        const u32x2 qv = __builtin_nontemporal_load(q + i);
        const u32x4 f = __builtin_nontemporal_load(ft + i);
        const float sc = scale[i / vec_per_row];
        const uint32_t qw[2] = {qv[0], qv[1]};
        const uint32_t fw[4] = {f[0], f[1], f[2], f[3]};
        uint32_t byte = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float vb = sc * (float)(int8_t)(qw[e >> 2] >> (8 * (e & 3)));
            const float vf = h2f((uint16_t)(fw[e >> 1] >> (16 * (e & 1))));
            const float d = vf - vb;
            byte |= (d > 0.0f ? 1u : 0u) << e;
            s += (double)__builtin_fabsf(d);
        }
        const uint32_t word = merge_quad_bytes(byte, lane);
        if ((lane & 3) == 0) packed[i >> 2] = word;
    }
    s = wave_sum(s);
    if (lane == 0) wave_part[threadIdx.x / kWave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kCompressThreads / kWave; ++w) t += wave_part[w];
        partial[blockIdx.x] = t;
    }
}

// The compressor (no earlier planes) over up to kCompressBatchMax matrices in one launch.  Matrix m is cut into
// blocks[m] blocks exactly as a launch of compress_kernel for it alone would be, so its partial sums -- and with
// them its scale -- are the same bit for bit.
__global__ __launch_bounds__(kCompressThreads) void compress_batch_kernel(const CompressBatch a, double* __restrict__ partial) {
    __shared__ double wave_part[kCompressThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    for (int m = 0; m < a.n; ++m) {
        if ((int)blockIdx.x >= a.blocks[m]) continue;   // uniform per block
        const u32x4* __restrict__ base = (const u32x4*)a.base[m];
        const u32x4* __restrict__ ft = (const u32x4*)a.ft[m];
        uint32_t* __restrict__ packed = a.packed[m];
        const int64_t n_vec = a.n_vec[m];
        const int64_t stride = (int64_t)a.blocks[m] * kCompressThreads;
        double s = 0.0;
        for (int64_t i = (int64_t)blockIdx.x * kCompressThreads + threadIdx.x; i < n_vec; i += stride) {
            const u32x4 b = __builtin_nontemporal_load(base + i);
            const u32x4 f = __builtin_nontemporal_load(ft + i);
            const uint32_t bw[4] = {b[0], b[1], b[2], b[3]};
            const uint32_t fw[4] = {f[0], f[1], f[2], f[3]};
            uint32_t byte = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float vb = h2f((uint16_t)(bw[e >> 1] >> (16 * (e & 1))));
                const float vf = h2f((uint16_t)(fw[e >> 1] >> (16 * (e & 1))));
                const float d = vf - vb;
                byte |= (d > 0.0f ? 1u : 0u) << e;
                s += (double)__builtin_fabsf(d);
            }
            const uint32_t word = merge_quad_bytes(byte, lane);
            if ((lane & 3) == 0) packed[i >> 2] = word;
        }
        s = wave_sum(s);
        if (lane == 0) wave_part[threadIdx.x / kWave] = s;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
#pragma unroll
            for (int w = 0; w < kCompressThreads / kWave; ++w) t += wave_part[w];
            partial[(size_t)m * kCompressMaxBlocks + blockIdx.x] = t;
        }
        __syncthreads();   // wave_part is free again
    }
}

// binary64 -> binary16 with ONE rounding to nearest even, returned as a float.  There is no such conversion in
// hardware; going through binary32 would round twice (a mean a hair above the middle between two binary16 neighbours
// lands on the middle first and then, as a tie, on the even neighbour).  So the binary32 step rounds to ODD instead:
// truncate towards zero and set the last bit if anything was dropped; binary32 keeps 13 more bits than binary16, so
// the final rounding then sees on which side of every binary16 middle the mean really lies.
__device__ __forceinline__ float f64_to_f16_once(const double v) {
    float f = (float)v;   // nearest even
    if ((double)f != v && __builtin_isfinite(f)) {   // inexact (NaN stays as it is)
        uint32_t bits = __builtin_bit_cast(uint32_t, f);
        if (__builtin_fabs((double)f) > __builtin_fabs(v)) bits -= 1u;   // back to the truncated value
        bits |= 1u;
        f = __builtin_bit_cast(float, bits);
    }
    return (float)(_Float16)f;
}

// alpha = fp16_rne( sum(partial) / count ), one block, fixed summation order.
__global__ __launch_bounds__(256) void alpha_finalize_kernel(const double* __restrict__ partial, int n_partial,
                                                             double count, float* __restrict__ alpha) {
    __shared__ double sm[256];
    double t = 0.0;
    for (int i = threadIdx.x; i < n_partial; i += 256) t += partial[i];
    sm[threadIdx.x] = t;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) sm[threadIdx.x] += sm[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double mean = count > 0.0 ? sm[0] / count : 0.0;
        *alpha = f64_to_f16_once(mean);   // one rounding to fp16, carried as a float
    }
}

// the same per matrix of a batch: block m finishes matrix m
__global__ __launch_bounds__(256) void alpha_finalize_batch_kernel(const double* __restrict__ partial, const CompressBatch a,
                                                                   float* __restrict__ alpha) {
    __shared__ double sm[256];
    const int m = blockIdx.x;
    const double* p = partial + (size_t)m * kCompressMaxBlocks;
    double t = 0.0;
    for (int i = threadIdx.x; i < a.blocks[m]; i += 256) t += p[i];
    sm[threadIdx.x] = t;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) sm[threadIdx.x] += sm[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double count = (double)a.n_vec[m] * 8.0;
        const double mean = count > 0.0 ? sm[0] / count : 0.0;
        alpha[m] = f64_to_f16_once(mean);
    }
}

int compress_grid_blocks(int64_t n_vec) {
    // enough blocks to fill 256 CUs several times over, few enough that the partial sums stay tiny
    const int64_t want = (n_vec + kCompressThreads - 1) / kCompressThreads;
    return (int)(want < 1 ? 1 : (want > kCompressMaxBlocks ? kCompressMaxBlocks : want));
}

hipError_t launch_pack_signs(const uint16_t* delta, int64_t out, int64_t in, uint32_t* packed, hipStream_t st) {
    const int64_t n_vec = out * in / 8;
    hipLaunchKernelGGL(pack_signs_kernel, dim3(compress_grid_blocks(n_vec)), dim3(kCompressThreads), 0, st,
                       (const u32x4*)delta, packed, n_vec);
    return hipGetLastError();
}

hipError_t launch_compress(const uint16_t* base, const uint16_t* ft, int64_t out, int64_t in, uint32_t* packed,
                           float* alpha, double* partial, hipStream_t st, const float* alpha_prev, int n_prev) {
    if (n_prev < 0 || n_prev > kCompressMaxPlanes - 1 || (n_prev > 0 && !alpha_prev)) return hipErrorInvalidValue;
    const int64_t n_vec = out * in / 8;
    int blocks = 0;
    if (n_vec > 0) {
        blocks = compress_grid_blocks(n_vec);
        const dim3 g(blocks), b(kCompressThreads);
        const u32x4 *pb = (const u32x4*)base, *pf = (const u32x4*)ft;
        switch (n_prev) {
            case 0: hipLaunchKernelGGL(compress_kernel<0>, g, b, 0, st, pb, pf, packed, partial, n_vec, alpha_prev); break;
            case 1: hipLaunchKernelGGL(compress_kernel<1>, g, b, 0, st, pb, pf, packed, partial, n_vec, alpha_prev); break;
            case 2: hipLaunchKernelGGL(compress_kernel<2>, g, b, 0, st, pb, pf, packed, partial, n_vec, alpha_prev); break;
            case 3: hipLaunchKernelGGL(compress_kernel<3>, g, b, 0, st, pb, pf, packed, partial, n_vec, alpha_prev); break;
            case 4: hipLaunchKernelGGL(compress_kernel<4>, g, b, 0, st, pb, pf, packed, partial, n_vec, alpha_prev); break;
            case 5: hipLaunchKernelGGL(compress_kernel<5>, g, b, 0, st, pb, pf, packed, partial, n_vec, alpha_prev); break;
            case 6: hipLaunchKernelGGL(compress_kernel<6>, g, b, 0, st, pb, pf, packed, partial, n_vec, alpha_prev); break;
            default: hipLaunchKernelGGL(compress_kernel<7>, g, b, 0, st, pb, pf, packed, partial, n_vec, alpha_prev); break;
        }
        static_assert(kCompressMaxPlanes - 1 == 7, "one instantiation per number of earlier planes");
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(alpha_finalize_kernel, dim3(1), dim3(256), 0, st, (const double*)partial, blocks,
                       (double)out * (double)in, alpha);
    return hipGetLastError();
}

hipError_t launch_compress_batch(CompressBatch a, float* alpha, double* partial, hipStream_t st) {
    if (a.n < 1 || a.n > kCompressBatchMax) return hipErrorInvalidValue;
    int grid = 0;
    for (int m = 0; m < a.n; ++m) {
        a.blocks[m] = a.n_vec[m] > 0 ? compress_grid_blocks(a.n_vec[m]) : 0;
        grid = a.blocks[m] > grid ? a.blocks[m] : grid;
    }
    if (grid > 0) {
        hipLaunchKernelGGL(compress_batch_kernel, dim3(grid), dim3(kCompressThreads), 0, st, a, partial);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(alpha_finalize_batch_kernel, dim3(a.n), dim3(256), 0, st, (const double*)partial, a, alpha);
    return hipGetLastError();
}

// ---- the compressor for callers that cannot allocate ----
// Its partial sums live in this array instead of a workspace of the caller's: kCompressMaxBlocks binary64 numbers,
// 16 KiB, held by every device the library runs on until the process ends.  In host code the name stands for the
// array, it is not its address: the address on the current device is asked for once per device and kept.
static __device__ __align__(256) double scratch[kCompressMaxBlocks];

static hipError_t scratch_on_current_device(double** out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<double*> ptr_of[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    double* p = ptr_of[dev].load(std::memory_order_acquire);
    if (!p) {   // first call on this device (two threads racing here get the same answer)
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr_of[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

// Every block of compress_kernel writes its slot before alpha_finalize_kernel reads slots [0, blocks): nothing in the
// array has to start at zero, and what an earlier (possibly larger) call left in the slots beyond `blocks` is never read.
hipError_t launch_compress_noalloc(const uint16_t* base, const uint16_t* ft, int64_t out, int64_t in, uint32_t* packed,
                                   float* alpha, hipStream_t st) {
    double* partial = nullptr;
    const hipError_t e = scratch_on_current_device(&partial);
    if (e != hipSuccess) return e;
    return launch_compress(base, ft, out, in, packed, alpha, partial, st, nullptr, 0);
}

hipError_t launch_quantize_rtn8(const uint16_t* w, int64_t out, int64_t in, int8_t* q, float* scale, hipStream_t st) {
    if (out > 0) hipLaunchKernelGGL(quantize_rtn8_kernel, dim3((unsigned)out), dim3(kCompressThreads), 0, st, w, q, scale, in);
    return hipGetLastError();
}

hipError_t launch_compress_q8(const int8_t* q, const float* scale, const uint16_t* ft, int64_t out, int64_t in,
                              uint32_t* packed, float* alpha, double* partial, hipStream_t st) {
    const int64_t n_vec = out * in / 8;
    int blocks = 0;
    if (n_vec > 0) {
        blocks = compress_grid_blocks(n_vec);
        hipLaunchKernelGGL(compress_q8_kernel, dim3(blocks), dim3(kCompressThreads), 0, st, (const u32x2*)q, scale,
                           (const u32x4*)ft, packed, partial, n_vec, in / 8);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(alpha_finalize_kernel, dim3(1), dim3(256), 0, st, (const double*)partial, blocks,
                       (double)out * (double)in, alpha);
    return hipGetLastError();
}

}  // namespace bd
