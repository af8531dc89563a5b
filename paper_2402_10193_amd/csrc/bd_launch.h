// Host-side launch functions of the kernel translation units, called by the C ABI layer.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <stdint.h>

#include "bd_device.h"

namespace bd {

constexpr int kCompressMaxPlanes = 8;      // iterations of the compressor one call can run
constexpr int kCompressMaxBlocks = 2048;   // also the number of binary64 partial sums in the workspace

hipError_t launch_pack_signs(const uint16_t* delta, int64_t out, int64_t in, uint32_t* packed, hipStream_t st);
// alpha_prev[0 .. n_prev): the scales of the iterations already done (device memory); n_prev = 0: the plain compressor
hipError_t launch_compress(const uint16_t* base, const uint16_t* ft, int64_t out, int64_t in, uint32_t* packed,
                           float* alpha, double* partial, hipStream_t st, const float* alpha_prev = nullptr, int n_prev = 0);

// the same with the partial sums in the library's own per-device array (no workspace, nothing allocated)
hipError_t launch_compress_noalloc(const uint16_t* base, const uint16_t* ft, int64_t out, int64_t in, uint32_t* packed,
                                   float* alpha, hipStream_t st);

// Several matrices of one fine-tune through the compressor in one launch (plus one to finish the scales).
constexpr int kCompressBatchMax = 8;
struct CompressBatch {
    const uint16_t* base[kCompressBatchMax];
    const uint16_t* ft[kCompressBatchMax];
    uint32_t* packed[kCompressBatchMax];
    int64_t n_vec[kCompressBatchMax];    // out * in / 8 of each matrix
    int32_t blocks[kCompressBatchMax];   // filled in by the launcher
    int32_t n;
};
// alpha: n floats; partial: n * kCompressMaxBlocks binary64 sums
hipError_t launch_compress_batch(CompressBatch a, float* alpha, double* partial, hipStream_t st);

// Plain vector-ALU linear: any T <= kMaxDecodeTokens per launch, tokens in caller order.
hipError_t launch_linear_rowwave(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                 const float* alpha_by_tenant, const DecodeMeta& meta, uint16_t* y, int64_t out,
                                 int64_t in, hipStream_t st);

// Prefill GEMM (many tokens per tenant).  row_token: n_mtiles * kPrefillTile ints, the token of every
// tile row or -1 for padding; tile_tenant: n_mtiles ints.  Both in device memory (the workspace).
constexpr int kPrefillTile = 128;   // tile of y: 128 tokens x 128 output features
constexpr int kPrefillK = 64;       // reduction elements per step
struct PrefillMetaChunk { int32_t v[960]; };
hipError_t launch_prefill_meta(const PrefillMetaChunk& chunk, int32_t* dst, int n, hipStream_t st);
// the same from runs: triples (first index in dst, first value, n: n > 0 values counting up, n < 0: -n copies), at most 320 per launch
hipError_t launch_prefill_meta_runs(const PrefillMetaChunk& chunk, int32_t* dst, int n_runs, hipStream_t st);
// k_planes = 0: one plane per tenant (tables indexed by tenant); k_planes = 1..8: tables indexed by tenant * k_planes +
// plane.  wscale != nullptr: w is the row-major int8 base ([out, in] bytes) and wscale its per-row scales.
hipError_t launch_linear_prefill(const uint16_t* x, const void* w, const uint32_t* const* packed_by_tenant,
                                 const float* alpha_by_tenant, const float* wscale, const int32_t* row_token,
                                 const int32_t* tile_tenant, int n_mtiles, uint16_t* y, int64_t out, int64_t in,
                                 int k_planes, hipStream_t st);
// the 128 x 256 tile GEMM of linear_prefill_big.hip; T = rows of x; halve_last_round (4 wavefronts only): the tiles of a
// last round that would occupy at most half of the compute units run as two workgroups of 64 token rows each;
// tiled (4 wavefronts only): w and the tenants' sign tensors are in the serving layout (bd_tile_base / bd_tile_signs)
bool prefill_big_fits(int64_t T, int64_t out, int64_t in);
hipError_t launch_linear_prefill_big(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                     const float* alpha_by_tenant, const int32_t* row_token, const int32_t* tile_tenant,
                                     int n_mtiles, uint16_t* y, int64_t T, int64_t out, int64_t in, int waves, bool halve_last_round,
                                     bool tiled, hipStream_t st);
// the same product as one GEMM on W + alpha S, the sum formed in fp16 on the way to the matrix cores; its token tiles
// (row_token, tile_tenant) have kPrefillMergedTile rows; halve_last_round: as above, with halves of 128 rows
constexpr int kPrefillMergedTile = 256;
hipError_t launch_linear_prefill_merged(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                        const float* alpha_by_tenant, const int32_t* row_token, const int32_t* tile_tenant,
                                        int n_mtiles, uint16_t* y, int64_t T, int64_t out, int64_t in, bool halve_last_round,
                                        bool tiled, hipStream_t st);

// 8-bit round-to-nearest base: q [out, in] int8 and one binary32 scale per row; the compressor against scale * q
hipError_t launch_quantize_rtn8(const uint16_t* w, int64_t out, int64_t in, int8_t* q, float* scale, hipStream_t st);
hipError_t launch_compress_q8(const int8_t* q, const float* scale, const uint16_t* ft, int64_t out, int64_t in,
                              uint32_t* packed, float* alpha, double* partial, hipStream_t st);
hipError_t launch_materialize(const uint16_t* w_base, const uint32_t* packed, const float* alpha, uint16_t* w_out,
                              int64_t out, int64_t in, hipStream_t st);
hipError_t launch_linear_naive(const uint16_t* x, const uint16_t* const* w_by_tenant, const DecodeMeta& meta,
                               uint16_t* y, int64_t out, int64_t in, hipStream_t st);
hipError_t launch_probe_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st);
hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t st);

// Per-device, once: a kernel attribute is a property of (kernel, device), and several host threads may
// launch at the same time.  `done` is one flag word per kernel instantiation (bit d = device d).
struct PerDeviceOnce {
    std::atomic<uint64_t> done{0};
    template <typename F>
    hipError_t run(F&& f) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const uint64_t bit = (uint64_t)1 << (dev & 63);
        if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
        e = f();   // idempotent: two threads racing here both set the same value
        if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
        return e;
    }
};

// Compute units of the current device, asked once per device (64 devices at most are remembered).
inline hipError_t device_cu_count(int* cus) {
    static std::atomic<int> cus_of[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    int c = cus_of[dev & 63].load(std::memory_order_relaxed);
    if (c == 0) {
        e = hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        if (c < 1) return hipErrorInvalidDevice;
        cus_of[dev & 63].store(c, std::memory_order_relaxed);
    }
    *cus = c;
    return hipSuccess;
}

}  // namespace bd
