// Device-side helpers shared by the gfx950 kernels of this library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bd {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kMaxDecodeTokens = 32;  // tokens one decode launch handles (two 16-column MFMA tiles)

// Token/tenant bookkeeping of one decode launch, passed by value in the kernel arguments so
// that a call needs no host-to-device copy (all fields are 32-bit so they arrive by scalar loads).  Columns are the launch's tokens sorted by tenant
// (stable); a "job" is one tenant's run of columns inside one 16-column tile.
struct DecodeMeta {
    int32_t T;                                  // tokens in this launch, 1..32
    int32_t n_jobs;                             // delta jobs, 1..32
    int32_t tenant_of_token[kMaxDecodeTokens];  // caller order
    int32_t token_of_col[kMaxDecodeTokens];     // sorted column -> token index inside this launch
    int32_t job_tenant[kMaxDecodeTokens];       // tenant id of the job
    int32_t job_tile[kMaxDecodeTokens];         // which 16-column tile the job's columns are in
    int32_t job_col_begin[kMaxDecodeTokens];    // first column (0..15, inside the tile)
    int32_t job_col_end[kMaxDecodeTokens];      // one past the last column (inside the tile)
    int32_t tenant_of_col[kMaxDecodeTokens];    // tenant of each sorted column
    int32_t tile_job_begin[2];                  // first job of each 16-column tile
    int32_t tile_job_end[2];                    // one past its last job
    // The same jobs laid out per tile in 16 fixed slots, so that the kernel reads them with
    // constant indices: slot s of tile t is job tile_job_begin[t] + s; slots beyond the tile's
    // jobs repeat its first tenant with an empty column range (never selected).
    int32_t slot_tenant[2][16];
    int32_t slot_col_begin[2][16];
    int32_t slot_col_end[2][16];
};

__device__ __forceinline__ float h2f(uint16_t bits) {
    return (float)__builtin_bit_cast(_Float16, bits);
}

__device__ __forceinline__ uint16_t f2h_rne(float v) {
    return __builtin_bit_cast(uint16_t, (_Float16)v);   // v_cvt_f16_f32: round to nearest even
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

}  // namespace bd
