// The serving ("tiled") layout of the base weight and of a packed 1-bit delta, and the kernel
// arguments of the decode kernel that reads it.
//
// A weight matrix [out, in] is cut into tiles of 16 output rows x 256 reduction elements, the
// unit one wavefront consumes per step.  Inside a tile every byte sits where the matrix-core
// instruction v_mfma_f32_16x16x32_f16 wants it: MFMA slice v (0..7) covers k = 32 v .. 32 v + 31
// of the tile, and lane l = (r, g) = (l % 16, l / 16) supplies row r, elements 8 g .. 8 g + 7 of the slice.
//
//   base   Wt[rb][kt][v][l][e]  fp16  = W[16 rb + r][256 kt + 32 v + 8 g + e]          (8 KiB per tile)
//   signs  St[rb][kt][l][v]     byte, bit e = sign of element (16 rb + r, 256 kt + 32 v + 8 g + e)  (512 B per tile)
//
// so one 128-bit load per lane fetches a whole slice of the base (1 KiB contiguous per wavefront)
// and one 64-bit load per lane fetches a tenant's signs of the whole tile (512 B contiguous).
// Rows beyond `out` and elements beyond `in` are stored as zeros.  Tiles are ordered [rb][kt], kt fastest.
//
// 8-bit base (quantised, one binary32 scale per output row): one byte per weight, u = q + 128, and a
// lane's 16 bytes of a load are two consecutive slices,
//   base8  Wq[rb][kt][i][l][h][e]  byte = 128 + q[16 rb + r][256 kt + 32 (2 i + h) + 8 g + e]   i<4, h<2   (4 KiB per tile)
// (padding: u = 128, i.e. q = 0).  The scales follow the tiles in the same tensor, one float per row of
// every row block (padded with zeros to 16 per block).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bd {

constexpr int kTileRows = 16;
constexpr int kTileK = 256;
constexpr int kTileBaseBytes = kTileRows * kTileK * 2;   // 8192
constexpr int kTileBaseQ8Bytes = kTileRows * kTileK;     // 4096
constexpr int kTileSignBytes = kTileRows * kTileK / 8;   // 512
constexpr int kTiledMaxMats = 3;                         // matrices one launch can cover (q,k,v or gate,up)
constexpr int kTiledMaxJobs = 16;                        // delta jobs (distinct tenants) per launch
constexpr int kTiledMaxTokens = 16;                      // one 16-column MFMA tile
constexpr int kTiledMaxCt = 2;                           // column tiles one launch can cover (32 tokens)
constexpr int kTiledMaxPlanes = 8;                       // sign planes per tenant (iterated compression)

inline int64_t tiled_row_blocks(int64_t out) { return (out + kTileRows - 1) / kTileRows; }
inline int64_t tiled_k_tiles(int64_t in) { return (in + kTileK - 1) / kTileK; }

// Everything the kernel needs arrives in the kernel arguments (scalar loads, no dependent
// fetch of a pointer table from memory before the first weight load can be issued).
struct TiledArgs {
    const uint16_t* x;                                        // [T, in] fp16
    const uint16_t* wt[kTiledMaxMats];                        // tiled base of each matrix
    uint16_t* y[kTiledMaxMats];                               // [T, out_m] fp16
    const float* alpha[kTiledMaxMats];                        // device array indexed by tenant id
    const float* wscale[kTiledMaxMats];                       // 8-bit base only: per-row scales, 16 per row block
    int32_t out[kTiledMaxMats];
    int32_t rb_end[kTiledMaxMats];                            // cumulative row blocks: matrix m owns blocks [rb_end[m-1], rb_end[m])
    int32_t in, KT, n_mats, n_ct;                             // n_ct column tiles of up to 16 tokens each
    int32_t T[kTiledMaxCt];                                   // tokens (columns in use) of each column tile
    // per column tile ct: its job slots and its sorted columns
    const uint32_t* signs[kTiledMaxCt][kTiledMaxMats][kTiledMaxJobs];   // tiled delta of job slot j, matrix m
    int32_t col_token[kTiledMaxCt][kTiledMaxTokens];          // sorted column -> token (row of x and y)
    int32_t col_job[kTiledMaxCt][kTiledMaxTokens];            // sorted column -> job slot owning it
    int32_t col_tenant[kTiledMaxCt][kTiledMaxTokens];         // sorted column -> index into alpha[m] (tenant, or tenant * k + plane)
    // Several sign planes per tenant (iterated compression): a token occupies `span` consecutive columns
    // that all carry its x, one per plane; the first holds span, the others 0.  Their results are added
    // when y is written and only the first contributes the base product.  One plane: all 1.
    int32_t col_span[kTiledMaxCt][kTiledMaxTokens];
    int32_t planes;                                           // k: 1 = plain 1-bit deltas
    // Row-major entry points only (wt[0] = W [out, in] row-major, signs[][][] unused): the caller's DEVICE table of
    // packed deltas [out, in/32], entry tenant * planes + plane, and the table index of every job slot (slots beyond
    // the jobs repeat slot 0's).
    const uint32_t* const* packed_by_tenant;
    int32_t job_tenant[kTiledMaxCt][kTiledMaxJobs];
};

hipError_t launch_fill_zero_u16(uint16_t* p, int64_t n, hipStream_t st);
hipError_t launch_tile_base(const uint16_t* w, int64_t out, int64_t in, uint16_t* wt, hipStream_t st);
hipError_t launch_tile_signs(const uint32_t* packed, int64_t out, int64_t in, uint32_t* st_out, hipStream_t st);
// n_jobs real job slots per column tile (1..16, the larger of the two); unused slots must repeat slot 0's pointers.
hipError_t launch_linear_decode_tiled(const TiledArgs& args, int n_jobs, hipStream_t st);
// the same kernel over the row-major tensors of bd_linear_multitenant (one matrix, in % 128 == 0)
hipError_t launch_linear_decode_rowmajor(const TiledArgs& args, int n_jobs, hipStream_t st);
// the same over an 8-bit base: args.wt point at base8 tiles, args.wscale at their scales
hipError_t launch_linear_decode_tiled_q8(const TiledArgs& args, int n_jobs, hipStream_t st);
// the row-major 8-bit base: args.wt[0] = q [out, in] int8, args.wscale[0] = the `out` scales (one matrix)
hipError_t launch_linear_decode_rowmajor_q8(const TiledArgs& args, int n_jobs, hipStream_t st);
// q [out, in] int8, scale [out] -> base8 tiles followed by the padded scales
hipError_t launch_tile_base_q8(const int8_t* q, const float* scale, int64_t out, int64_t in, unsigned char* wq, hipStream_t st);

}  // namespace bd
