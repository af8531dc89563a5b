// C ABI of the library (include/bitdelta.h): argument checks, token grouping, kernel choice.
// Everything here runs on the host; nothing is enqueued before the arguments have passed.
#include "bitdelta.h"

#include <algorithm>
#include <cstring>
#include <vector>

#include "bd_launch.h"
#include "bd_tiled.h"

namespace {

using bd::DecodeMeta;
using bd::kMaxDecodeTokens;

constexpr int kVersion = 220;   // 0.2.20
constexpr int kVariantRowWave = 1;
constexpr int kVariantRowMajorMfma = 2;   // the matrix-core decode kernel on the row-major tensors (in % 128 == 0)
constexpr int kVariantPrefillSmall = 4;   // T > 32 with a workspace: the 128 x 128 tile GEMM
constexpr int kVariantPrefillBig = 5;     // ... the 128 x 256 tile GEMM (in % 64 == 0), one wavefront per SIMD
constexpr int kVariantPrefillBig8 = 6;    // ... the same tile with two wavefronts per SIMD
constexpr int kVariantPrefillBigWhole = 7;   // ... as 5, but never cutting the tiles of the last round in two
constexpr int kVariantPrefillMerged = 8;     // ... one product on W + alpha S, formed in fp16 on the way to the matrix cores (256 x 256 tiles)

inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

inline bool overlaps(const void* a, size_t abytes, const void* b, size_t bbytes) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

// Tokens [t0, t0 + n) of the call -> one launch's bookkeeping: columns sorted by tenant
// (stable), jobs = runs of equal tenant cut at the 16-column tile boundary.
void build_meta(const int32_t* tenant_of_token, int64_t t0, int n, DecodeMeta* m) {
    std::memset(m, 0, sizeof(*m));
    m->T = n;
    int order[kMaxDecodeTokens];
    for (int i = 0; i < n; ++i) {
        order[i] = i;
        m->tenant_of_token[i] = tenant_of_token[t0 + i];
    }
    std::stable_sort(order, order + n, [&](int a, int b) { return m->tenant_of_token[a] < m->tenant_of_token[b]; });
    int jobs = 0;
    for (int col = 0; col < n; ++col) {
        const int tok = order[col];
        const int tenant = m->tenant_of_token[tok];
        m->token_of_col[col] = (int32_t)tok;
        m->tenant_of_col[col] = tenant;
        const int tile = col >> 4, cin = col & 15;
        if (jobs > 0 && m->job_tenant[jobs - 1] == tenant && m->job_tile[jobs - 1] == tile) {
            m->job_col_end[jobs - 1] = (int32_t)(cin + 1);
        } else {
            m->job_tenant[jobs] = tenant;
            m->job_tile[jobs] = (int32_t)tile;
            m->job_col_begin[jobs] = (int32_t)cin;
            m->job_col_end[jobs] = (int32_t)(cin + 1);
            ++jobs;
        }
    }
    m->n_jobs = jobs;
    for (int tile = 0; tile < 2; ++tile) {
        int b = 0;
        while (b < jobs && m->job_tile[b] < tile) ++b;
        int e = b;
        while (e < jobs && m->job_tile[e] == tile) ++e;
        m->tile_job_begin[tile] = b;
        m->tile_job_end[tile] = e;
        for (int sl = 0; sl < 16; ++sl) {
            const bool real = b + sl < e;
            m->slot_tenant[tile][sl] = real ? m->job_tenant[b + sl] : (b < e ? m->job_tenant[b] : 0);
            m->slot_col_begin[tile][sl] = real ? m->job_col_begin[b + sl] : 0;
            m->slot_col_end[tile][sl] = real ? m->job_col_end[b + sl] : 0;
        }
    }
}

bd_status check_linear_args(const void* x, const void* w, const void* packed_by_tenant, const void* alpha_by_tenant,
                            const int32_t* tenant_of_token, const void* y, int64_t T, int64_t out, int64_t in,
                            int32_t n_tenants, size_t w_bytes_per_el = 2) {
    if (T < 0 || out < 0 || in < 0 || n_tenants < 0 || T > 65535) return BD_ERR_SHAPE;
    if (in % 32 != 0) return BD_ERR_SHAPE;
    if (out > (int64_t)1 << 31 || in > (int64_t)1 << 31) return BD_ERR_SHAPE;
    if (T == 0 || out == 0) return BD_OK;
    if (!x || !w || !packed_by_tenant || !alpha_by_tenant || !tenant_of_token || !y) return BD_ERR_NULL;
    if (misaligned(x, 16) || misaligned(w, 16) || misaligned(y, 16) || misaligned(packed_by_tenant, 8) ||
        misaligned(alpha_by_tenant, 4))
        return BD_ERR_ALIGN;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return BD_ERR_TENANT;
    const size_t ybytes = (size_t)T * out * 2;
    if (overlaps(y, ybytes, x, (size_t)T * in * 2) || overlaps(y, ybytes, w, (size_t)out * in * w_bytes_per_el)) return BD_ERR_ALIAS;
    return BD_OK;
}

// Prefill (T > 32): the token permutation and the tenant of every 128-row tile live in the workspace.
// At most ceil(T / 128) full tiles plus one ragged tile per tenant that has a token.
size_t prefill_table_bytes(int64_t T, int32_t n_tenants, bool merged_too = false);
size_t prefill_workspace_bytes(int64_t T, int32_t n_tenants) {
    if (T <= kMaxDecodeTokens || n_tenants < 0) return 0;
    return prefill_table_bytes(T, n_tenants, true);
}
size_t tiled_gemm_workspace_bytes(int64_t T, int32_t n_tenants);
// The token tables of the GEMM: tiles of 128 rows (merged_too: or of the 256 rows of the one-product form, whichever
// table is larger); every tenant with a token ends in one partly filled tile at most.
size_t prefill_table_bytes(int64_t T, int32_t n_tenants, bool merged_too) {
    if (T < 1 || n_tenants < 0) return 0;
    size_t bytes = 0;
    for (const int64_t rows : {(int64_t)bd::kPrefillTile, (int64_t)bd::kPrefillMergedTile}) {
        if (rows != bd::kPrefillTile && !merged_too) continue;
        const int64_t tiles = (T + rows - 1) / rows + std::min<int64_t>(n_tenants, T);
        bytes = std::max(bytes, (size_t)tiles * (size_t)(rows + 1) * sizeof(int32_t));
    }
    return (bytes + 255) & ~(size_t)255;
}

// bd_linear_multitenant_tiled_gemm: the token tables and, behind them, the table of the tenants' sign pointers
size_t tiled_gemm_workspace_bytes(int64_t T, int32_t n_tenants) {
    const size_t tables = prefill_table_bytes(T, n_tenants, true);
    if (tables == 0) return 0;
    return tables + (((size_t)n_tenants * 8 + 8 + 255) & ~(size_t)255);
}

// Sorts the tokens by tenant (stable), cuts them into tiles of 128 rows (merged: 256) that never mix tenants, writes
// the two tables into the workspace (through kernel arguments: no host-to-device copy call) and runs the GEMM.
// k_planes = 0: one plane per tenant; 1..8: tables indexed by tenant * k_planes + plane.  wscale: the 8-bit base's row
// scales (w is then the int8 tensor).  Both go through the 128 x 128 tiles (big_waves = 0).
hipError_t run_prefill(const uint16_t* x, const void* w, const uint32_t* const* packed_by_tenant,
                       const float* alpha_by_tenant, const int32_t* tenant_of_token, uint16_t* y, int64_t T, int64_t out,
                       int64_t in, void* workspace, hipStream_t st, int big_waves, bool halve_last_round,
                       int k_planes = 0, const float* wscale = nullptr, bool merged = false,
                       const uint32_t* const* tiled_by_tenant_host = nullptr, int32_t n_tenants = 0) {
    const int64_t tile_rows = merged ? bd::kPrefillMergedTile : bd::kPrefillTile;
    std::vector<int32_t> order((size_t)T);
    for (int64_t i = 0; i < T; ++i) order[(size_t)i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return tenant_of_token[a] < tenant_of_token[b]; });
    std::vector<int32_t> row_token, tile_tenant;
    for (int64_t i = 0; i < T;) {
        const int32_t tenant = tenant_of_token[order[(size_t)i]];
        int64_t e = i;
        while (e < T && tenant_of_token[order[(size_t)e]] == tenant) ++e;
        for (int64_t t0 = i; t0 < e; t0 += tile_rows) {
            tile_tenant.push_back(tenant);
            for (int64_t rrow = 0; rrow < tile_rows; ++rrow)
                row_token.push_back(t0 + rrow < e ? order[(size_t)(t0 + rrow)] : -1);
        }
        i = e;
    }
    const int n_mtiles = (int)tile_tenant.size();
    std::vector<int32_t> all(row_token);
    all.insert(all.end(), tile_tenant.begin(), tile_tenant.end());
    // Serving layout: the tenants' sign pointers come as a host array; the GEMM reads them from a device table, which
    // travels behind the token tables (8-byte aligned).
    const bool tiled = tiled_by_tenant_host != nullptr;
    size_t pointer_table_at = 0;
    if (tiled) {
        if (all.size() & 1) all.push_back(0);
        pointer_table_at = all.size();
        for (int32_t t = 0; t < n_tenants; ++t) {
            const uint64_t p = (uint64_t)(uintptr_t)tiled_by_tenant_host[t];
            all.push_back((int32_t)(uint32_t)p);
            all.push_back((int32_t)(uint32_t)(p >> 32));
        }
    }
    int32_t* dst = (int32_t*)workspace;
    // The tables as runs of values that count up or repeat (tokens that arrive grouped by tenant: a few runs for the
    // whole batch), where that takes fewer launches than the values themselves.
    std::vector<int32_t> runs;   // triples: first index, first value, n (> 0 counting up, < 0 repeated)
    for (size_t i = 0; i < all.size();) {
        size_t e = i + 1;
        const int32_t step = e < all.size() ? all[e] - all[i] : 0;
        if (step == 0 || step == 1)
            while (e < all.size() && all[e] - all[e - 1] == step) ++e;
        runs.insert(runs.end(), {(int32_t)i, all[i], step == 1 ? (int32_t)(e - i) : -(int32_t)(e - i)});
        i = e;
    }
    if ((runs.size() / 3 + 319) / 320 < (all.size() + 959) / 960) {
        for (size_t off = 0; off < runs.size(); off += 960) {
            bd::PrefillMetaChunk c;
            const int n = (int)std::min<size_t>(960, runs.size() - off);
            std::memcpy(c.v, runs.data() + off, (size_t)n * sizeof(int32_t));
            const hipError_t e = bd::launch_prefill_meta_runs(c, dst, n / 3, st);
            if (e != hipSuccess) return e;
        }
    } else {
        for (size_t off = 0; off < all.size(); off += 960) {
            bd::PrefillMetaChunk c;
            const int n = (int)std::min<size_t>(960, all.size() - off);
            std::memcpy(c.v, all.data() + off, (size_t)n * sizeof(int32_t));
            const hipError_t e = bd::launch_prefill_meta(c, dst + off, n, st);
            if (e != hipSuccess) return e;
        }
    }
    if (tiled) packed_by_tenant = (const uint32_t* const*)(dst + pointer_table_at);
    if (merged)
        return bd::launch_linear_prefill_merged(x, (const uint16_t*)w, packed_by_tenant, alpha_by_tenant, dst,
                                                dst + row_token.size(), n_mtiles, y, T, out, in, halve_last_round, tiled, st);
    if (big_waves)
        return bd::launch_linear_prefill_big(x, (const uint16_t*)w, packed_by_tenant, alpha_by_tenant, dst,
                                             dst + row_token.size(), n_mtiles, y, T, out, in, big_waves, halve_last_round, tiled, st);
    if (tiled) return hipErrorInvalidValue;   // the 128 x 128 tiles read the row-major tensors only
    return bd::launch_linear_prefill(x, w, packed_by_tenant, alpha_by_tenant, wscale, dst, dst + row_token.size(), n_mtiles, y,
                                     out, in, k_planes, st);
}

// Which way is quicker for T > 32 tokens when both are possible: one GEMM launch, whose tiles of 128 token rows
// never mix tenants (a tenant with 3 tokens still costs a whole tile), or decode launches of 32 tokens each, which
// re-read the base per launch but spend nothing on empty rows.  Rough model from measured rates (MI355X, graph
// replay): a 128 x 256 tile takes 1.45 us per 64-wide k step plus 10 us around the loop, one tile per compute unit at
// a time; a decode launch of the matrix-core kernel on the row-major tensors takes 7 us plus its base bytes at
// 6.2 TB/s plus the sign bytes of its job slots (4, 8 or 16: at least 4 are multiplied) at 3.1 TB/s (7B shapes,
// 1 to 16 tenants: 20 to 35 us per launch); the vector-ALU kernel streams everything at 1.3 TB/s plus 8 us.  A wrong guess costs time, never correctness.
bool prefill_gemm_pays(const int32_t* tenant_of_token, int64_t T, int64_t out, int64_t in, int32_t n_tenants, bool big,
                       bool decode_on_matrix_cores) {
    std::vector<int32_t> count((size_t)n_tenants, 0);
    for (int64_t i = 0; i < T; ++i) ++count[(size_t)tenant_of_token[i]];
    int64_t n_mtiles = 0;
    for (int32_t t = 0; t < n_tenants; ++t) n_mtiles += (count[(size_t)t] + bd::kPrefillTile - 1) / bd::kPrefillTile;
    int cus = 256;
    if (bd::device_cu_count(&cus) != hipSuccess || cus < 1) cus = 256;
    const double steps = (double)in / 64.0;
    double gemm_us;
    if (big) {
        const int64_t tiles = n_mtiles * ((out + 255) / 256);
        gemm_us = (double)((tiles + cus - 1) / cus) * (steps * 1.45 + 10.0);
    } else {   // 128 x 128 tiles, two workgroups per compute unit
        const int64_t tiles = n_mtiles * ((out + 127) / 128);
        gemm_us = (double)((tiles + 2 * cus - 1) / (2 * cus)) * (steps * 1.9 + 10.0);
    }
    double decode_us = 0.0;
    std::vector<int32_t> seen((size_t)n_tenants, -1);
    for (int64_t t0 = 0, chunk = 0; t0 < T; t0 += kMaxDecodeTokens, ++chunk) {
        const int64_t n = std::min<int64_t>(kMaxDecodeTokens, T - t0);
        int distinct = 0;
        for (int64_t i = t0; i < t0 + n; ++i) {
            int32_t& s = seen[(size_t)tenant_of_token[i]];
            if (s != (int32_t)chunk) {
                s = (int32_t)chunk;
                ++distinct;
            }
        }
        const double elems = (double)out * (double)in;
        decode_us += decode_on_matrix_cores ? 7.0 + 2.0 * elems / 6.2e6 + (double)std::max(distinct, 4) * elems / 8.0 / 3.1e6
                                            : 8.0 + elems * (2.0 + (double)distinct / 8.0) / 1.3e6;
    }
    return gemm_us < decode_us;
}

}  // namespace

extern "C" {

const char* bd_status_string(bd_status s) {
    switch (s) {
        case BD_OK: return "ok";
        case BD_ERR_NULL: return "a required pointer is NULL";
        case BD_ERR_SHAPE: return "bad shape: negative, too large, or in not a multiple of 32";
        case BD_ERR_ALIGN: return "a tensor pointer is not 16-byte aligned";
        case BD_ERR_TENANT: return "tenant id outside [0, n_tenants)";
        case BD_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
        case BD_ERR_DEVICE: return "the HIP runtime reported an error";
        case BD_ERR_UNSUPPORTED: return "unsupported op or kernel variant for these sizes";
        case BD_ERR_ALIAS: return "the output overlaps an input";
        case BD_ERR_FORMAT: return "malformed delta image";
        case BD_ERR_IO: return "file could not be opened, read or written";
        case BD_ERR_TOO_LARGE: return "size beyond the fixed limit of this entry point";
    }
    return "unknown status";
}

int bd_version(void) { return kVersion; }

size_t bd_workspace_bytes(bd_op op, int64_t T, int64_t out, int64_t in, int32_t n_tenants) {
    if (out < 0 || in < 0 || in % 32 != 0) return 0;
    switch (op) {
        case BD_OP_COMPRESS: return (size_t)bd::kCompressMaxBlocks * sizeof(double);
        case BD_OP_PACK_SIGNS: return 0;
        case BD_OP_LINEAR_MULTITENANT: return prefill_workspace_bytes(T, n_tenants);
        case BD_OP_LINEAR_GEMM: return prefill_table_bytes(T, n_tenants);
        case BD_OP_LINEAR_TILED_GEMM: return tiled_gemm_workspace_bytes(T, n_tenants);
    }
    return 0;
}

bd_status bd_pack_signs(const uint16_t* delta_f16, int64_t out, int64_t in, uint32_t* packed, void* stream) {
    if (out < 0 || in < 0 || in % 32 != 0) return BD_ERR_SHAPE;
    if (out == 0 || in == 0) return BD_OK;
    if (!delta_f16 || !packed) return BD_ERR_NULL;
    if (misaligned(delta_f16, 16) || misaligned(packed, 16)) return BD_ERR_ALIGN;
    if (overlaps(packed, (size_t)out * in / 8, delta_f16, (size_t)out * in * 2)) return BD_ERR_ALIAS;
    return bd::launch_pack_signs(delta_f16, out, in, packed, (hipStream_t)stream) == hipSuccess ? BD_OK : BD_ERR_DEVICE;
}

bd_status bd_compress(const uint16_t* w_base_f16, const uint16_t* w_ft_f16, int64_t out, int64_t in, uint32_t* packed,
                      float* alpha, void* workspace, size_t workspace_bytes, void* stream) {
    if (out < 0 || in < 0 || in % 32 != 0) return BD_ERR_SHAPE;
    if (!alpha) return BD_ERR_NULL;
    if (misaligned(alpha, 4)) return BD_ERR_ALIGN;
    const bool empty = (out == 0 || in == 0);
    if (!empty) {
        if (!w_base_f16 || !w_ft_f16 || !packed) return BD_ERR_NULL;
        if (misaligned(w_base_f16, 16) || misaligned(w_ft_f16, 16) || misaligned(packed, 16)) return BD_ERR_ALIGN;
        const size_t wbytes = (size_t)out * in * 2, pbytes = (size_t)out * in / 8;
        if (overlaps(packed, pbytes, w_base_f16, wbytes) || overlaps(packed, pbytes, w_ft_f16, wbytes)) return BD_ERR_ALIAS;
    }
    const size_t need = bd_workspace_bytes(BD_OP_COMPRESS, 0, out, in, 1);
    if (!workspace || workspace_bytes < need || misaligned(workspace, 256)) return BD_ERR_WORKSPACE;
    return bd::launch_compress(w_base_f16, w_ft_f16, out, in, packed, alpha, (double*)workspace,
                               (hipStream_t)stream) == hipSuccess
               ? BD_OK
               : BD_ERR_DEVICE;
}

bd_status bd_compress_noalloc(const uint16_t* w_base_f16, const uint16_t* w_ft_f16, int64_t out, int64_t in,
                              uint32_t* packed, float* alpha, void* stream) {
    if (out < 0 || in < 0 || in % 32 != 0) return BD_ERR_SHAPE;
    if (!alpha) return BD_ERR_NULL;
    if (misaligned(alpha, 4)) return BD_ERR_ALIGN;
    // the size limit of this entry point, checked without overflow (out, in >= 0 here)
    if (out > 0 && in > BD_COMPRESS_NOALLOC_MAX_ELEMENTS / out) return BD_ERR_TOO_LARGE;
    if (out > 0 && in > 0) {
        if (!w_base_f16 || !w_ft_f16 || !packed) return BD_ERR_NULL;
        if (misaligned(w_base_f16, 16) || misaligned(w_ft_f16, 16) || misaligned(packed, 16)) return BD_ERR_ALIGN;
        const size_t wbytes = (size_t)out * in * 2, pbytes = (size_t)out * in / 8;
        if (overlaps(packed, pbytes, w_base_f16, wbytes) || overlaps(packed, pbytes, w_ft_f16, wbytes)) return BD_ERR_ALIAS;
    }
    return bd::launch_compress_noalloc(w_base_f16, w_ft_f16, out, in, packed, alpha, (hipStream_t)stream) == hipSuccess
               ? BD_OK
               : BD_ERR_DEVICE;
}

bd_status bd_compress_batch(int32_t n, const uint16_t* const* w_base_f16, const uint16_t* const* w_ft_f16,
                            const int64_t* out, const int64_t* in, uint32_t* const* packed, float* alpha, void* workspace,
                            size_t workspace_bytes, void* stream) {
    if (n < 0) return BD_ERR_SHAPE;
    if (n == 0) return BD_OK;
    if (!w_base_f16 || !w_ft_f16 || !out || !in || !packed || !alpha) return BD_ERR_NULL;
    if (misaligned(alpha, 4)) return BD_ERR_ALIGN;
    for (int32_t m = 0; m < n; ++m) {
        if (out[m] < 0 || in[m] < 0 || in[m] % 32 != 0) return BD_ERR_SHAPE;
        if (out[m] == 0 || in[m] == 0) continue;
        if (!w_base_f16[m] || !w_ft_f16[m] || !packed[m]) return BD_ERR_NULL;
        if (misaligned(w_base_f16[m], 16) || misaligned(w_ft_f16[m], 16) || misaligned(packed[m], 16)) return BD_ERR_ALIGN;
        const size_t wbytes = (size_t)out[m] * in[m] * 2, pbytes = (size_t)out[m] * in[m] / 8;
        for (int32_t o = 0; o < n; ++o) {   // no plane of signs may lie over any matrix that is still to be read
            if (out[o] == 0 || in[o] == 0) continue;
            const size_t obytes = (size_t)out[o] * in[o] * 2;
            if (overlaps(packed[m], pbytes, w_base_f16[o], obytes) || overlaps(packed[m], pbytes, w_ft_f16[o], obytes))
                return BD_ERR_ALIAS;
            if (o != m && overlaps(packed[m], pbytes, packed[o], (size_t)out[o] * in[o] / 8)) return BD_ERR_ALIAS;
        }
        (void)wbytes;
    }
    const size_t need = (size_t)BD_COMPRESS_BATCH_MAX * bd_workspace_bytes(BD_OP_COMPRESS, 0, 1, 32, 1);
    if (!workspace || workspace_bytes < need || misaligned(workspace, 256)) return BD_ERR_WORKSPACE;
    for (int32_t m0 = 0; m0 < n; m0 += bd::kCompressBatchMax) {   // launches of up to 8 matrices, in stream order
        bd::CompressBatch a;
        std::memset(&a, 0, sizeof(a));
        a.n = std::min<int32_t>(bd::kCompressBatchMax, n - m0);
        for (int i = 0; i < a.n; ++i) {
            const int32_t m = m0 + i;
            a.base[i] = w_base_f16[m];
            a.ft[i] = w_ft_f16[m];
            a.packed[i] = packed[m];
            a.n_vec[i] = out[m] * in[m] / 8;
        }
        if (bd::launch_compress_batch(a, alpha + m0, (double*)workspace, (hipStream_t)stream) != hipSuccess) return BD_ERR_DEVICE;
    }
    return BD_OK;
}

bd_status bd_compress_iterated(const uint16_t* w_base_f16, const uint16_t* w_ft_f16, int64_t out, int64_t in, int32_t k,
                               uint32_t* packed, float* alpha, void* workspace, size_t workspace_bytes, void* stream) {
    if (out < 0 || in < 0 || in % 32 != 0 || k < 1 || k > bd::kCompressMaxPlanes) return BD_ERR_SHAPE;
    if (!alpha) return BD_ERR_NULL;
    if (misaligned(alpha, 4)) return BD_ERR_ALIGN;
    const bool empty = (out == 0 || in == 0);
    const size_t plane_words = (size_t)out * in / 32;
    if (!empty) {
        if (!w_base_f16 || !w_ft_f16 || !packed) return BD_ERR_NULL;
        if (misaligned(w_base_f16, 16) || misaligned(w_ft_f16, 16) || misaligned(packed, 16)) return BD_ERR_ALIGN;
        const size_t wbytes = (size_t)out * in * 2, pbytes = plane_words * 4 * (size_t)k;
        if (overlaps(packed, pbytes, w_base_f16, wbytes) || overlaps(packed, pbytes, w_ft_f16, wbytes)) return BD_ERR_ALIAS;
    }
    const size_t need = bd_workspace_bytes(BD_OP_COMPRESS, 0, out, in, 1);
    if (!workspace || workspace_bytes < need || misaligned(workspace, 256)) return BD_ERR_WORKSPACE;
    // iteration j reads the scales 0 .. j-1 that the iterations before it left in `alpha` (same stream)
    for (int j = 0; j < k; ++j)
        if (bd::launch_compress(w_base_f16, w_ft_f16, out, in, packed + (size_t)j * plane_words, alpha + j, (double*)workspace,
                                (hipStream_t)stream, alpha, j) != hipSuccess)
            return BD_ERR_DEVICE;
    return BD_OK;
}

namespace {
bd_status tiled_linear_impl(int32_t n_mats, const uint16_t* x_f16, const uint16_t* const* w_tiled,
                            const uint32_t* const* tiled_by_mat_tenant, const float* const* alpha_by_mat,
                            const int32_t* tenant_of_token, uint16_t* const* y_f16, int64_t T, const int64_t* out,
                            int64_t in, int32_t n_tenants, int32_t k, void* stream, bool q8,
                            const uint32_t* const* packed_rowmajor_dev, const float* wscale_rowmajor = nullptr);
}

bd_status bd_linear_multitenant_variant(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                        const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                        const int32_t* tenant_of_token, uint16_t* y_f16, int64_t T, int64_t out,
                                        int64_t in, int32_t n_tenants, void* workspace, size_t workspace_bytes,
                                        void* stream, int32_t variant) {
    const bd_status st = check_linear_args(x_f16, w_base_f16, packed_by_tenant, alpha_by_tenant, tenant_of_token, y_f16,
                                           T, out, in, n_tenants);
    if (st != BD_OK) return st;
    const bool merged_variant = variant == kVariantPrefillMerged;
    const bool big_variant = variant == kVariantPrefillBig || variant == kVariantPrefillBig8 || variant == kVariantPrefillBigWhole ||
                             merged_variant;
    const bool prefill_variant = variant == kVariantPrefillSmall || big_variant;
    if (variant != 0 && variant != kVariantRowWave && variant != kVariantRowMajorMfma && !prefill_variant)
        return BD_ERR_UNSUPPORTED;
    if (T == 0 || out == 0) return BD_OK;
    // 128-bit sign loads need whole, aligned 4-word groups; 32-bit lane offsets need tensors below 4 GiB
    const bool mfma_ok = (in % 128 == 0) && in > 0 && (uint64_t)out * (uint64_t)in * 2 < ((uint64_t)1 << 32) &&
                         (uint64_t)T * (uint64_t)in * 2 < ((uint64_t)1 << 32);
    if (variant >= 2 && !prefill_variant && !mfma_ok) return BD_ERR_UNSUPPORTED;
    int use = variant;
    if (use == 0) use = mfma_ok ? kVariantRowMajorMfma : kVariantRowWave;

    hipStream_t hs = (hipStream_t)stream;
    // More than one decode launch worth of tokens: the prefill GEMM, if the caller brought its workspace
    // (without one the call still works, as a sequence of decode launches that re-read the base).
    const size_t need = prefill_workspace_bytes(T, n_tenants);
    const bool can_prefill = need > 0 && in > 0 && workspace && workspace_bytes >= need && !misaligned(workspace, 256);
    if (prefill_variant && !can_prefill) return need > 0 && in > 0 ? BD_ERR_WORKSPACE : BD_ERR_UNSUPPORTED;
    if (big_variant && !bd::prefill_big_fits(T, out, in)) return BD_ERR_UNSUPPORTED;
    const bool big_default = out >= 256 && bd::prefill_big_fits(T, out, in);
    if (can_prefill &&
        (prefill_variant || (variant == 0 && prefill_gemm_pays(tenant_of_token, T, out, in, n_tenants, big_default, mfma_ok)))) {
        // the large tile (one workgroup per CU, 256 output features wide) pays off when there are at least that many
        int big_waves = 0;
        if (variant == kVariantPrefillBig8) big_waves = 8;
        if (variant == kVariantPrefillBig || variant == kVariantPrefillBigWhole || variant == kVariantPrefillMerged ||
            (variant == 0 && big_default))
            big_waves = 4;
        return run_prefill(x_f16, w_base_f16, packed_by_tenant, alpha_by_tenant, tenant_of_token, y_f16, T, out, in,
                           workspace, hs, big_waves, variant != kVariantPrefillBigWhole, 0, nullptr, merged_variant) == hipSuccess
                   ? BD_OK
                   : BD_ERR_DEVICE;
    }
    if (prefill_variant) use = mfma_ok ? kVariantRowMajorMfma : kVariantRowWave;   // not reached: can_prefill held above
    if (use == kVariantRowMajorMfma && in > 0)
        // the decode kernel of the serving path, reading the row-major tensors as they are; all tokens are grouped by
        // tenant first, then cut into launches of 32
        return tiled_linear_impl(1, x_f16, &w_base_f16, nullptr, &alpha_by_tenant, tenant_of_token, &y_f16, T, &out, in,
                                 n_tenants, 1, stream, false, packed_by_tenant);
    for (int64_t t0 = 0; t0 < T; t0 += kMaxDecodeTokens) {
        const int n = (int)std::min<int64_t>(kMaxDecodeTokens, T - t0);
        DecodeMeta meta;
        build_meta(tenant_of_token, t0, n, &meta);
        const uint16_t* xs = x_f16 + t0 * in;
        uint16_t* ys = y_f16 + t0 * out;
        hipError_t e;
        // the vector-ALU kernel; also the empty reduction, y = 0 (its loop body never runs)
        e = bd::launch_linear_rowwave(xs, w_base_f16, packed_by_tenant, alpha_by_tenant, meta, ys, out, in, hs);
        if (e != hipSuccess) return BD_ERR_DEVICE;
    }
    return BD_OK;
}

bd_status bd_linear_multitenant(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                const int32_t* tenant_of_token, uint16_t* y_f16, int64_t T, int64_t out, int64_t in,
                                int32_t n_tenants, void* workspace, size_t workspace_bytes, void* stream) {
    return bd_linear_multitenant_variant(x_f16, w_base_f16, packed_by_tenant, alpha_by_tenant, tenant_of_token, y_f16, T,
                                         out, in, n_tenants, workspace, workspace_bytes, stream, 0);
}

// ---- tiled serving layout ------------------------------------------------------------------

namespace {

bool tiled_shape_ok(int64_t out, int64_t in) {
    if (out < 0 || in < 0 || in % 32 != 0) return false;
    if (out > ((int64_t)1 << 31) - 16 || in > ((int64_t)1 << 31) - 256) return false;
    // 32-bit byte offsets inside one tiled tensor
    const uint64_t tiles = (uint64_t)bd::tiled_row_blocks(out) * (uint64_t)bd::tiled_k_tiles(in);
    return tiles * (uint64_t)bd::kTileBaseBytes < ((uint64_t)1 << 32);
}

}  // namespace

size_t bd_tiled_base_bytes(int64_t out, int64_t in) {
    if (!tiled_shape_ok(out, in)) return 0;
    return (size_t)(bd::tiled_row_blocks(out) * bd::tiled_k_tiles(in)) * bd::kTileBaseBytes;
}

size_t bd_tiled_signs_bytes(int64_t out, int64_t in) {
    if (!tiled_shape_ok(out, in)) return 0;
    return (size_t)(bd::tiled_row_blocks(out) * bd::tiled_k_tiles(in)) * bd::kTileSignBytes;
}

bd_status bd_tile_base(const uint16_t* w_f16, int64_t out, int64_t in, uint16_t* w_tiled, void* stream) {
    if (!tiled_shape_ok(out, in)) return BD_ERR_SHAPE;
    if (out == 0 || in == 0) return BD_OK;
    if (!w_f16 || !w_tiled) return BD_ERR_NULL;
    if (misaligned(w_f16, 16) || misaligned(w_tiled, 16)) return BD_ERR_ALIGN;
    if (overlaps(w_tiled, bd_tiled_base_bytes(out, in), w_f16, (size_t)out * in * 2)) return BD_ERR_ALIAS;
    return bd::launch_tile_base(w_f16, out, in, w_tiled, (hipStream_t)stream) == hipSuccess ? BD_OK : BD_ERR_DEVICE;
}

bd_status bd_tile_signs(const uint32_t* packed, int64_t out, int64_t in, uint32_t* signs_tiled, void* stream) {
    if (!tiled_shape_ok(out, in)) return BD_ERR_SHAPE;
    if (out == 0 || in == 0) return BD_OK;
    if (!packed || !signs_tiled) return BD_ERR_NULL;
    if (misaligned(packed, 16) || misaligned(signs_tiled, 16)) return BD_ERR_ALIGN;
    if (overlaps(signs_tiled, bd_tiled_signs_bytes(out, in), packed, (size_t)out * in / 8)) return BD_ERR_ALIAS;
    return bd::launch_tile_signs(packed, out, in, signs_tiled, (hipStream_t)stream) == hipSuccess ? BD_OK : BD_ERR_DEVICE;
}

namespace {

// The tiled linear over n_mats matrices that share x, with k sign planes per tenant (k = 1: plain 1-bit
// deltas).  Pointer table index: (m * n_tenants + tenant) * k + plane; scale index: tenant * k + plane.
// q8: w_tiled point at 8-bit base tiles followed by their per-row scales (bd_tile_base_q8).
// packed_rowmajor_dev != NULL: the row-major entry point.  w_tiled[0] is then W [out, in] row-major, the deltas are
// reached through that DEVICE table of n_tenants pointers (tiled_by_mat_tenant is not used), n_mats = k = 1.
bd_status tiled_linear_impl(int32_t n_mats, const uint16_t* x_f16, const uint16_t* const* w_tiled,
                            const uint32_t* const* tiled_by_mat_tenant, const float* const* alpha_by_mat,
                            const int32_t* tenant_of_token, uint16_t* const* y_f16, int64_t T, const int64_t* out,
                            int64_t in, int32_t n_tenants, int32_t k, void* stream, bool q8,
                            const uint32_t* const* packed_rowmajor_dev, const float* wscale_rowmajor) {
    const bool rm = packed_rowmajor_dev != nullptr;
    if (rm && (n_mats != 1 || in % 128 != 0 || (q8 && (!wscale_rowmajor || k != 1)))) return BD_ERR_UNSUPPORTED;
    if (n_mats < 1 || n_mats > bd::kTiledMaxMats) return BD_ERR_SHAPE;
    if (k < 1 || k > bd::kTiledMaxPlanes) return BD_ERR_SHAPE;
    if (!out) return BD_ERR_NULL;
    if (T < 0 || n_tenants < 0 || T > 65535) return BD_ERR_SHAPE;
    int64_t row_blocks = 0;
    for (int m = 0; m < n_mats; ++m) {
        if (!tiled_shape_ok(out[m], in)) return BD_ERR_SHAPE;
        row_blocks += bd::tiled_row_blocks(out[m]);
    }
    if (row_blocks > 0x7fffffff) return BD_ERR_SHAPE;
    if ((uint64_t)T * (uint64_t)in * 2 >= ((uint64_t)1 << 32)) return BD_ERR_SHAPE;   // 32-bit byte offsets into x
    if (T == 0 || row_blocks == 0) return BD_OK;
    if (in == 0) {   // empty reduction: y = 0, nothing else is read
        if (!y_f16) return BD_ERR_NULL;
        for (int m = 0; m < n_mats; ++m)
            if (out[m] > 0 && !y_f16[m]) return BD_ERR_NULL;
        for (int m = 0; m < n_mats; ++m)
            if (out[m] > 0 && bd::launch_fill_zero_u16(y_f16[m], T * out[m], (hipStream_t)stream) != hipSuccess) return BD_ERR_DEVICE;
        return BD_OK;
    }
    if (!x_f16 || !w_tiled || (!rm && !tiled_by_mat_tenant) || !alpha_by_mat || !tenant_of_token || !y_f16) return BD_ERR_NULL;
    if (misaligned(x_f16, 16)) return BD_ERR_ALIGN;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return BD_ERR_TENANT;
    for (int m = 0; m < n_mats; ++m) {
        if (out[m] == 0) continue;
        if (!w_tiled[m] || !alpha_by_mat[m] || !y_f16[m]) return BD_ERR_NULL;
        if (misaligned(w_tiled[m], 16) || misaligned(y_f16[m], 2) || misaligned(alpha_by_mat[m], 4)) return BD_ERR_ALIGN;
        const size_t ybytes = (size_t)T * out[m] * 2;
        const size_t wbytes = rm ? (size_t)out[m] * in * (q8 ? 1 : 2) : (q8 ? bd_tiled_base_q8_bytes(out[m], in) : bd_tiled_base_bytes(out[m], in));
        if (overlaps(y_f16[m], ybytes, x_f16, (size_t)T * in * 2) || overlaps(y_f16[m], ybytes, w_tiled[m], wbytes))
            return BD_ERR_ALIAS;
        for (int64_t t = 0; t < T && !rm; ++t)
            for (int j = 0; j < k; ++j) {
                const uint32_t* p = tiled_by_mat_tenant[((size_t)m * n_tenants + tenant_of_token[t]) * k + j];
                if (!p) return BD_ERR_NULL;
                if (misaligned(p, 16)) return BD_ERR_ALIGN;
            }
    }
    // A token takes k columns (one per plane) of a 16-column tile; a launch covers two tiles.  More tokens than one
    // launch takes: all of them are sorted by tenant first (stable), so that a tenant's tokens share launches and
    // its delta is streamed as few times as possible; the kernel finds the rows of x and y through the token ids.
    const int per_tile = bd::kTiledMaxTokens / k;
    const int per_launch = per_tile * bd::kTiledMaxCt;
    std::vector<int32_t> order((size_t)T);
    for (int64_t i = 0; i < T; ++i) order[(size_t)i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(), [&](int32_t p, int32_t q) { return tenant_of_token[p] < tenant_of_token[q]; });
    for (int64_t t0 = 0; t0 < T; t0 += per_launch) {
        const int n = (int)std::min<int64_t>(per_launch, T - t0);
        bd::TiledArgs a;
        std::memset(&a, 0, sizeof(a));
        a.x = x_f16;
        a.in = (int32_t)in;
        a.KT = (int32_t)bd::tiled_k_tiles(in);
        a.n_ct = n > per_tile ? 2 : 1;
        a.planes = k;
        a.packed_by_tenant = packed_rowmajor_dev;
        int32_t rb = 0;
        int mats = 0;
        int mat_of[bd::kTiledMaxMats] = {0, 0, 0};
        for (int m = 0; m < n_mats; ++m) {
            if (out[m] == 0) continue;
            a.wt[mats] = w_tiled[m];
            a.y[mats] = y_f16[m];
            a.alpha[mats] = alpha_by_mat[m];
            if (q8 && rm)
                a.wscale[mats] = wscale_rowmajor;
            else if (q8)   // the scales follow the tiles
                a.wscale[mats] = (const float*)((const unsigned char*)w_tiled[m] +
                                                (size_t)(bd::tiled_row_blocks(out[m]) * bd::tiled_k_tiles(in)) * bd::kTileBaseQ8Bytes);
            a.out[mats] = (int32_t)out[m];
            rb += (int32_t)bd::tiled_row_blocks(out[m]);
            a.rb_end[mats] = rb;
            mat_of[mats] = m;
            ++mats;
        }
        a.n_mats = mats;
        int max_jobs = 1;
        for (int ct = 0; ct < bd::kTiledMaxCt; ++ct) {
            // a column tile beyond n_ct mirrors tile 0 (never read by the kernel, but every pointer stays valid)
            const int src = ct < a.n_ct ? ct : 0;
            const int tok_begin = src * per_tile, tok_end = std::min(n, tok_begin + per_tile);
            int n_runs = 0, run_tenant[bd::kTiledMaxTokens];
            int col = 0;
            for (int i = tok_begin; i < tok_end; ++i) {
                const int tok = order[(size_t)(t0 + i)];
                const int tenant = tenant_of_token[tok];
                if (n_runs == 0 || run_tenant[n_runs - 1] != tenant) run_tenant[n_runs++] = tenant;
                for (int j = 0; j < k; ++j, ++col) {   // the token's columns: plane j is job slot (run, j)
                    a.col_token[ct][col] = tok;
                    a.col_tenant[ct][col] = tenant * k + j;
                    a.col_job[ct][col] = (n_runs - 1) * k + j;
                    a.col_span[ct][col] = j == 0 ? k : 0;
                }
            }
            a.T[ct] = col;
            for (; col < bd::kTiledMaxTokens; ++col) a.col_job[ct][col] = -1;
            const int n_jobs = n_runs * k;
            max_jobs = std::max(max_jobs, n_jobs);
            for (int sl = 0; sl < bd::kTiledMaxJobs; ++sl) {   // slots beyond the jobs repeat slot 0 (never selected)
                const int s = sl < n_jobs ? sl : 0;
                a.job_tenant[ct][sl] = run_tenant[s / k] * k + s % k;   // index into the caller's table: (tenant, plane)
                for (int mi = 0; mi < mats && !rm; ++mi)
                    a.signs[ct][mi][sl] = tiled_by_mat_tenant[((size_t)mat_of[mi] * n_tenants + run_tenant[s / k]) * k + s % k];
            }
        }
        const hipError_t e = rm   ? (q8 ? bd::launch_linear_decode_rowmajor_q8(a, max_jobs, (hipStream_t)stream)
                                        : bd::launch_linear_decode_rowmajor(a, max_jobs, (hipStream_t)stream))
                             : q8 ? bd::launch_linear_decode_tiled_q8(a, max_jobs, (hipStream_t)stream)
                                  : bd::launch_linear_decode_tiled(a, max_jobs, (hipStream_t)stream);
        if (e != hipSuccess) return BD_ERR_DEVICE;
    }
    return BD_OK;
}

}  // namespace

// ---- 8-bit round-to-nearest base ----

size_t bd_tiled_base_q8_bytes(int64_t out, int64_t in) {
    if (!tiled_shape_ok(out, in)) return 0;
    const size_t RB = (size_t)bd::tiled_row_blocks(out), KT = (size_t)bd::tiled_k_tiles(in);
    return RB * KT * bd::kTileBaseQ8Bytes + RB * bd::kTileRows * sizeof(float);
}

bd_status bd_quantize_base_q8(const uint16_t* w_f16, int64_t out, int64_t in, int8_t* q, float* scale, void* stream) {
    if (out < 0 || in < 0 || out > ((int64_t)1 << 31) - 1) return BD_ERR_SHAPE;
    if (out == 0) return BD_OK;
    if (!scale || (in > 0 && (!w_f16 || !q))) return BD_ERR_NULL;
    if (misaligned(w_f16, 2) || misaligned(scale, 4)) return BD_ERR_ALIGN;
    if (in > 0 && overlaps(q, (size_t)out * in, w_f16, (size_t)out * in * 2)) return BD_ERR_ALIAS;
    return bd::launch_quantize_rtn8(w_f16, out, in, q, scale, (hipStream_t)stream) == hipSuccess ? BD_OK : BD_ERR_DEVICE;
}

bd_status bd_tile_base_q8(const int8_t* q, const float* scale, int64_t out, int64_t in, void* wq_tiled, void* stream) {
    if (!tiled_shape_ok(out, in)) return BD_ERR_SHAPE;
    if (out == 0) return BD_OK;
    if (!scale || !wq_tiled || (in > 0 && !q)) return BD_ERR_NULL;
    if (misaligned(wq_tiled, 16) || misaligned(scale, 4)) return BD_ERR_ALIGN;
    const size_t bytes = bd_tiled_base_q8_bytes(out, in);
    if (overlaps(wq_tiled, bytes, q, (size_t)out * in) || overlaps(wq_tiled, bytes, scale, (size_t)out * 4)) return BD_ERR_ALIAS;
    return bd::launch_tile_base_q8(q, scale, out, in, (unsigned char*)wq_tiled, (hipStream_t)stream) == hipSuccess ? BD_OK
                                                                                                                  : BD_ERR_DEVICE;
}

bd_status bd_compress_q8(const int8_t* q, const float* scale, const uint16_t* w_ft_f16, int64_t out, int64_t in,
                         uint32_t* packed, float* alpha, void* workspace, size_t workspace_bytes, void* stream) {
    if (out < 0 || in < 0 || in % 32 != 0) return BD_ERR_SHAPE;
    if (!alpha) return BD_ERR_NULL;
    if (misaligned(alpha, 4)) return BD_ERR_ALIGN;
    if (out > 0 && in > 0) {
        if (!q || !scale || !w_ft_f16 || !packed) return BD_ERR_NULL;
        if (misaligned(q, 8) || misaligned(scale, 4) || misaligned(w_ft_f16, 16) || misaligned(packed, 16)) return BD_ERR_ALIGN;
        const size_t pbytes = (size_t)out * in / 8;
        if (overlaps(packed, pbytes, q, (size_t)out * in) || overlaps(packed, pbytes, w_ft_f16, (size_t)out * in * 2) ||
            overlaps(packed, pbytes, scale, (size_t)out * 4))
            return BD_ERR_ALIAS;
    }
    const size_t need = bd_workspace_bytes(BD_OP_COMPRESS, 0, out, in, 1);
    if (!workspace || workspace_bytes < need || misaligned(workspace, 256)) return BD_ERR_WORKSPACE;
    return bd::launch_compress_q8(q, scale, w_ft_f16, out, in, packed, alpha, (double*)workspace, (hipStream_t)stream) ==
                   hipSuccess
               ? BD_OK
               : BD_ERR_DEVICE;
}

bd_status bd_linear_multitenant_tiled_group_q8(int32_t n_mats, const uint16_t* x_f16, const void* const* wq_tiled,
                                               const uint32_t* const* tiled_by_mat_tenant,
                                               const float* const* alpha_by_mat, const int32_t* tenant_of_token,
                                               uint16_t* const* y_f16, int64_t T, const int64_t* out, int64_t in,
                                               int32_t n_tenants, void* stream) {
    return tiled_linear_impl(n_mats, x_f16, (const uint16_t* const*)wq_tiled, tiled_by_mat_tenant, alpha_by_mat, tenant_of_token,
                             y_f16, T, out, in, n_tenants, 1, stream, true, nullptr);
}

bd_status bd_linear_multitenant_tiled_q8(const uint16_t* x_f16, const void* wq_tiled, const uint32_t* const* tiled_by_tenant,
                                         const float* alpha_by_tenant, const int32_t* tenant_of_token, uint16_t* y_f16,
                                         int64_t T, int64_t out, int64_t in, int32_t n_tenants, void* stream) {
    const uint16_t* w = (const uint16_t*)wq_tiled;
    return tiled_linear_impl(1, x_f16, &w, tiled_by_tenant, &alpha_by_tenant, tenant_of_token, &y_f16, T, &out, in, n_tenants, 1,
                             stream, true, nullptr);
}

bd_status bd_linear_multitenant_tiled_group(int32_t n_mats, const uint16_t* x_f16, const uint16_t* const* w_tiled,
                                            const uint32_t* const* tiled_by_mat_tenant,
                                            const float* const* alpha_by_mat, const int32_t* tenant_of_token,
                                            uint16_t* const* y_f16, int64_t T, const int64_t* out, int64_t in,
                                            int32_t n_tenants, void* stream) {
    return tiled_linear_impl(n_mats, x_f16, w_tiled, tiled_by_mat_tenant, alpha_by_mat, tenant_of_token, y_f16, T, out, in,
                             n_tenants, 1, stream, false, nullptr);
}

bd_status bd_linear_multitenant_tiled(const uint16_t* x_f16, const uint16_t* w_tiled,
                                      const uint32_t* const* tiled_by_tenant, const float* alpha_by_tenant,
                                      const int32_t* tenant_of_token, uint16_t* y_f16, int64_t T, int64_t out, int64_t in,
                                      int32_t n_tenants, void* stream) {
    return tiled_linear_impl(1, x_f16, &w_tiled, tiled_by_tenant, &alpha_by_tenant, tenant_of_token, &y_f16, T, &out, in,
                             n_tenants, 1, stream, false, nullptr);
}

bd_status bd_linear_multitenant_tiled_gemm(const uint16_t* x_f16, const uint16_t* w_tiled, const uint32_t* const* tiled_by_tenant,
                                           const float* alpha_by_tenant, const int32_t* tenant_of_token, uint16_t* y_f16,
                                           int64_t T, int64_t out, int64_t in, int32_t n_tenants, int32_t one_product,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    if (T < 0 || n_tenants < 0 || T > 65535 || !tiled_shape_ok(out, in)) return BD_ERR_SHAPE;
    if ((uint64_t)T * (uint64_t)in * 2 >= ((uint64_t)1 << 32)) return BD_ERR_SHAPE;   // 32-bit byte offsets into x
    if (T == 0 || out == 0) return BD_OK;
    if (!x_f16 || !w_tiled || !tiled_by_tenant || !alpha_by_tenant || !tenant_of_token || !y_f16) return BD_ERR_NULL;
    if (misaligned(x_f16, 16) || misaligned(w_tiled, 16) || misaligned(y_f16, 2) || misaligned(alpha_by_tenant, 4)) return BD_ERR_ALIGN;
    for (int64_t t = 0; t < T; ++t) {
        const int32_t e = tenant_of_token[t];
        if (e < 0 || e >= n_tenants) return BD_ERR_TENANT;
        if (!tiled_by_tenant[e]) return BD_ERR_NULL;          // a tenant with a token needs its delta
        if (misaligned(tiled_by_tenant[e], 16)) return BD_ERR_ALIGN;
    }
    const size_t ybytes = (size_t)T * (size_t)out * 2;
    if (overlaps(y_f16, ybytes, x_f16, (size_t)T * (size_t)in * 2) || overlaps(y_f16, ybytes, w_tiled, bd_tiled_base_bytes(out, in)))
        return BD_ERR_ALIAS;
    if (in == 0 || !bd::prefill_big_fits(T, out, in)) return BD_ERR_UNSUPPORTED;   // whole k steps of 64
    const size_t need = tiled_gemm_workspace_bytes(T, n_tenants);
    if (!workspace || workspace_bytes < need || misaligned(workspace, 256)) return BD_ERR_WORKSPACE;
    return run_prefill(x_f16, w_tiled, nullptr, alpha_by_tenant, tenant_of_token, y_f16, T, out, in, workspace, (hipStream_t)stream, 4,
                       true, 0, nullptr, one_product != 0, tiled_by_tenant, n_tenants) == hipSuccess
               ? BD_OK
               : BD_ERR_DEVICE;
}

bd_status bd_linear_multitenant_tiled_group_kbit(int32_t n_mats, const uint16_t* x_f16, const uint16_t* const* w_tiled,
                                                 const uint32_t* const* planes_by_mat_tenant,
                                                 const float* const* alpha_by_mat, const int32_t* tenant_of_token,
                                                 uint16_t* const* y_f16, int64_t T, const int64_t* out, int64_t in,
                                                 int32_t n_tenants, int32_t k, void* stream) {
    return tiled_linear_impl(n_mats, x_f16, w_tiled, planes_by_mat_tenant, alpha_by_mat, tenant_of_token, y_f16, T, out, in,
                             n_tenants, k, stream, false, nullptr);
}

bd_status bd_linear_multitenant_kbit(const uint16_t* x_f16, const uint16_t* w_base_f16, const uint32_t* const* planes_by_tenant,
                                     const float* alpha_by_tenant, const int32_t* tenant_of_token, uint16_t* y_f16, int64_t T,
                                     int64_t out, int64_t in, int32_t n_tenants, int32_t k, void* stream) {
    if (k < 1 || k > bd::kTiledMaxPlanes) return BD_ERR_SHAPE;
    const bd_status st = check_linear_args(x_f16, w_base_f16, planes_by_tenant, alpha_by_tenant, tenant_of_token, y_f16, T, out, in,
                                           n_tenants);
    if (st != BD_OK) return st;
    if (T == 0 || out == 0) return BD_OK;
    // the matrix-core kernel on the row-major tensors: whole groups of four sign words, 32-bit byte offsets
    if (in % 128 != 0 || in == 0 || (uint64_t)out * (uint64_t)in * 2 >= ((uint64_t)1 << 32)) return BD_ERR_UNSUPPORTED;
    return tiled_linear_impl(1, x_f16, &w_base_f16, nullptr, &alpha_by_tenant, tenant_of_token, &y_f16, T, &out, in, n_tenants, k,
                             stream, false, planes_by_tenant);
}

// The GEMM form for any T >= 1 with k planes per tenant or the 8-bit base (128 x 128 tiles).
static bd_status gemm_entry(const uint16_t* x_f16, const void* w, size_t w_bytes_per_el, const uint32_t* const* packed_by_tenant,
                            const float* alpha_by_tenant, const float* wscale, const int32_t* tenant_of_token, uint16_t* y_f16,
                            int64_t T, int64_t out, int64_t in, int32_t n_tenants, int k_planes, void* workspace,
                            size_t workspace_bytes, void* stream) {
    const bd_status st = check_linear_args(x_f16, w, packed_by_tenant, alpha_by_tenant, tenant_of_token, y_f16, T, out, in,
                                           n_tenants, w_bytes_per_el);
    if (st != BD_OK) return st;
    if (T == 0 || out == 0) return BD_OK;
    if (in == 0) return BD_ERR_UNSUPPORTED;   // the empty reduction (y = 0) is bd_linear_multitenant's
    const size_t need = prefill_table_bytes(T, n_tenants);
    if (!workspace || workspace_bytes < need || misaligned(workspace, 256)) return BD_ERR_WORKSPACE;
    return run_prefill(x_f16, w, packed_by_tenant, alpha_by_tenant, tenant_of_token, y_f16, T, out, in, workspace,
                       (hipStream_t)stream, 0, false, k_planes, wscale) == hipSuccess
               ? BD_OK
               : BD_ERR_DEVICE;
}

bd_status bd_linear_multitenant_gemm_kbit(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                          const uint32_t* const* planes_by_tenant, const float* alpha_by_tenant,
                                          const int32_t* tenant_of_token, uint16_t* y_f16, int64_t T, int64_t out, int64_t in,
                                          int32_t n_tenants, int32_t k, void* workspace, size_t workspace_bytes, void* stream) {
    if (k < 1 || k > bd::kTiledMaxPlanes) return BD_ERR_SHAPE;
    return gemm_entry(x_f16, w_base_f16, 2, planes_by_tenant, alpha_by_tenant, nullptr, tenant_of_token, y_f16, T, out, in,
                      n_tenants, k, workspace, workspace_bytes, stream);
}

bd_status bd_linear_multitenant_gemm_q8(const uint16_t* x_f16, const int8_t* q, const float* wscale,
                                        const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                        const int32_t* tenant_of_token, uint16_t* y_f16, int64_t T, int64_t out, int64_t in,
                                        int32_t n_tenants, void* workspace, size_t workspace_bytes, void* stream) {
    if (T > 0 && out > 0 && !wscale) return BD_ERR_NULL;
    if (misaligned(wscale, 4)) return BD_ERR_ALIGN;
    return gemm_entry(x_f16, q, 1, packed_by_tenant, alpha_by_tenant, wscale, tenant_of_token, y_f16, T, out, in, n_tenants, 0,
                      workspace, workspace_bytes, stream);
}

bd_status bd_linear_multitenant_q8(const uint16_t* x_f16, const int8_t* q, const float* wscale,
                                   const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                   const int32_t* tenant_of_token, uint16_t* y_f16, int64_t T, int64_t out, int64_t in,
                                   int32_t n_tenants, void* stream) {
    const bd_status st = check_linear_args(x_f16, q, packed_by_tenant, alpha_by_tenant, tenant_of_token, y_f16, T, out, in,
                                           n_tenants, 1);
    if (st != BD_OK) return st;
    if (T == 0 || out == 0) return BD_OK;
    if (!wscale) return BD_ERR_NULL;
    if (misaligned(wscale, 4)) return BD_ERR_ALIGN;
    // the matrix-core kernel on the row-major tensors: whole groups of four sign words, 32-bit byte offsets
    if (in % 128 != 0 || in == 0 || (uint64_t)out * (uint64_t)in >= ((uint64_t)1 << 32)) return BD_ERR_UNSUPPORTED;
    const uint16_t* w = (const uint16_t*)q;
    return tiled_linear_impl(1, x_f16, &w, nullptr, &alpha_by_tenant, tenant_of_token, &y_f16, T, &out, in, n_tenants, 1, stream,
                             true, packed_by_tenant, wscale);
}

bd_status bd_linear_multitenant_tiled_kbit(const uint16_t* x_f16, const uint16_t* w_tiled,
                                           const uint32_t* const* planes_by_tenant, const float* alpha_by_tenant,
                                           const int32_t* tenant_of_token, uint16_t* y_f16, int64_t T, int64_t out,
                                           int64_t in, int32_t n_tenants, int32_t k, void* stream) {
    return tiled_linear_impl(1, x_f16, &w_tiled, planes_by_tenant, &alpha_by_tenant, tenant_of_token, &y_f16, T, &out, in,
                             n_tenants, k, stream, false, nullptr);
}

bd_status bd_group_tokens(const int32_t* tenant_of_token, int32_t T, int32_t* token_of_col, int32_t* job_tenant,
                          int32_t* job_tile, int32_t* job_col_begin, int32_t* job_col_end, int32_t* n_jobs) {
    if (T < 1 || T > kMaxDecodeTokens) return BD_ERR_SHAPE;
    if (!tenant_of_token || !token_of_col || !job_tenant || !job_tile || !job_col_begin || !job_col_end || !n_jobs)
        return BD_ERR_NULL;
    DecodeMeta m;
    build_meta(tenant_of_token, 0, T, &m);
    for (int i = 0; i < T; ++i) token_of_col[i] = m.token_of_col[i];
    for (int j = 0; j < m.n_jobs; ++j) {
        job_tenant[j] = m.job_tenant[j];
        job_tile[j] = m.job_tile[j];
        job_col_begin[j] = m.job_col_begin[j];
        job_col_end[j] = m.job_col_end[j];
    }
    *n_jobs = m.n_jobs;
    return BD_OK;
}

bd_status bd_materialize(const uint16_t* w_base_f16, const uint32_t* packed, const float* alpha, uint16_t* w_out_f16,
                         int64_t out, int64_t in, void* stream) {
    if (out < 0 || in < 0 || in % 32 != 0) return BD_ERR_SHAPE;
    if (out == 0 || in == 0) return BD_OK;
    if (!w_base_f16 || !packed || !alpha || !w_out_f16) return BD_ERR_NULL;
    if (misaligned(w_base_f16, 16) || misaligned(packed, 16) || misaligned(w_out_f16, 16)) return BD_ERR_ALIGN;
    return bd::launch_materialize(w_base_f16, packed, alpha, w_out_f16, out, in, (hipStream_t)stream) == hipSuccess
               ? BD_OK
               : BD_ERR_DEVICE;
}

bd_status bd_linear_naive(const uint16_t* x_f16, const uint16_t* const* w_by_tenant, const int32_t* tenant_of_token,
                          uint16_t* y_f16, int64_t T, int64_t out, int64_t in, int32_t n_tenants, void* stream) {
    if (T < 0 || out < 0 || in < 0 || n_tenants < 0 || in % 8 != 0 || T > 65535) return BD_ERR_SHAPE;
    if (T == 0 || out == 0) return BD_OK;
    if (!x_f16 || !w_by_tenant || !tenant_of_token || !y_f16) return BD_ERR_NULL;
    if (misaligned(x_f16, 16) || misaligned(y_f16, 2)) return BD_ERR_ALIGN;
    for (int64_t t = 0; t < T; ++t)
        if (tenant_of_token[t] < 0 || tenant_of_token[t] >= n_tenants) return BD_ERR_TENANT;
    for (int64_t t0 = 0; t0 < T; t0 += kMaxDecodeTokens) {
        const int n = (int)std::min<int64_t>(kMaxDecodeTokens, T - t0);
        DecodeMeta meta;
        build_meta(tenant_of_token, t0, n, &meta);
        if (bd::launch_linear_naive(x_f16 + t0 * in, w_by_tenant, meta, y_f16 + t0 * out, out, in,
                                    (hipStream_t)stream) != hipSuccess)
            return BD_ERR_DEVICE;
    }
    return BD_OK;
}

bd_status bd_probe_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
    if (bytes % 16 != 0) return BD_ERR_SHAPE;
    if (bytes == 0) return BD_OK;
    if (!src || !sink) return BD_ERR_NULL;
    if (misaligned(src, 16) || misaligned(sink, 4)) return BD_ERR_ALIGN;
    return bd::launch_probe_read(src, bytes, sink, (hipStream_t)stream) == hipSuccess ? BD_OK : BD_ERR_DEVICE;
}

bd_status bd_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (bytes % 16 != 0) return BD_ERR_SHAPE;
    if (bytes == 0) return BD_OK;
    if (!dst || !src) return BD_ERR_NULL;
    if (misaligned(src, 16) || misaligned(dst, 16)) return BD_ERR_ALIGN;
    if (overlaps(dst, bytes, src, bytes)) return BD_ERR_ALIAS;
    return bd::launch_probe_copy(dst, src, bytes, (hipStream_t)stream) == hipSuccess ? BD_OK : BD_ERR_DEVICE;
}

}  // extern "C"
