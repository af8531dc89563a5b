// Decode kernel of the multi-tenant linear (Eq. 6 of the paper) over the tiled serving layout:
//     y[t, n] = sum_k x[t,k] W_base[n,k]  +  alpha_e * sum_k x[t,k] s_e[n,k],   e = tenant(t).
//
// At decode every token has its own tenant, so a packed sign word is used exactly once and
// the kernel is a pure stream: per byte of base weight it must turn B/16 sign bits into
// multiply-add operands.  Both products run on v_mfma_f32_16x16x32_f16 (A = 16 output rows x
// 32 k, B = 32 k x 16 token columns, tokens sorted by tenant); a delta "job" is one tenant's
// signs against all 16 columns, of which only that tenant's columns are kept.
//
// Sign expansion.  A byte of 8 signs becomes the 8 fp16 values +-1.0 (one 128-bit MFMA operand
// register group) by ONE look-up in LDS: the table has 256 entries x 16 B, replicated 16 times
// so that lane l reads copy l % 16 and a group of 16 lanes never shares a bank.  The address
// is built by one v_perm_b32 (sign byte -> address bits 8..15, lane copy -> bits 4..7), so the
// vector ALU spends one instruction per 8 signs; the LDS read port does the rest, next to the
// matrix pipe.  (Expanding with and-or instructions costs >= 8 per 8 signs and, at one token per
// tenant, makes the vector ALU the bottleneck long before HBM.)
//
// Decomposition.  The grid is persistent: one workgroup per compute unit, each owning a
// contiguous range of the launch's 16-row blocks (all matrices of a grouped launch laid end to
// end); its wavefronts split the k tiles into contiguous ranges.  A task = one (row block, k tile):
// 8 KiB of base (8 loads of 1 KiB), 512 B of signs per job (one 64-bit load per lane) and the
// 16 x 256 block of x, which each lane loads straight from global memory (L2 hits) in B-operand
// order: no staging, no barrier in the loop.  When a wavefront has at most two k tiles its x
// stays in registers for all of its row blocks (x is then fetched once per workgroup instead
// of once per task; the L1 is an in-order queue, so every x request it does not carry leaves
// room for a weight request).  Otherwise x is double-buffered per task.
// Everything of task t+1 is requested while task t is being multiplied: W[v] right after its
// MFMA, the signs of job j right after their addresses are formed.  Per row block the
// wavefronts' partial tiles go to LDS slots and are added in a fixed order when the slots are
// full or the work is done; y is written once.
//
// Quantised base (Q8; Sec. 4.2 of the paper, quantized base models).  The base tile then holds one
// byte per weight, u = q + 128, and a lane's 8 bytes of a slice become the MFMA operand by four
// v_perm_b32: byte u next to the constant 0x64 is the fp16 number 1024 + u, exactly.  The base
// accumulator therefore holds sum_k x (1152 + q); a second MFMA per slice with an all-ones A operand
// accumulates sum_k x, and the finished row block is scale[n] * (acc - 1152 * sum_k x): no
// arithmetic per weight beyond the byte shuffle.
//
// Row-major tensors (RM; what bd_compress writes and bd_linear_multitenant takes).  The same kernel reads W
// [out, in] fp16 and packed signs [out, in/32] as they are: slice v of a base tile is then 16 rows x 64 bytes
// (lane (r, g) reads 16 bytes of row r), and a tenant's signs of a tile are 16 rows x 32 bytes, of which lane
// (r, g) loads words 2 g and 2 g + 1.  Those hold sign BYTE i of slices 2 g and 2 g + 1 for every lane group i,
// while the lane needs byte g of all eight slices: the four lanes of a row exchange them with two byte shuffles,
// a swap between the wavefront's halves, two more shuffles and a swap between neighbouring rows of 16 lanes
// (v_permlane32_swap / v_permlane16_swap), six vector instructions per job and task.  The tenants' pointers
// come from the caller's device table (one scalar load each) instead of the kernel arguments.
//
// This header is the kernel; linear_decode_tiled.hip, linear_decode_tiled_q8.hip and linear_decode_rowmajor.hip
// instantiate it for the fp16 base, the 8-bit base and the row-major tensors (three translation units, so that
// they compile side by side).
#pragma once

#include <type_traits>

#include "bd_device.h"
#include "bd_launch.h"
#include "bd_tiled.h"

namespace bd {

namespace {

constexpr int kLutBytes = 256 * 16 * 16;          // 256 entries x 16 copies x 16 B
constexpr int kRedBytesPerWave = 16 * 16 * 4;     // one 16 x 16 fp32 tile
constexpr int kMaxWavesTiled = 8;
// x staging of one wavefront: 16 token rows x (512 B + 16 B pad), the pad spreads the 16 rows over all banks
constexpr int kStageRowBytes = kTileK * 2 + 16;
constexpr int kStageBytes = 16 * kStageRowBytes;
// LDS after the table: one region per wavefront = slots for the partial tiles of finished row blocks.
// Resident x is staged there before the first task (the slots overlay the staging rows).
template <int XSTEPS> struct LdsPlan {
    static constexpr int kRedSlots = 8;   // 16 x 16 tiles; a row block takes one per column tile
    static constexpr int kRegion = (XSTEPS > 0 && kStageBytes > kRedSlots * kRedBytesPerWave) ? kStageBytes : kRedSlots * kRedBytesPerWave;
    // behind the regions: (span, token) of every column of both column tiles, for the threads that write y
    static constexpr int kMeta = kLutBytes + kMaxWavesTiled * kRegion;
    static constexpr int kTotal = kMeta + kTiledMaxCt * kTiledMaxTokens * 8;
};
static_assert(LdsPlan<0>::kTotal <= 160 * 1024 && LdsPlan<2>::kTotal <= 160 * 1024, "LDS budget");

__device__ __forceinline__ void lds_wave_sync() {   // order this wavefront's LDS writes before its later reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef const u32x4 __attribute__((address_space(3)))* lds_u32x4_ptr;

__device__ __forceinline__ u32x4 ldg16_stream(const unsigned char* base, uint32_t off) {
    return __builtin_nontemporal_load((const u32x4*)(base + off));
}
__device__ __forceinline__ u32x2 ldg8_stream(const unsigned char* base, uint32_t off) {
    return __builtin_nontemporal_load((const u32x2*)(base + off));
}
__device__ __forceinline__ u32x4 ldg16(const unsigned char* base, uint32_t off) {
    return *(const u32x4*)(base + off);
}

// The MFMA operand of slice v of a job's tile: byte v of the lane's sign words -> table entry.
// `lanebits` = 16 * (lane % 16) in byte 0; the selector puts sign byte (v % 4) of word v / 4
// into byte 1 and zeros above: address = 256 * byte + 16 * copy (the table starts at LDS address 0).
__device__ __forceinline__ u32x4 lut_read(const u32x2 s, const int v, const uint32_t lanebits) {
    const uint32_t addr = __builtin_amdgcn_perm(s[v >> 2], lanebits, 0x0C0C0000u | ((4u + (v & 3)) << 8));
    return *(lds_u32x4_ptr)(uintptr_t)addr;
}

// Row-major signs.  In: this lane's words 2 g and 2 g + 1 of its row (lane (r, g) = (lane % 16, lane / 16)); byte i of
// word w is the sign byte of slice w for lane group i.  Out: s[0] = byte g of words 0, 1, 4, 5 and s[1] = byte g of
// words 2, 3, 6, 7 (in that order), i.e. everything lane (r, g) needs.  All 64 lanes must be active.
__device__ __forceinline__ u32x2 rm_gather_sign_bytes(const u32x2 w) {
    // bytes for lane groups 0, 1 and for 2, 3, the two words interleaved
    const uint32_t p = __builtin_amdgcn_perm(w[1], w[0], 0x05010400u);
    const uint32_t q = __builtin_amdgcn_perm(w[1], w[0], 0x07030602u);
    // lanes 32..63 of p against lanes 0..31 of q: groups 0, 1 now hold both halves' p, groups 2, 3 both halves' q
    const auto h = __builtin_amdgcn_permlane32_swap(p, q, false, false);
    // split by the parity of the byte index, then trade with the neighbouring group
    const uint32_t u = __builtin_amdgcn_perm(h[1], h[0], 0x05040100u);
    const uint32_t t = __builtin_amdgcn_perm(h[1], h[0], 0x07060302u);
    const auto f = __builtin_amdgcn_permlane16_swap(u, t, false, false);
    return u32x2{f[0], f[1]};
}
// Row-major 8-bit base.  In: the 16 bytes lane (r, g) loaded, q[row r][64 i + 16 g ..] (two's complement).  Out: the
// lane's 8 bytes of slice 2 i in words 0, 1 and of slice 2 i + 1 in words 2, 3, as u = q + 128 (what the tiled 8-bit base
// holds).  The four lanes of a row hold [lo, hi] halves; lane g' needs half g' % 2 of lane g' / 2 (slice 2 i) and of
// lane 2 + g' / 2 (slice 2 i + 1): a swap between neighbouring rows of 16 lanes, then one between the wavefront's halves.
__device__ __forceinline__ u32x4 rm_gather_q8(const u32x4 w) {
    u32x4 r;
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const auto s16 = __builtin_amdgcn_permlane16_swap(w[d], w[2 + d], false, false);
        const auto s32 = __builtin_amdgcn_permlane32_swap(s16[0], s16[1], false, false);
        r[d] = s32[0] ^ 0x80808080u;
        r[2 + d] = s32[1] ^ 0x80808080u;
    }
    return r;
}
// slice v of the gathered bytes: word (v / 2) % 2, byte v % 2 + 2 * (v / 4)
__device__ __forceinline__ u32x4 lut_read_rm(const u32x2 s, const int v, const uint32_t lanebits) {
    const uint32_t addr = __builtin_amdgcn_perm(s[(v >> 1) & 1], lanebits, 0x0C0C0000u | ((4u + ((v & 1) | ((v & 4) >> 1))) << 8));
    return *(lds_u32x4_ptr)(uintptr_t)addr;
}

}  // namespace

// XSTEPS = 1 or 2: every wavefront has exactly that many k tiles and keeps their x in registers.
// XSTEPS = 0: any number of k tiles per wavefront, x double-buffered per task.
// NCT = 2 (streamed x only): 17..32 tokens as two column tiles; the tasks of one (row block, k tile)
// then come in pairs that share the base registers, so the base is still read once.
// RM: row-major W (fp16, or the int8 q of the 8-bit base with its `out` scales) and packed signs (one matrix,
// in % 128 == 0) instead of the tiled tensors.
template <int NJ, int XSTEPS, int NCT, bool Q8, bool RM = false>
__global__ __launch_bounds__(kMaxWavesTiled * kWave) void linear_decode_tiled_kernel(const TiledArgs a) {
    constexpr uint32_t kWTile = Q8 ? kTileBaseQ8Bytes : kTileBaseBytes;   // bytes of one base tile
    constexpr int kWLoads = Q8 ? 4 : 8;                                   // 1 KiB loads per base tile
    extern __shared__ __align__(16) unsigned char smem[];   // [0, 64 KiB): table; then one region per wavefront
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    const int c = lane & 15;   // A row (output row) for loads, B/D column (token) for MFMA operands and results
    const int g = lane >> 4;
    using Plan = LdsPlan<XSTEPS>;
    static_assert(NCT == 1 || XSTEPS == 0, "two column tiles only with streamed x");
    // Touch every 64-byte line of the kernel arguments at once: the first read of a line is a trip
    // to memory, and taken one after the other (pointer tables are indexed by values read before)
    // those trips would delay the first weight request by microseconds.
    {
        const unsigned char __attribute__((address_space(4)))* ka =
            (const unsigned char __attribute__((address_space(4)))*)__builtin_amdgcn_kernarg_segment_ptr();
        constexpr int kLines = (int)((sizeof(TiledArgs) + 63) / 64);
        uint32_t touched[kLines];
#pragma unroll
        for (int i = 0; i < kLines; ++i) {
            const uint32_t off = (uint32_t)i * 64u;
            asm volatile("s_load_dword %0, %1, %2" : "=s"(touched[i]) : "s"(ka), "s"(off));
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int i = 0; i < kLines; ++i) asm volatile("" ::"s"(touched[i]));
    }
    const int KT = a.KT;
    const int rb_total = a.rb_end[a.n_mats - 1];
    // this workgroup's row blocks [r0, r1) of the concatenated matrices (the host keeps grid <= rb_total)
    const int r0 = (int)((int64_t)blockIdx.x * rb_total / gridDim.x);
    const int r1 = (int)((int64_t)(blockIdx.x + 1) * rb_total / gridDim.x);
    const int n_rb = r1 - r0;
    // This wavefront's k tiles: kb, kb + kstride, ... (`steps` of them).  Tiled tensors: a contiguous range.  Row-major: every
    // nw-th tile, so that the wavefronts of a workgroup are on neighbouring tiles at the same time: a 128-byte line of a
    // row's signs covers four k tiles, and taken by one wavefront in four consecutive tasks it would come from HBM four times.
    const int kb = RM ? wave : wave * KT / nw;
    const int kstride = RM ? nw : 1;
    const int steps = XSTEPS > 0 ? XSTEPS : (RM ? (KT - wave + nw - 1) / nw : (wave + 1) * KT / nw - kb);
    const bool have_work = n_rb > 0 && steps > 0;

    auto mat_of = [&](const int rbg, int& m, int& rb) {
        m = 0;
        if (a.n_mats > 1 && rbg >= a.rb_end[0]) m = 1;
        if (a.n_mats > 2 && rbg >= a.rb_end[1]) m = 2;
        rb = rbg - (m > 0 ? a.rb_end[m - 1] : 0);
    };

    // ---- pointers of the matrix whose tiles are being REQUESTED (the task being multiplied only
    // needs registers); reloaded from the kernel arguments when the requests cross into the next matrix
    int m_req, rb_req;
    mat_of(r0, m_req, rb_req);
    const unsigned char* wt = (const unsigned char*)a.wt[m_req];
    const unsigned char* sp[NCT][NJ];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
        for (int j = 0; j < NJ; ++j) sp[ct][j] = RM ? nullptr : (const unsigned char*)a.signs[ct][m_req][j];
    // Row-major: the tenants' pointers come from the caller's table in device memory.  Sixteen pointers held as
    // scalars cannot be dropped and fetched again like kernel arguments, and would push the kernel's vector
    // registers into scratch; so lane j of one register pair holds the pointer of job slot j, and a sign load
    // takes its base address from there with two v_readlane.
    uint32_t ptr_lo[NCT], ptr_hi[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        ptr_lo[ct] = ptr_hi[ct] = 0u;
        if constexpr (RM) {
            int tenant_l = a.job_tenant[ct][0];
#pragma unroll
            for (int i = 1; i < kTiledMaxJobs; ++i) tenant_l = (lane == i) ? a.job_tenant[ct][i] : tenant_l;
            const uint64_t pv = (uint64_t)a.packed_by_tenant[tenant_l];
            ptr_lo[ct] = (uint32_t)pv;
            ptr_hi[ct] = (uint32_t)(pv >> 32);
        }
    }
    auto sign_ptr = [&](const int ct, const int j) -> const unsigned char* {
        if constexpr (RM) {
            const uint32_t lo = __builtin_amdgcn_readlane(ptr_lo[ct], j), hi = __builtin_amdgcn_readlane(ptr_hi[ct], j);
            return (const unsigned char*)(((uint64_t)hi << 32) | lo);
        } else {
            return sp[ct][j];
        }
    };
    // Byte offsets of a task's loads = a uniform part (tile) + this lane's part.  Tiled: the lane's part is its place
    // inside a tile.  Row-major: the uniform part is the k tile only and the lane's part carries the row, so it
    // changes with the row block (rows beyond `out` read the last row again; their results are never stored).
    uint32_t lane16 = (uint32_t)lane * 16u, lane8 = (uint32_t)lane * 8u;
    auto rm_lane_offsets = [&](const int rb) {
        const int row = min(rb * kTileRows + c, a.out[0] - 1);
        lane16 = (uint32_t)row * ((uint32_t)a.in * (Q8 ? 1u : 2u)) + (uint32_t)g * 16u;
        lane8 = (uint32_t)row * ((uint32_t)a.in >> 3) + (uint32_t)g * 8u;
    };
    if constexpr (RM) rm_lane_offsets(rb_req);
    auto w_off = [&](const int rb, const int kt) {   // uniform byte offset of tile (rb, kt) of the base
        return RM ? (uint32_t)kt * (uint32_t)(kTileK * (Q8 ? 1 : 2)) : (uint32_t)(rb * KT + kt) * kWTile;
    };
    auto s_off = [&](const int rb, const int kt) {   // ... of a tenant's signs
        return RM ? (uint32_t)kt * (uint32_t)(kTileK / 8) : (uint32_t)(rb * KT + kt) * (uint32_t)kTileSignBytes;
    };
    constexpr uint32_t kSliceStride = RM ? 64u : 1024u;   // bytes between a lane's loads of consecutive slices
    // The tiled tensors are read once, whole cache lines at a time, with non-temporal loads (nothing of a line is
    // needed again).  Row-major, a load takes half a line of the base and a quarter of a line of signs per row; the rest
    // of the line belongs to the next slice or to the neighbouring wavefront's tiles, so those loads are ordinary ones
    // and the line stays in L2 for them (non-temporal, every line came from HBM 1.6 to 2.3 times).
    auto ld_w = [](const unsigned char* p, const uint32_t off) { return RM ? ldg16(p, off) : ldg16_stream(p, off); };
    auto ld_s = [](const unsigned char* p, const uint32_t off) {
        return RM ? *(const u32x2*)(p + off) : ldg8_stream(p, off);
    };
    // Row-major, `in` = 128 mod 256: the last k tile of a row has 4 slices.  No load may reach beyond the row (the
    // last row ends the tensor), so slices 4..7 of such a tile read slices 0..3 again and are replaced by zeros when
    // they are multiplied; lane groups 2, 3 read the row's first sign words instead of theirs (any valid words do:
    // their x is zero).  All of it is uniform arithmetic per task, no branch around a load.
    const int kt_short = (RM && (a.in % kTileK) != 0) ? KT - 1 : -1;
    auto w_base_hi = [&](const int kt) {   // the pointer slices 4..7 of tile kt are read through
        return (RM && kt == kt_short) ? wt - (kWLoads / 2) * kSliceStride : wt;
    };
    auto s_lane_off = [&](const uint32_t off_u, const uint32_t l8, const int kt) {
        uint32_t off = off_u + l8;
        if constexpr (RM) off = (kt == kt_short && g >= 2) ? l8 - (uint32_t)g * 8u : off;
        return off;
    };

    // x of one k tile is a [16 tokens][256] fp16 block.  It is fetched with loads whose lanes are
    // contiguous in memory (load i: token rows 2i and 2i+1, 512 B each) and brought into B-operand
    // order (lane (c, g): row c, elements 32 v + 8 g ..) through this wavefront's LDS staging rows:
    // fetching it in operand order directly would make every lane its own 16-byte access.
    // Rows of columns beyond T read token col_token[0] (valid memory); their results are never stored.
    const unsigned char* xg = (const unsigned char*)a.x;
    const int xh = lane >> 5;                                   // which of the two rows of a load
    const uint32_t xcol = (uint32_t)(lane & 31) * 16u;          // byte inside the tile row
    const int k_ragged = (a.in % kTileK != 0) ? KT - 1 : -1;    // the tile that reaches beyond `in`, if any
    const uint32_t row_bytes = (uint32_t)a.in * 2u;
    auto x_fetch = [&](u32x4 (&xraw)[8], const int kt) {
        uint32_t xc = xcol;
        asm volatile("" : "+v"(xc));   // keep "base + lane offset" a 32-bit offset (see task())
        const uint32_t off = xc + (uint32_t)kt * (uint32_t)(kTileK * 2);
        const bool inside = (kt != k_ragged) || (kt * kTileK + (lane & 31) * 8 < a.in);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ra = 2 * i < a.T[0] ? a.col_token[0][2 * i] : a.col_token[0][0];
            const int rbw = 2 * i + 1 < a.T[0] ? a.col_token[0][2 * i + 1] : a.col_token[0][0];
            const uint32_t tokoff = (uint32_t)(xh ? rbw : ra) * row_bytes;
            xraw[i] = u32x4{0u, 0u, 0u, 0u};
            if (inside) xraw[i] = ldg16(xg, tokoff + off);
        }
    };
    // Streamed x (a fresh tile per task) is fetched in operand order directly: lane (c, g), slice v reads
    // x[token of column c][256 kt + 32 v + 8 g ..]; a trip through LDS per task would sit on the critical path.
    uint32_t xlane[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        int tok_c = a.col_token[ct][0];
#pragma unroll
        for (int i = 0; i < kTiledMaxTokens; ++i) tok_c = (c == i && i < a.T[ct]) ? a.col_token[ct][i] : tok_c;
        xlane[ct] = (uint32_t)tok_c * row_bytes + (uint32_t)g * 16u;
    }
    // A slice that lies beyond `in` (ragged tile only) reads the lane's last slice inside the row again (or the row's first
    // bytes if it has none), valid memory, and x_zero_beyond replaces it by zeros once it has arrived: both paths issue the
    // same eight loads, so the count of loads in flight at any later point is known at compile time and nothing has to
    // wait for more than it needs.  The common path keeps its constant offsets (no address arithmetic per slice).
    auto x_fetch_operands = [&](u32x4 (&xop)[8], const int kt, const int ct) __attribute__((always_inline)) {
        uint32_t xl = ct == 0 ? xlane[0] : xlane[NCT - 1];
        asm volatile("" : "+v"(xl));
        const uint32_t off = xl + (uint32_t)kt * (uint32_t)(kTileK * 2);
        if (kt != k_ragged) {
#pragma unroll
            for (int v = 0; v < 8; ++v) xop[v] = ldg16(xg, off + v * 64);
        } else {
            const int n_in = (a.in - kt * kTileK - 8 * g + 31) >> 5;   // this lane's slices inside the row (may be <= 0)
            const uint32_t last = n_in > 0 ? off + (uint32_t)(n_in - 1) * 64u : xl;
#pragma unroll
            for (int v = 0; v < 8; ++v) xop[v] = ldg16(xg, min(off + (uint32_t)v * 64u, last));
        }
    };
    auto x_zero_beyond = [&](u32x4 (&xop)[8], const int kt) __attribute__((always_inline)) {
        if (kt == k_ragged) {
#pragma unroll
            for (int v = 0; v < 8; ++v)
                if (kt * kTileK + 32 * v + 8 * g >= a.in) xop[v] = u32x4{0u, 0u, 0u, 0u};
        }
    };
    // ---- requests of the first task: x first, then the base, (the table,) then the signs.  x is small and every
    // workgroup asks for the same lines; asked for behind the first base tiles of all compute units (16 MB) it arrives
    // microseconds after them and the first base product waits for it.  (Measured: 1.3 % on launches of one matrix, nothing
    // on the grouped launches, whose end is set by the stream.)
    constexpr int XR = XSTEPS > 0 ? XSTEPS : 1;   // x register sets in operand order
    u32x4 xs[XR][8];
    u32x4 xraw[XR][8];                            // resident x as fetched; streamed x: the next task's operands
    if (have_work) {
        if constexpr (XSTEPS > 0) x_fetch(xraw[0], kb);
        else x_fetch_operands(xs[0], kb, 0);
        if constexpr (XSTEPS == 2) x_fetch(xraw[1], kb + kstride);
    }
    u32x4 wr[kWLoads];   // fp16 base: slice v; 8-bit base: slices 2 i and 2 i + 1 (8 bytes each)
    u32x2 sr[NJ];
    if (have_work) {
        const uint32_t woff0 = w_off(rb_req, kb) + lane16;
        const unsigned char* const wt_hi0 = w_base_hi(kb);
#pragma unroll
        for (int v = 0; v < kWLoads; ++v) wr[v] = ld_w(v >= kWLoads / 2 ? wt_hi0 : wt, woff0 + (uint32_t)v * kSliceStride);
    }

    // ---- the table: entry b, copy cp at 256 b + 16 cp; element e = bit e of b ? +1.0 : -1.0.
    // Built (and the workgroup synchronised) while only the first base requests are in flight: the
    // later requests queue up behind the memory system, and a barrier behind them would hold the
    // first multiplications back by microseconds.
    // Consecutive lanes write consecutive 16-byte copies (16 per entry), a wavefront 1 KiB at a stretch: with a
    // lane per entry the writes of a wavefront were 128 bytes apart, eight of them on every bank.
    for (int q = threadIdx.x; q < 256 * 16; q += blockDim.x) {
        const uint32_t b = (uint32_t)q >> 4;
        u32x4 e;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            e[i] = 0xBC00BC00u ^ (((b >> (2 * i)) & 1u) << 15) ^ (((b >> (2 * i + 1)) & 1u) << 31);
        *(u32x4*)(smem + q * 16) = e;
    }
    // What the write of y needs per column, read from the kernel arguments with a lane's own index (a load from memory)
    // here, where it waits with everything else, and from LDS when a row block is finished: at the end of a launch a trip
    // to memory for it would be added to the launch's time.
    if (threadIdx.x < kTiledMaxCt * kTiledMaxTokens) {
        const int ct = threadIdx.x / kTiledMaxTokens, col = threadIdx.x % kTiledMaxTokens;
        *(u32x2*)(smem + Plan::kMeta + threadIdx.x * 8) = u32x2{(uint32_t)a.col_span[ct][col], (uint32_t)a.col_token[ct][col]};
    }
    __syncthreads();


    unsigned char* const region = smem + kLutBytes + wave * Plan::kRegion;
    auto x_to_operands = [&](const u32x4 (&xraw)[8], u32x4 (&xop)[8]) {
        lds_wave_sync();   // earlier reads of the staging rows are done
#pragma unroll
        for (int i = 0; i < 8; ++i) *(u32x4*)(region + (2 * i + xh) * kStageRowBytes + xcol) = xraw[i];
        lds_wave_sync();
#pragma unroll
        for (int v = 0; v < 8; ++v) xop[v] = *(const u32x4*)(region + c * kStageRowBytes + 64 * v + 16 * g);
    };

    if (have_work) {
        const uint32_t soff0 = s_lane_off(s_off(rb_req, kb), lane8, kb);
#pragma unroll
        for (int j = 0; j < NJ; ++j) sr[j] = ld_s(sign_ptr(0, j), soff0);
    }

    // this lane's column: owning job, tenant (for the scale)
    int myjob[NCT];
    float alpha_m[NCT][kTiledMaxMats];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        int tenant = 0;
        myjob[ct] = -1;
#pragma unroll
        for (int i = 0; i < kTiledMaxTokens; ++i) {
            myjob[ct] = (c == i && i < a.T[ct]) ? a.col_job[ct][i] : myjob[ct];
            tenant = (c == i && i < a.T[ct]) ? a.col_tenant[ct][i] : tenant;
        }
#pragma unroll
        for (int m = 0; m < kTiledMaxMats; ++m) alpha_m[ct][m] = m < a.n_mats ? a.alpha[m][tenant] : 0.f;
    }

    if (!have_work) return;   // uniform per workgroup (n_rb) / never true for steps (host: waves <= k tiles)
    if constexpr (XSTEPS == 0) {
        x_zero_beyond(xs[0], kb);
        // Everything requested so far (the first task's tiles, the scales) has to be there before the first delta job
        // anyway.  Waiting for it here, once, keeps the compiler from putting a wait for a register of the prologue at
        // the top of the task loop, where it would drain the loads in flight at every task.
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    }
#pragma unroll
    for (int i = 0; i < (XSTEPS > 0 ? XR : 0); ++i) x_to_operands(xraw[i], xs[i]);
    const uint32_t lanebits = (uint32_t)c << 4;

    float4v accb[NCT], dsel[NCT], accs[NCT];   // accs (8-bit base only): sum_k x of the column, in every row
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) accb[ct] = dsel[ct] = accs[ct] = float4v{0.f, 0.f, 0.f, 0.f};
    const half8 ones = __builtin_bit_cast(half8, u32x4{0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u});
    // 8 bytes u -> 8 fp16 (1024 + u): byte next to 0x64
    auto q8_operand = [](const u32x4 w2, const int h) {
        const uint32_t lo = w2[2 * h], hi = w2[2 * h + 1];
        return __builtin_bit_cast(half8, u32x4{__builtin_amdgcn_perm(0x64646464u, lo, 0x04010400u),
                                               __builtin_amdgcn_perm(0x64646464u, lo, 0x04030402u),
                                               __builtin_amdgcn_perm(0x64646464u, hi, 0x04010400u),
                                               __builtin_amdgcn_perm(0x64646464u, hi, 0x04030402u)});
    };

    // One task = (row block, k tile, column tile CT).  MORE: there is a next task; its tile index is
    // tile_next and its pointers are current (wt, sp).  The base registers are re-requested by the
    // last column tile of a (row block, k tile) only.  xr: this task's x in operand order; with
    // streamed x the next task's (kt_next, next column tile) is fetched into xnext during the task
    // and replaces xr at its end.
    // (always_inline on the lambdas: left to its own judgement the compiler may keep one a function, and everything it
    // captures by reference -- every register array of the kernel -- then lives in scratch)
    auto task = [&](auto more_tag, auto ct_tag, u32x4 (&xr)[8], const int kt_cur, const int rb_next, const int kt_next,
                    u32x4 (&xnext)[8]) __attribute__((always_inline)) {
        constexpr bool MORE = decltype(more_tag)::value;
        constexpr int CT = decltype(ct_tag)::value;
        constexpr int CT_NEXT = (CT + 1) % NCT;
        constexpr bool NEW_BASE = CT == NCT - 1;   // the next task is on another tile of W
        // The lane offsets pass through an empty asm in every task: otherwise the compiler hoists
        // "uniform base + lane offset" of every load out of the loop as a 64-bit register pair per load.
        uint32_t l16 = lane16, l8 = lane8;
        asm volatile("" : "+v"(l16), "+v"(l8));
        const uint32_t woff = w_off(rb_next, kt_next) + l16, soff = s_lane_off(s_off(rb_next, kt_next), l8, kt_next);
        const unsigned char* const wt_hi = w_base_hi(kt_next);
        const bool short_cur = RM && kt_cur == kt_short;
        // ---- base product; W[v] of the next task goes into the register group just read.  The wavefront runs at a higher
        // priority while it sends these requests (and x's): the other wavefront of the SIMD is in its delta jobs, and a
        // request that waits for an issue slot behind them is a request the memory system gets later (0.3 to 0.7 %).
        __builtin_amdgcn_s_setprio(2);
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            if constexpr (Q8) {
                if constexpr (RM && CT == 0) {   // the first column tile finds the registers as loaded; the second, gathered
                    if ((v & 1) == 0) wr[v >> 1] = rm_gather_q8(wr[v >> 1]);
                }
                accb[CT] = __builtin_amdgcn_mfma_f32_16x16x32_f16(q8_operand(wr[v >> 1], v & 1),
                                                                  __builtin_bit_cast(half8, xr[v]), accb[CT], 0, 0, 0);
                accs[CT] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, __builtin_bit_cast(half8, xr[v]), accs[CT], 0, 0, 0);
                if constexpr (MORE && NEW_BASE) {
                    if (v & 1) wr[v >> 1] = ld_w((v >> 1) >= kWLoads / 2 ? wt_hi : wt, woff + (uint32_t)(v >> 1) * kSliceStride);
                }
            } else {
                u32x4 wv = wr[v];
                if (RM && v >= 4) wv = short_cur ? u32x4{0u, 0u, 0u, 0u} : wv;
                accb[CT] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, wv),
                                                                  __builtin_bit_cast(half8, xr[v]), accb[CT], 0, 0, 0);
                if constexpr (MORE && NEW_BASE) wr[v] = ld_w(v >= 4 ? wt_hi : wt, woff + (uint32_t)v * kSliceStride);
            }
            __builtin_amdgcn_sched_barrier(0);   // keep each request behind the MFMA that frees its registers
        }
        if constexpr (MORE && XSTEPS == 0) x_fetch_operands(xnext, kt_next, CT_NEXT);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        // ---- delta jobs.  The 8 NJ (job, slice) pairs of the task form one sequence; the table
        // look-up of pair i + kLookAhead is issued before the MFMA of pair i, through a ring of
        // operand registers, and a job's sign words are re-requested as soon as its last address exists.
        // (row-major with 16 jobs and resident x: a shorter ring, so that the two registers the row offsets take do not end up
        // in scratch.  Measured with rings of 4 to 14 look-ups ahead: the depth does not change the time of a task.)
        constexpr int kLookAhead = (RM && NJ == 16 && XSTEPS > 0) ? 4 : 6, kRing = kLookAhead + 2, kPairs = 8 * NJ;
        u32x4 ring[kRing];
        float4v sel = {0.f, 0.f, 0.f, 0.f};   // the job owning this lane's column, this tile
        auto look_up = [&](const int i) __attribute__((always_inline)) {      // i = 8 * job + slice
            const int j = i >> 3, v = i & 7;
            if constexpr (RM) {
                if (v == 0) sr[j] = rm_gather_sign_bytes(sr[j]);
                ring[i % kRing] = lut_read_rm(sr[j], v, lanebits);
            } else {
                ring[i % kRing] = lut_read(sr[j], v, lanebits);
            }
            if constexpr (MORE) {
                if (v == 7) sr[j] = ld_s(sign_ptr(CT_NEXT, j), soff);
            }
        };
#pragma unroll
        for (int i = 0; i < kLookAhead; ++i) look_up(i);
        float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < kPairs; ++i) {
            if (i + kLookAhead < kPairs) look_up(i + kLookAhead);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, ring[i % kRing]),
                                                         __builtin_bit_cast(half8, xr[i & 7]), acc, 0, 0, 0);
            if ((i & 7) == 7) {
                const bool mine = (myjob[CT] == (i >> 3));
#pragma unroll
                for (int q = 0; q < 4; ++q) sel[q] = mine ? acc[q] : sel[q];
                // pin the selection here: left alone, the compiler sinks all of them below the last job
                // and keeps one live accumulator per job
                asm volatile("" : "+v"(sel[0]), "+v"(sel[1]), "+v"(sel[2]), "+v"(sel[3]));
                acc = float4v{0.f, 0.f, 0.f, 0.f};
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        dsel[CT] += sel;
        if constexpr (MORE && XSTEPS == 0) {   // this task's x is spent: move the next one in
            x_zero_beyond(xnext, kt_next);
#pragma unroll
            for (int v = 0; v < 8; ++v) xr[v] = xnext[v];
        }
    };

    // The partial tiles of `n` finished row blocks, first one rbg0: add the wavefronts in a fixed order, write y.
    auto flush = [&](const int rbg0, const int n, const bool more_follow) {
        __syncthreads();
        for (int idx = threadIdx.x; idx < n * 256; idx += blockDim.x) {   // n slots = n / NCT row blocks
            const int slot = idx >> 8, e = idx & 255, col = e >> 4, row = e & 15;
            const int ct = slot % NCT;
            int m, rb;
            mat_of(rbg0 + slot / NCT, m, rb);
            const int out = a.out[m], n_row = rb * kTileRows + row;
            const u32x2 meta = *(const u32x2*)(smem + Plan::kMeta + (ct * kTiledMaxTokens + col) * 8);
            const int span = (int)meta[0];   // columns of this token (its planes); 0: not a token's first column
            if (col < a.T[ct] && n_row < out && span > 0) {
                float s = 0.f;
                for (int p = 0; p < span; ++p)
                    for (int wv = 0; wv < nw; ++wv)
                        s += *(const float*)(smem + kLutBytes + wv * Plan::kRegion + (slot * 256 + e + p * 16) * 4);
                a.y[m][(int64_t)(int)meta[1] * out + n_row] = f2h_rne(s);
            }
        }
        if (more_follow) {
            // The stores of y must not be outstanding when the task loop goes on: loads and stores share one counter,
            // and with both kinds in flight the compiler can only wait for all of them -- it would put that wait at
            // the top of the task loop, where it drains the requested tiles at every task.
            if constexpr (XSTEPS == 0) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __syncthreads();
        }
    };

    int slot = 0, flush_base = r0;
    int m_cur = m_req;
    int rbi = 0;            // the row block being multiplied: r0 + rbi
    bool last_rb = false;
    float4v sc = {1.f, 1.f, 1.f, 1.f};   // 8-bit base: the scales of this lane's 4 output rows, asked for a row block ahead of their use
    int m_nx = m_req, rb_nx = 0;         // where the requests go after this row block's last task
    auto begin_rb = [&]() __attribute__((always_inline)) {
        last_rb = rbi + 1 == n_rb;
        if constexpr (Q8) {
            int m_c, rb_c;
            mat_of(r0 + rbi, m_c, rb_c);
            const float* ws = m_c == 0 ? a.wscale[0] : (m_c == 1 ? a.wscale[1] : a.wscale[2]);
            if constexpr (RM) {   // the caller's array of `out` scales: rows beyond `out` read the last one (never stored)
#pragma unroll
                for (int i = 0; i < 4; ++i) sc[i] = ws[min(rb_c * kTileRows + 4 * g + i, a.out[0] - 1)];
            } else {
                sc = *(const float4v*)(ws + rb_c * kTileRows + 4 * g);   // the scale array is padded to whole row blocks
            }
        }
        m_nx = m_req;
        rb_nx = 0;
        if (!last_rb) mat_of(r0 + rbi + 1, m_nx, rb_nx);
    };
    auto cross = [&]() __attribute__((always_inline)) {   // requests move on to the next row block: switch the pointers if it is in another matrix
        if constexpr (RM) rm_lane_offsets(rb_nx);
        if (m_nx != m_req) {
            wt = (const unsigned char*)a.wt[m_nx];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
                for (int j = 0; j < NJ; ++j) sp[ct][j] = (const unsigned char*)a.signs[ct][m_nx][j];
        }
    };
    // row block done: this wavefront's partial tiles -> slots; the slots are added up and written when they are full
    // more_tag: std::true_type / std::false_type where the caller knows whether another row block follows, RbDynamic
    // where last_rb tells
    struct RbDynamic {};
    auto end_rb = [&](auto more_tag) __attribute__((always_inline)) {
        bool last;
        if constexpr (std::is_same<decltype(more_tag), RbDynamic>::value) last = last_rb;
        else last = !decltype(more_tag)::value;
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            const float al = m_cur == 0 ? alpha_m[ct][0] : (m_cur == 1 ? alpha_m[ct][1] : alpha_m[ct][2]);
            if (a.planes > 1) {   // several planes per token: only a token's first column carries the base product
                int cc = c;
                asm volatile("" : "+v"(cc));   // derived here, once per row block, instead of living in a register
                bool first = false;
#pragma unroll
                for (int i = 0; i < kTiledMaxTokens; ++i) first = (cc == i && a.col_span[ct][i] > 0) ? true : first;
                if (!first) accb[ct] = accs[ct] = float4v{0.f, 0.f, 0.f, 0.f};
            }
            float4v r;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float base = Q8 ? sc[i] * (accb[ct][i] - 1152.f * accs[ct][i]) : accb[ct][i];
                r[i] = base + al * dsel[ct][i];
            }
            *(float4v*)(region + ((slot + ct) * 256 + c * 16 + 4 * g) * 4) = r;   // [column][row]
            accb[ct] = dsel[ct] = accs[ct] = float4v{0.f, 0.f, 0.f, 0.f};
        }
        slot += NCT;
        if (slot == Plan::kRedSlots || last) {
            flush(flush_base, slot, !last);
            flush_base += slot / NCT;
            slot = 0;
        }
        m_cur = m_nx;
        m_req = m_nx;
        rb_req = rb_nx;
        ++rbi;
    };
    using Ct0 = std::integral_constant<int, 0>;
    using CtL = std::integral_constant<int, NCT - 1>;
    if constexpr (XSTEPS > 0) {
        while (rbi < n_rb) {
            begin_rb();
#pragma unroll
            for (int ki = 0; ki < XSTEPS; ++ki) {
                if (ki + 1 < XSTEPS) {
                    task(std::true_type{}, Ct0{}, xs[ki], kb + ki * kstride, rb_req, kb + (ki + 1) * kstride, xraw[0]);
                } else if (!last_rb) {
                    cross();
                    task(std::true_type{}, Ct0{}, xs[ki], kb + ki * kstride, rb_nx, kb, xraw[0]);
                } else {
                    task(std::false_type{}, Ct0{}, xs[ki], kb + ki * kstride, 0, 0, xraw[0]);
                }
            }
            end_rb(RbDynamic{});
        }
    } else {
        // Streamed x: ONE loop over all (row block, k tile) pairs but the last, with a single copy of the task that requests
        // its successor, and the last task after the loop.  (As a loop nest with the last task inside it, the compiler
        // kept two sets of registers for the requested tiles, copied one into the other at the end of every task and
        // waited there for every outstanding load: nothing was in flight across a task boundary.)
        begin_rb();
        int ki = 0;
        const int total = n_rb * steps;
        for (int t = 0; t + 1 < total; ++t) {
            const bool inner = ki + 1 < steps;
            const int kt = kb + ki * kstride;
            // all but the last column tile: the next task stays on this tile (same k tile, next columns)
            if constexpr (NCT == 2) task(std::true_type{}, Ct0{}, xs[0], kt, rb_req, kt, xraw[0]);
            if (!inner) cross();
            task(std::true_type{}, CtL{}, xs[0], kt, inner ? rb_req : rb_nx, inner ? kt + kstride : kb, xraw[0]);
            if (inner) {
                ++ki;
            } else {
                end_rb(std::true_type{});
                begin_rb();
                ki = 0;
            }
        }
        const int kt = kb + ki * kstride;
        if constexpr (NCT == 2) task(std::true_type{}, Ct0{}, xs[0], kt, rb_req, kt, xraw[0]);
        task(std::false_type{}, CtL{}, xs[0], kt, 0, 0, xraw[0]);
        end_rb(std::false_type{});
    }
}

template <bool Q8, bool RM, int NJ, int XSTEPS, int NCT = 1>
static hipError_t launch_inst(const TiledArgs& args, int n_waves, unsigned grid, hipStream_t st) {
    auto kernel = linear_decode_tiled_kernel<NJ, XSTEPS, NCT, Q8, RM>;
    const size_t lds = (size_t)LdsPlan<XSTEPS>::kTotal;
    static PerDeviceOnce lds_limit;   // one per instantiation
    const hipError_t ea = lds_limit.run([&] {
        hipFuncAttributes fa;
        const hipError_t e = hipFuncGetAttributes(&fa, (const void*)kernel);
        if (e != hipSuccess) return e;
        if (fa.sharedSizeBytes != 0) return hipErrorInvalidValue;   // the table must start at LDS address 0
        return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    if (ea != hipSuccess) return ea;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(n_waves * kWave), lds, st, args);
    return hipGetLastError();
}

template <bool Q8, bool RM, int NJ>
static hipError_t launch_nj(const TiledArgs& args, int n_waves, int xsteps, unsigned grid, hipStream_t st) {
    if (xsteps == 1) return launch_inst<Q8, RM, NJ, 1>(args, n_waves, grid, st);
    if (xsteps == 2) return launch_inst<Q8, RM, NJ, 2>(args, n_waves, grid, st);
    return launch_inst<Q8, RM, NJ, 0>(args, n_waves, grid, st);
}

template <bool Q8, bool RM = false>
static hipError_t launch_tiled_t(const TiledArgs& args, int n_jobs, hipStream_t st) {
    if (RM && (args.n_mats != 1 || args.in % 128 != 0 || args.in < 128 || !args.packed_by_tenant)) return hipErrorInvalidValue;
    if (n_jobs < 1 || n_jobs > kTiledMaxJobs || args.n_mats < 1 || args.n_mats > kTiledMaxMats || args.n_ct < 1 ||
        args.n_ct > kTiledMaxCt)
        return hipErrorInvalidValue;
    const int rb_total = args.rb_end[args.n_mats - 1];
    if (rb_total < 1 || args.KT < 1) return hipErrorInvalidValue;
    // compute units of the current device, asked once per device (0 = not asked yet; 64 devices at most are remembered)
    static std::atomic<int> cus_of[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    int cus = cus_of[dev & 63].load(std::memory_order_relaxed);
    if (cus == 0) {
        int v = 0;
        cus = (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) ? v : 256;
        cus_of[dev & 63].store(cus, std::memory_order_relaxed);
    }
    // Persistent grid: at most one workgroup per compute unit, never more workgroups than row blocks -- and of the
    // grids that need the same number of rounds (row blocks per workgroup, rounded up) the SMALLEST: 1376 row blocks
    // (gate,up of Llama-2-7B) on 256 units are 6 rounds either way, but 256 workgroups leave 160 units idle during the
    // sixth while 230 workgroups of 6 (four of them 5) keep all of theirs streaming to the end.  The launch is bound by
    // HBM, not by the number of units, so it then takes the time of 5.4 rounds instead of 6.
    // 8 wavefronts, never more than k tiles (an empty reduction, KT == 0, never gets here: the host writes y = 0)
    const int rounds = (rb_total + cus - 1) / cus;
    const unsigned grid = (unsigned)((rb_total + rounds - 1) / rounds);
    int n_waves = kMaxWavesTiled;
    while (n_waves > 1 && n_waves > args.KT) n_waves >>= 1;
    if (args.n_ct == 2) {   // 17..32 tokens: two column tiles, streamed x
        if (n_jobs <= 4) return launch_inst<Q8, RM, 4, 0, 2>(args, n_waves, grid, st);
        if (n_jobs <= 8) return launch_inst<Q8, RM, 8, 0, 2>(args, n_waves, grid, st);
        return launch_inst<Q8, RM, 16, 0, 2>(args, n_waves, grid, st);
    }
    int xsteps = 0;
    if (args.KT > 0 && args.KT % n_waves == 0 && args.KT / n_waves <= 2) xsteps = args.KT / n_waves;
    if (n_jobs <= 4) return launch_nj<Q8, RM, 4>(args, n_waves, xsteps, grid, st);
    if (n_jobs <= 8) return launch_nj<Q8, RM, 8>(args, n_waves, xsteps, grid, st);
    return launch_nj<Q8, RM, 16>(args, n_waves, xsteps, grid, st);
}

}  // namespace bd
