// Large-tile form of the prefill GEMM (Eq. 6 of the paper with many tokens per tenant; see
// linear_prefill.hip for the formulation).  One workgroup of 4 wavefronts per compute unit, each
// wavefront alone on its SIMD with the whole register file: it owns 128 tokens x 64 output features
// of a 128 x 256 tile and multiplies with v_mfma_f32_32x32x16_f16 (A = 32 tokens x 16 k, B = 16 k x
// 32 features, 32 cycles): a lone wavefront issues an instruction only every 8 cycles or so, and the
// larger MFMA leaves room for the three other instructions (LDS reads, address arithmetic, loads)
// that each one needs.  The 16 accumulator tiles (base and delta separately, alpha applied at the
// end) fill the 256 accumulation registers.
//   x tile   128 tokens x 64 k  fp16  -> LDS, rows of 8 chunks in the order chunk ^ ((row / 2) % 8)
//   W tile   256 rows   x 64 k  fp16  -> LDS, same order
//   signs    256 rows   x 2 words     -> LDS as they are; a lane's byte of 8 signs becomes the
//            operand (8 fp16 of +-1.0) by one read of a byte table (256 entries x 8 copies x 16 B,
//            lane l reading copy l % 8)
// LDS is double-buffered (one barrier per step of 64 k); the global loads of step s + 3 are issued
// into the registers that have just been written out for step s + 1, so two steps of loads are in
// flight while a step is multiplied.  A wavefront alone on its SIMD issues in order, so everything
// else is dealt out between the MFMAs in portions that fit into the 32 cycles of one: behind the first
// MFMA of a pair one operand read of the next 16-wide k slice, behind the second one LDS write and one
// global load.  The step's barrier sits before its last slice, whose operands are in registers by
// then, so that the first reads of the next step overlap those MFMAs.  The finished tile leaves
// through LDS as fp16 rows, in 16-byte stores.
// Used when in % 64 == 0; other shapes take the 128 x 128 kernel.
// The same tile body also runs the left-hand side of Eq. 6, X (W + alpha S) with the bracket rounded to
// fp16, as ONE product on tiles of 256 tokens x 256 features (linear_prefill_merged_kernel; the caller
// asks for it by name): see MERGED at prefill_big_tile.
#include "bd_device.h"
#include "bd_launch.h"

namespace bd {

namespace {

constexpr int kBgM = 128, kBgN = 256, kBgK = 64;
constexpr int kMergedTile = kPrefillMergedTile;          // token rows of a tile of the merged form
constexpr int kBgRowBytes = kBgK * 2;                    // 128
constexpr int kBgWBytes = kBgN * kBgRowBytes;            // 32768
constexpr int kBgSBytes = kBgN * 8;                      // 2048
// LDS of a tile of TM token rows: [2 buffers: x, W, sign words][byte table][the tile's token of every row].  The x
// tile is laid out for 128 rows (half tiles use the first 64) or for 256; beside the larger one the table keeps
// 4 copies of every entry instead of 8.
template <int TM>
struct BgLds {
    static constexpr int kRows = TM > kBgM ? TM : kBgM;
    static constexpr int kX = kRows * kBgRowBytes;              // 16384 | 32768
    static constexpr int kBuf = kX + kBgWBytes + kBgSBytes;
    static constexpr int kLutCopies = TM > kBgM ? 4 : 8;
    static constexpr int kLutEntry = kLutCopies * 16;
    static constexpr int kLut = 256 * kLutEntry;
    static constexpr int kTok = kRows * 4;
    static constexpr int kTotal = 2 * kBuf + kLut + kTok;       // 135680 | 152576
    // 128 rows: buffer 1 follows buffer 0 (x, W, signs | x, W, signs), 51200 bytes on.  256 rows: x | x | W | W |
    // signs | signs, so that the distance between a region's two buffers still fits the 16-bit offset of an LDS instruction.
    static constexpr bool kByRegion = TM > kBgM;
    static constexpr int kXStride = kByRegion ? kX : kBuf;
    static constexpr int kWBase = kByRegion ? 2 * kX : kX, kWStride = kByRegion ? kBgWBytes : kBuf;
    static constexpr int kSBase = kByRegion ? 2 * kX + 2 * kBgWBytes : kX + kBgWBytes, kSStride = kByRegion ? kBgSBytes : kBuf;
};
constexpr int kBgLdsBytes = BgLds<kBgM>::kTotal;
// Epilogue: a wavefront's rows of y as fp16, 64 features + 16 B of padding each (rows 4 apart, which one LDS
// instruction writes together, then fall into different banks), in the tile buffers, which are free by then.
constexpr int kBgOutRowBytes = 64 * 2 + 16;
constexpr int kBgPanel = 4, kBgChunk = 32, kBgXcds = 8;  // launch order: 8 x 4 tiles (1024 tokens x 1024 features) per XCD at a time

__device__ __forceinline__ int bg_off(const int row, const int chunk) {
    return row * kBgRowBytes + ((chunk ^ ((row >> 1) & 7)) << 4);
}

// Workgroup barrier that orders LDS traffic only (__syncthreads also drains the global loads in flight).
__device__ __forceinline__ void bg_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

typedef const uint32_t __attribute__((address_space(1)))* bg_global_words;
typedef const uint16_t __attribute__((address_space(1)))* bg_global_halfwords;

// LDS through pointers in the LDS address space, made from byte offsets.  The kernel has no static LDS, so its
// dynamic LDS starts at address 0 (the host checks that): no instruction is spent on adding the (relocated, zero)
// base of the array, and a constant added to such a pointer travels in the offset field of the LDS instruction.
typedef unsigned char __attribute__((address_space(3)))* lds_bytes;
__device__ __forceinline__ lds_bytes lds_at(const uint32_t off) { return (lds_bytes)(uintptr_t)off; }
template <typename T>
__device__ __forceinline__ T lds_get(const lds_bytes p) {
    return *(const T __attribute__((address_space(3)))*)p;
}
template <typename T>
__device__ __forceinline__ void lds_put(const lds_bytes p, const T v) {
    *(T __attribute__((address_space(3)))*)p = v;
}

// acc += A . B with the accumulator held in place in the accumulation registers.  (Left to itself the
// compiler gives every MFMA a fresh destination and copies it back, four moves per MFMA, once all
// 256 accumulation registers are taken.)  Written as an asm statement the instruction is opaque to the
// compiler's hazard bookkeeping, so the callers keep to what needs none: A and B come straight from
// LDS reads, no accumulator is touched again within the next 15 MFMAs, and the epilogue waits
// explicitly before it reads the accumulators.
typedef float float16v __attribute__((ext_vector_type(16)));
__device__ __forceinline__ void mfma_in_place(float16v& acc, const half8 a, const half8 b) {
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

}  // namespace

// One tile: TM token rows r0 .. r0 + TM of token tile mt (whose rows' tokens are tile_tokens[]), output features
// 256 nt .. + 256.
// WM = 1: 4 wavefronts (1 x 4), each TM tokens x 64 features, alone on its SIMD; two sets of staging registers
// (loads two steps ahead).  WM = 2: 8 wavefronts (2 x 4), each TM / 2 x 64, two per SIMD; one set (one step ahead).
// TM = 128, or 64 (WM = 1 only): half a tile, for the tiles of a last round that would leave most units idle.
// MERGED: one product instead of two.  The table holds +-alpha (alpha rounded to fp16) instead of +-1, a lane adds
// its sign operand to its W operand in fp16 (one rounding per weight: the fine-tuned weight W + alpha S as an fp16
// model would store it, the left-hand side of Eq. 6) and multiplies once: half the matrix-core work, and a result
// that differs from the two-product form by that rounding of the weights.
// TILED: W and the signs are read from the serving layout of the decode kernel (tiles of 16 rows x 256 k in
// matrix-core operand order, bd_tile_base / bd_tile_signs): a 16-byte chunk of a row is a 16-byte chunk there too,
// 2 KiB per row block and step in one piece, and a row's sign bytes of a step are four 2-byte pieces 128 bytes apart.
template <int WM, int TM, bool MERGED, bool TILED>
__device__ __forceinline__ void prefill_big_tile(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, const int32_t* __restrict__ tile_tokens, const int32_t* __restrict__ tile_tenant,
    uint16_t* __restrict__ y, const int64_t out, const int64_t in, const int mt, const int nt, const int r0) {
    extern __shared__ __align__(16) unsigned char lds[];   // [2 buffers: x, W, sign words][table][tokens]
    using Lds = BgLds<TM>;
    constexpr int kBgBufBytes = Lds::kBuf, kBgLutBytes = Lds::kLut;
    // the result rows of all wavefronts fit in front of the tokens (the merged form's last table reads are issued
    // before the last barrier, so its table may be overwritten as well)
    static_assert(TM * kBgOutRowBytes * 4 <= 2 * kBgBufBytes + (MERGED ? kBgLutBytes : 0), "the epilogue's rows overlap the tokens");
    unsigned char* const lut = lds + 2 * kBgBufBytes;

    constexpr int kThreads = 256 * WM, kWaveM = TM / WM, MI = kWaveM / 32;
    // mfma_in_place hides the accumulators from the compiler's hazard bookkeeping, so the schedule itself has to keep
    // an accumulator's uses apart.  A k slice issues, for every (i, j), one MFMA into accb[i][j] and one into accd[i][j]:
    // 4 MI MFMAs, each accumulator once, always in the same order, so 4 MI - 1 other MFMAs (each 8 passes = 32 cycles of
    // the matrix pipe) lie between two uses of one accumulator.  The dependent-accumulate hazard of the 8-pass
    // instructions is below 20 cycles; 7 MFMAs (MI = 2: 64-row halves, or two wavefronts per SIMD) are 224.
    // The epilogue reads the accumulators with vector instructions after two `s_nop 15` (32 wait states; the rule for
    // reading the result of an 8-pass MFMA asks for 18).  Every instantiation has a full-output parity test.
    // (MERGED: 2 MI MFMAs per slice, each accumulator once: 3 or 7 others, 96 cycles or more, between two uses.)
    constexpr int kMfmasBetweenUses = (MERGED ? 2 : 4) * MI - 1;
    static_assert(MI == 2 || MI == 4 || (MERGED && MI == 8), "the slice schedules below are written for these token blocks per wavefront");
    static_assert(kMfmasBetweenUses >= (MERGED ? 3 : 7), "an accumulator would be used again while its last MFMA may still be in the pipe");
    constexpr int kBgXPer = TM * 8 / kThreads, kBgWPer = kBgN * 8 / kThreads;   // 16-byte chunks per thread and step
    constexpr int kSets = (WM == 1 && TM <= kBgM) ? 2 : 1;   // (256 rows: the registers hold one set)
    static_assert(!MERGED || WM == 1, "the merged form runs one wavefront per SIMD");
    static_assert(!TILED || WM == 1, "the tiled sources are written for one row of signs per thread");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int64_t n0 = (int64_t)nt * kBgN;
    const int64_t words_per_row = in >> 5;
    const int n_steps = (int)(in / kBgK), last = n_steps - 1;

    // What this thread fetches per step.  Empty token rows read token 0 and output rows beyond `out` the last
    // row: their products are never stored, so nothing has to be zeroed and no load is conditional.
    // Global addresses are a uniform base plus a 32-bit byte offset per thread (the host checks the ranges).
    // The prologue asks for things in the order in which their addresses become known, so that the trips to memory
    // overlap: W (kernel arguments only), then the tile's tenant and tokens; behind those x, the sign pointer, the signs.
    const unsigned char* const xbase = (const unsigned char*)x;
    const int64_t k_tiles = (in + 255) >> 8;                       // of the serving layout
    constexpr int kWStep = TILED ? 2048 : kBgRowBytes;              // bytes a thread's W address advances per step
    const unsigned char* const wbase = TILED ? (const unsigned char*)w + (n0 >> 4) * k_tiles * 8192 : (const unsigned char*)(w + n0 * in);
    uint32_t xsrc[kBgXPer], wsrc[kBgWPer];
    lds_bytes xdst[kBgXPer], wdst[kBgWPer];   // in buffer 0
    struct Staged {
        u32x4 xg[kBgXPer], wg[kBgWPer];
        uint32_t s0, s1;      // row-major signs: the row's two words of the step
        uint32_t su[4];       // tiled signs: the 2 bytes (slices 2 (step % 4), + 1) of the row's lanes g = 0..3
    };
    Staged set0, set1;
    const int step_b = 1 < last ? 1 : last;   // what the second set holds first
#pragma unroll
    for (int i = 0; i < kBgWPer; ++i) {
        const int q = tid + kThreads * i, row = q >> 3, c8 = q & 7;
        const int64_t wrow = n0 + row < out ? row : out - 1 - n0;
        // tiled: row block wrow / 16, slice c8 / 4 of the step's two, lane (wrow % 16, c8 % 4)
        wsrc[i] = TILED ? (uint32_t)((wrow >> 4) * k_tiles * 8192) + (c8 >> 2) * 1024 + (c8 & 3) * 256 + (uint32_t)(wrow & 15) * 16
                        : (uint32_t)(wrow * in * 2) + c8 * 16;
        wdst[i] = lds_at(Lds::kWBase + bg_off(row, c8));
        asm volatile("" : "+v"(wdst[i]));   // a register of its own: derived from xdst[i], it would cost an addition per use
        set0.wg[i] = *(const u32x4*)(wbase + wsrc[i]);
    }
    const int tenant = tile_tenant[mt];
    int tokv[kBgXPer];
#pragma unroll
    for (int i = 0; i < kBgXPer; ++i) tokv[i] = tile_tokens[r0 + ((tid + kThreads * i) >> 3)];
    if (kSets == 2) {
#pragma unroll
        for (int i = 0; i < kBgWPer; ++i) set1.wg[i] = *(const u32x4*)(wbase + (int64_t)step_b * kWStep + wsrc[i]);
    }
    __builtin_amdgcn_sched_barrier(0);

    // byte -> 8 fp16 (+1.0 where the bit is set, else -1.0; MERGED: +alpha, -alpha), element e = bit e; entry
    // [byte][copy].  Consecutive lanes write consecutive 16-byte copies (a wavefront 1 KiB at a stretch; a lane per
    // entry would put its writes 128 bytes apart, several of them on every bank).
    float alpha = 0.f;
    uint32_t minus = 0xBC00BC00u;
    if constexpr (MERGED) {
        alpha = alpha_by_tenant[tenant];
        const uint32_t h = (uint32_t)f2h_rne(alpha) ^ 0x8000u;
        minus = h | (h << 16);
    }
    for (int q = tid; q < 256 * Lds::kLutCopies; q += kThreads) {
        const uint32_t bb = (uint32_t)q / Lds::kLutCopies;
        u32x4 e;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            e[i] = minus ^ (((bb >> (2 * i)) & 1u) << 15) ^ (((bb >> (2 * i + 1)) & 1u) << 31);
        *(u32x4*)(lut + q * 16) = e;
    }
    const lds_bytes lut_lane = lds_at(2 * kBgBufBytes + (lane & (Lds::kLutCopies - 1)) * 16);
    __builtin_amdgcn_sched_barrier(0);

    if constexpr (!MERGED) alpha = alpha_by_tenant[tenant];
    // sign words: 256 threads take a row's two words each, 512 threads one word each
    const int s_row = WM == 1 ? tid : tid >> 1, s_word = WM == 1 ? 0 : tid & 1;
    const int64_t srow = n0 + s_row < out ? n0 + s_row : out - 1;
    const uint32_t* const tenant_signs = packed_by_tenant[tenant];
    const bg_global_words ssrc = (bg_global_words)(tenant_signs + srow * words_per_row) + s_word;
    const bg_global_halfwords ssrc_tiled = (bg_global_halfwords)((const unsigned char*)tenant_signs + (srow >> 4) * k_tiles * 512 + (srow & 15) * 8);
    auto fetch_signs = [&](Staged& st, const int step) {
        if constexpr (TILED) {
            const int at = (step >> 2) * 256 + (step & 3);   // in 2-byte units: tile step / 4, slices 2 (step % 4), + 1
#pragma unroll
            for (int g = 0; g < 4; ++g) st.su[g] = ssrc_tiled[at + g * 64];
        } else {
            st.s0 = ssrc[2 * step];
            if (WM == 1) st.s1 = ssrc[2 * step + 1];
        }
    };
#pragma unroll
    for (int i = 0; i < kBgXPer; ++i) {
        const int q = tid + kThreads * i, row = q >> 3, c8 = q & 7;
        const int tok = tokv[i];
        xsrc[i] = (uint32_t)((int64_t)(tok >= 0 ? tok : 0) * in * 2) + c8 * 16;
        if (c8 == 0) lds_put<int>(lds_at(2 * kBgBufBytes + kBgLutBytes + row * 4), tok);   // for the epilogue
        xdst[i] = lds_at(bg_off(row, c8));
        set0.xg[i] = *(const u32x4*)(xbase + xsrc[i]);
        if (kSets == 2) set1.xg[i] = *(const u32x4*)(xbase + (int64_t)step_b * kBgRowBytes + xsrc[i]);
    }
    fetch_signs(set0, 0);
    if (kSets == 2) fetch_signs(set1, step_b);

    const lds_bytes sdst = lds_at(Lds::kSBase + tid * (WM == 1 ? 8 : 4));
    // items: the x chunks, the W chunks, the sign word(s)
    constexpr int kItems = kBgXPer + kBgWPer + 1;
    auto fetch_item = [&](Staged& st, const int step, const int item) {
        // uniform address of the step plus the lane's 32-bit offset (passed through an empty asm statement: otherwise
        // "base + lane offset" is hoisted out of the loop as a 64-bit register pair per load, and added to per step)
        if (item < kBgXPer) {
            asm volatile("" : "+v"(xsrc[item]));
            st.xg[item] = *(const u32x4*)(xbase + (int64_t)step * kBgRowBytes + xsrc[item]);
        } else if (item < kBgXPer + kBgWPer) {
            asm volatile("" : "+v"(wsrc[item - kBgXPer]));
            st.wg[item - kBgXPer] = *(const u32x4*)(wbase + (int64_t)step * kWStep + wsrc[item - kBgXPer]);
        } else {
            fetch_signs(st, step);
        }
    };
    auto stage_item = [&](const Staged& st, const int buf, const int item) {
        if (item < kBgXPer) lds_put<u32x4>(xdst[item] + buf * Lds::kXStride, st.xg[item]);
        else if (item < kBgXPer + kBgWPer) lds_put<u32x4>(wdst[item - kBgXPer] + buf * Lds::kWStride, st.wg[item - kBgXPer]);
        else if (TILED) {
            // su[g] = (byte of slice v, byte of slice v + 1) of lane g: the row's words are (v: g = 0..3), (v + 1: g = 0..3)
            const uint32_t lo = st.su[0] | (st.su[1] << 16), hi = st.su[2] | (st.su[3] << 16);
            lds_put<u32x2>(sdst + buf * Lds::kSStride,
                           u32x2{__builtin_amdgcn_perm(hi, lo, 0x06040200u), __builtin_amdgcn_perm(hi, lo, 0x07050301u)});
        } else if (WM == 1) lds_put<u32x2>(sdst + buf * Lds::kSStride, u32x2{st.s0, st.s1});
        else lds_put<uint32_t>(sdst + buf * Lds::kSStride, st.s0);
    };
    auto fetch = [&](Staged& st, const int step) {
#pragma unroll
        for (int it = 0; it < kItems; ++it) fetch_item(st, step, it);
    };
    auto stage = [&](const Staged& st, const int buf) {
#pragma unroll
        for (int it = 0; it < kItems; ++it) stage_item(st, buf, it);
    };

    float16v accb[MI][2], accd[MI][2];   // [token block of 32][feature block of 32]
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) accb[i][j][e] = accd[i][j][e] = 0.f;

    // Operand of k slice s (16 k): lane (l % 32, l / 32) reads row base + l % 32, chunk 2 s + l / 32; the swizzle
    // mask (row / 2) % 8 depends on the lane only.
    const int r32 = lane & 31, hi = lane >> 5;
    const int mask = (r32 >> 1) & 7;
    lds_bytes xrd[4], wrd[4];   // this lane's x and W operand of k slice sl in buffer 0
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
        const int cho = ((2 * sl + hi) ^ mask) << 4;
        xrd[sl] = lds_at((wm * kWaveM + r32) * kBgRowBytes + cho);
        wrd[sl] = lds_at(Lds::kWBase + (wn * 64 + r32) * kBgRowBytes + cho);
        asm volatile("" : "+v"(xrd[sl]), "+v"(wrd[sl]));
    }
    const lds_bytes srd = lds_at(Lds::kSBase + (wn * 64 + r32) * 8);
    half8 a[2][MI], bw[2][2], bs[2][2];   // operands of two k slices: one being multiplied, one being read
    u32x2 sw[2];                         // this lane's row of the 2 feature blocks: the step's 8 sign bytes each
    auto read_signs = [&](const int buf) {
#pragma unroll
        for (int j = 0; j < 2; ++j) sw[j] = lds_get<u32x2>(srd + buf * Lds::kSStride + j * 32 * 8);
    };
    // The MI + 4 operand reads of a k slice, in the order the MFMAs of the slice need them.
    constexpr int kReads = MI + 4;
    const uint32_t sh[2] = {8u * hi, 16u + 8u * hi};   // bit position of the lane's sign byte in the word: slice 2 w + (0 | 1)
    auto read_item = [&](const int buf, const int sl, const int set, const int r) {
        const int b = buf * kBgBufBytes;   // (128 rows: the stride of every region)
        // r: 0 W(0), 1 signs(0), 2 x(0), 3 W(1), 4 signs(1), 5.. x(1..)
        if (r == 0 || r == 3) {
            const int j = r / 3;
            bw[set][j] = lds_get<half8>(wrd[sl] + (b + j * 32 * kBgRowBytes));
        } else if (r == 1 || r == 4) {
            const int j = r / 3;
            const uint32_t byte = __builtin_amdgcn_ubfe(sl < 2 ? sw[j][0] : sw[j][1], sh[sl & 1], 8u);   // byte 2 sl + hi of the row's 8
            bs[set][j] = lds_get<half8>(lut_lane + byte * Lds::kLutEntry);
        } else {
            const int i = r == 2 ? 0 : r - 4;
            a[set][i] = lds_get<half8>(xrd[sl] + (b + i * 32 * kBgRowBytes));
        }
    };
    auto read_slice = [&](const int buf, const int sl, const int set) {
#pragma unroll
        for (int r = 0; r < kReads; ++r) read_item(buf, sl, set, r);
    };

    // MERGED.  The MFMAs of a slice run feature block 0 first (slots 0 .. MI-1), then block 1 (slots MI .. 2 MI-1).
    // Behind the first slots the next slice's W(0), signs(0), W(1), signs(1) are read (8 token blocks: behind every
    // other one); behind slot MI + i, the last one that uses x operand i, that operand of the next slice.  W(0) +
    // signs(0) of the next slice are added up in the second half of this slice and W(1) + signs(1) in the first
    // half of the next one.  With 8 token blocks the step's LDS writes and global loads alternate over the slots
    // 0 .. 2 kItems - 1, so that no slot carries more than one of them.
    auto read_item_m = [&](const int buf, const int sl, const int set, const int r) {
        if (r < 4) {
            const int j = r >> 1;
            if ((r & 1) == 0) {
                bw[set][j] = lds_get<half8>(wrd[sl] + (buf * Lds::kWStride + j * 32 * kBgRowBytes));
            } else {
                const uint32_t byte = __builtin_amdgcn_ubfe(sl < 2 ? sw[j][0] : sw[j][1], sh[sl & 1], 8u);
                bs[set][j] = lds_get<half8>(lut_lane + byte * Lds::kLutEntry);
            }
        } else {
            // one set of x operands: a[i] is read again right behind the last MFMA of the slice that uses it
            a[0][r - 4] = lds_get<half8>(xrd[sl] + (buf * Lds::kXStride + (r - 4) * 32 * kBgRowBytes));
        }
    };
    auto merge_word = [&](const int set, const int j, const int m) {   // one packed addition
        const half2v sum = half2v{bw[set][j][2 * m], bw[set][j][2 * m + 1]} + half2v{bs[set][j][2 * m], bs[set][j][2 * m + 1]};
        bw[set][j][2 * m] = sum[0];
        bw[set][j][2 * m + 1] = sum[1];
    };

    // While step `step` is multiplied, the tiles of step + 1 (in `next`) go into the other buffer and `next` is
    // refilled with step + 1 + kSets -- one LDS write or one global load behind every other MFMA, so that the
    // wavefronts do not queue up at the LDS and at the address unit while their matrix pipes idle.  On entry the
    // operands of slice 0 are in operand set 0 (read behind the previous step's barrier).
    // pairs of MFMAs between an item's LDS write and its next load: where the step is long enough, all the writes
    // first and then all the loads, so that no pair carries both
    constexpr int kLagMax = 4 * MI * 2 - kItems, kLag = kLagMax < kItems ? kLagMax : kItems;
    static_assert(kLag >= 1, "an item is written out before it is fetched again");
    static_assert(kItems <= 3 * MI * 2 && kItems - 1 + kLag < 4 * MI * 2, "all items are staged before the barrier slice and fetched within the step");
    auto do_step = [&](const int step, const int buf, Staged& next) {
        const int step3 = step + 1 + kSets < last ? step + 1 + kSets : last;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {                        // k slice: 16 MFMAs
            const int cur = sl & 1;
            if (sl == 3) {
                // every read of this buffer has been issued (its last slice sits in operand set 1) and every item of
                // step + 1 has been written: the other buffer is complete once all wavefronts are here
                bg_barrier();
                read_signs(buf ^ 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    // A wavefront alone on its SIMD issues in order, an instruction every 8 cycles or so: what follows an
                    // MFMA must fit into its 32 cycles, or the next MFMA starts late.  Behind the first MFMA of pair q of
                    // the slice: its share of the next slice's operand reads; behind the second: one LDS write, one load.
                    mfma_in_place(accb[i][j], a[cur][i], bw[cur][j]);
                    const int q = i * 2 + j;
#pragma unroll
                    for (int r = q * kReads / (MI * 2); r < (q + 1) * kReads / (MI * 2); ++r) {
                        if (sl < 3) read_item(buf, sl + 1, cur ^ 1, r);
                        else read_item(buf ^ 1, 0, 0, r);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_in_place(accd[i][j], a[cur][i], bs[cur][j]);
                    // pair p of the step: item p leaves for LDS after pair p, and is fetched again after pair p + kLag
                    const int p = sl * MI * 2 + q;
                    if (p < kItems) stage_item(next, buf ^ 1, p);
                    if (p >= kLag && p - kLag < kItems) fetch_item(next, step3, p - kLag);
                    __builtin_amdgcn_sched_barrier(0);
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    auto do_step_merged = [&](const int step, const int buf, Staged& next) {
        const int step3 = step + 1 + kSets < last ? step + 1 + kSets : last;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {                        // k slice: 2 MI MFMAs
            const int cur = sl & 1;
            if (sl == 3) {
                bg_barrier();
                read_signs(buf ^ 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    // through the builtin: the compiler keeps the distance that the matrix cores need behind the packed
                    // additions that write bw
                    accb[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], bw[cur][j], accb[i][j], 0, 0, 0);
                    const int q = j * MI + i;   // slot of the slice
                    // reads of the next slice's operands
                    const int r_lo = q >= MI ? 4 + q - MI : (MI == 2 ? 2 * q : (MI == 4 ? q : q / 2));
                    const int r_hi = q >= MI ? r_lo + 1 : (MI == 2 ? r_lo + 2 : (MI == 4 || (q & 1) == 0 ? r_lo + 1 : r_lo));
#pragma unroll
                    for (int r = r_lo; r < r_hi; ++r) {
                        if (sl < 3) read_item_m(buf, sl + 1, cur ^ 1, r);
                        else read_item_m(buf ^ 1, 0, 0, r);
                    }
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        if (q == m * MI / 4) merge_word(cur, 1, m);              // this slice's feature block 1
                        if (q == MI + m * MI / 4) merge_word(cur ^ 1, 0, m);     // the next slice's feature block 0
                    }
                    const int p = sl * MI * 2 + q;
                    if constexpr (MI == 8) {
                        static_assert(MI != 8 || 2 * kItems <= 3 * MI * 2, "all items are staged before the barrier slice");
                        if ((p & 1) == 0 && p / 2 < kItems) stage_item(next, buf ^ 1, p / 2);
                        if ((p & 1) == 1 && p / 2 < kItems) fetch_item(next, step3, p / 2);
                    } else {
                        if (p < kItems) stage_item(next, buf ^ 1, p);
                        if (p >= kLag && p - kLag < kItems) fetch_item(next, step3, p - kLag);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    stage(set0, 0);   // both sets were requested at the top
    fetch(set0, kSets < last ? kSets : last);
    bg_barrier();       // the table and the tiles of step 0 are complete
    read_signs(0);
    int step = 0;
    if constexpr (MERGED) {
#pragma unroll
        for (int r = 0; r < kReads; ++r) read_item_m(0, 0, 0, r);
#pragma unroll
        for (int m = 0; m < 4; ++m) merge_word(0, 0, m);
        for (; step + 1 < n_steps; step += 2) {
            do_step_merged(step, 0, kSets == 2 ? set1 : set0);
            do_step_merged(step + 1, 1, set0);
        }
        if (step < n_steps) do_step_merged(step, 0, kSets == 2 ? set1 : set0);
    } else {
        read_slice(0, 0, 0);
        for (; step + 1 < n_steps; step += 2) {
            do_step(step, 0, kSets == 2 ? set1 : set0);
            do_step(step + 1, 1, set0);
        }
        if (step < n_steps) do_step(step, 0, kSets == 2 ? set1 : set0);
    }

    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMAs have left the pipe before their results are read
    // Every wavefront has passed the last step's barrier, so nobody reads the tiles or the table any more (the
    // operand reads issued behind that barrier fetch a step that does not exist; their results are never used).
    // 32 x 32 result tile (i, j), element e of a lane: token row 32 i + 8 (e / 4) + 4 (l / 32) + e % 4, feature
    // 32 j + l % 32 of the wavefront's 64.  The rows go to LDS as fp16 and leave as whole 16-byte pieces: written
    // from the accumulator layout y would take 256 two-byte stores per lane.
    const lds_bytes orow = lds_at(wave * (kWaveM * kBgOutRowBytes));
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = 32 * i + 8 * (e >> 2) + 4 * hi + (e & 3);
                lds_put<uint16_t>(orow + row * kBgOutRowBytes + (32 * j + r32) * 2,
                                  f2h_rne(MERGED ? accb[i][j][e] : accb[i][j][e] + alpha * accd[i][j][e]));
            }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const bool whole = (out & 7) == 0;   // rows of y start on 16-byte boundaries
#pragma unroll 4
    for (int it = 0; it < kWaveM * 8 / 64; ++it) {
        const int q = it * 64 + lane, row = q >> 3, piece = q & 7;
        const int tok = lds_get<int>(lds_at(2 * kBgBufBytes + kBgLutBytes + (wm * kWaveM + row) * 4));
        const u32x4 v = lds_get<u32x4>(orow + row * kBgOutRowBytes + piece * 16);
        const int64_t n = n0 + wn * 64 + piece * 8;
        if (tok < 0 || n >= out) continue;
        uint16_t* const dst = y + (int64_t)tok * out + n;
        if (whole) {
            *(u32x4*)dst = v;
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (n + k < out) dst[k] = (uint16_t)(v[k >> 1] >> (16 * (k & 1)));
        }
    }
}

// Launch order -> tile.  Tiles are numbered in panels of 8 N tiles, row-major inside, and an XCD takes chunks of 32
// consecutive numbers, so that the workgroups it runs together form a compact block of tiles.  The tiles from n_full
// on are run as two workgroups of half a tile each (n_full = all of them: none).  Returns false for a surplus workgroup.
__device__ __forceinline__ bool bg_tile_of_block(const int n_mtiles, const int n_ntiles, const int n_full, int* mt, int* nt,
                                                 int* half) {
    const int L = blockIdx.x, xcd = L % kBgXcds, slot = L / kBgXcds;
    const int chunk = (slot / kBgChunk) * kBgXcds + xcd;
    const int v = chunk * kBgChunk + slot % kBgChunk;
    const int n_tiles = n_mtiles * n_ntiles;
    if (v >= n_full + 2 * (n_tiles - n_full)) return false;
    const int t = v < n_full ? v : n_full + ((v - n_full) >> 1);
    const int per_panel = n_mtiles * kBgPanel;
    const int panel = t / per_panel, tp = t - panel * per_panel;
    const int width = n_ntiles - panel * kBgPanel < kBgPanel ? n_ntiles - panel * kBgPanel : kBgPanel;
    *mt = tp / width;
    *nt = panel * kBgPanel + tp % width;
    *half = v < n_full ? -1 : (v - n_full) & 1;
    return true;
}

template <int WM, bool TILED>
__global__ __launch_bounds__(256 * WM, 1) void linear_prefill_big_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, const int32_t* __restrict__ row_token, const int32_t* __restrict__ tile_tenant,
    uint16_t* __restrict__ y, const int64_t out, const int64_t in, const int n_mtiles, const int n_ntiles, const int n_full) {
    int mt, nt, half;
    if (!bg_tile_of_block(n_mtiles, n_ntiles, n_full, &mt, &nt, &half)) return;
    const int32_t* const tile_tokens = row_token + mt * kBgM;
    if constexpr (WM == 1) {
        if (half >= 0) {
            prefill_big_tile<1, kBgM / 2, false, TILED>(x, w, packed_by_tenant, alpha_by_tenant, tile_tokens, tile_tenant, y, out, in, mt, nt,
                                                 half * (kBgM / 2));
            return;
        }
    }
    prefill_big_tile<WM, kBgM, false, TILED>(x, w, packed_by_tenant, alpha_by_tenant, tile_tokens, tile_tenant, y, out, in, mt, nt, 0);
}

// The merged form on token tiles of 256 rows (row_token holds 256 entries per tile): a wavefront multiplies 256
// tokens x 64 features per operand of W that it reads, looks up and adds, which is what lets the matrix cores run
// most of the time although every such operand costs eight instructions.  A tile whose upper 128 rows are empty (a
// tenant's last tile; the rows of a tile are filled from the top) runs as 128 rows; the tiles from n_full on run as
// two workgroups of 128 rows each.
template <bool TILED>
__global__ __launch_bounds__(256, 1) void linear_prefill_merged_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, const int32_t* __restrict__ row_token, const int32_t* __restrict__ tile_tenant,
    uint16_t* __restrict__ y, const int64_t out, const int64_t in, const int n_mtiles, const int n_ntiles, const int n_full) {
    int mt, nt, half;
    if (!bg_tile_of_block(n_mtiles, n_ntiles, n_full, &mt, &nt, &half)) return;
    const int32_t* const tile_tokens = row_token + mt * kMergedTile;
    if (half >= 0 || tile_tokens[kBgM] < 0) {
        const int r0 = half > 0 ? kBgM : 0;
        if (tile_tokens[r0] < 0) return;   // nothing in this half
        prefill_big_tile<1, kBgM, true, TILED>(x, w, packed_by_tenant, alpha_by_tenant, tile_tokens, tile_tenant, y, out, in, mt, nt, r0);
        return;
    }
    prefill_big_tile<1, kMergedTile, true, TILED>(x, w, packed_by_tenant, alpha_by_tenant, tile_tokens, tile_tenant, y, out, in, mt, nt, 0);
}

// T: rows of x (its byte offsets and those inside one 256-row band of W must fit 32 bits)
bool prefill_big_fits(int64_t T, int64_t out, int64_t in) {
    return in >= kBgK && in % kBgK == 0 && out >= 1 && (uint64_t)T * (uint64_t)in * 2 < ((uint64_t)1 << 32) &&
           (uint64_t)kBgN * (uint64_t)in * 2 < ((uint64_t)1 << 32);
}

namespace {

// One workgroup per compute unit at a time: when the last round of tiles would keep at most half of the units
// busy, its tiles are cut in two, which takes little more than half the time of a round.
hipError_t whole_tiles(int64_t tiles, bool halve_last_round, int64_t* n_full) {
    *n_full = tiles;
    if (!halve_last_round) return hipSuccess;
    int cus = 0;
    const hipError_t ec = device_cu_count(&cus);
    if (ec != hipSuccess) return ec;
    const int64_t r = tiles % cus;
    if (r != 0 && 2 * r <= cus) *n_full = tiles - r;
    return hipSuccess;
}

template <typename Kernel>
hipError_t launch_tiles(Kernel kernel, PerDeviceOnce& lds_limit, int lds_bytes, int threads, const uint16_t* x, const uint16_t* w,
                        const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant, const int32_t* row_token,
                        const int32_t* tile_tenant, int n_mtiles, int n_ntiles, uint16_t* y, int64_t out, int64_t in,
                        bool halve_last_round, hipStream_t st) {
    const hipError_t ea = lds_limit.run([&] {
        hipFuncAttributes fa;
        const hipError_t e = hipFuncGetAttributes(&fa, (const void*)kernel);
        if (e != hipSuccess) return e;
        if (fa.sharedSizeBytes != 0) return hipErrorInvalidValue;   // the kernel addresses its dynamic LDS from 0
        return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    if (ea != hipSuccess) return ea;
    const int64_t tiles = (int64_t)n_mtiles * n_ntiles, round = (int64_t)kBgChunk * kBgXcds;
    int64_t n_full = tiles;
    const hipError_t ew = whole_tiles(tiles, halve_last_round, &n_full);
    if (ew != hipSuccess) return ew;
    const int64_t n_virtual = n_full + 2 * (tiles - n_full);
    const unsigned grid = (unsigned)((n_virtual + round - 1) / round * round);   // surplus workgroups return at once
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), lds_bytes, st, x, w, packed_by_tenant, alpha_by_tenant, row_token,
                       tile_tenant, y, out, in, n_mtiles, n_ntiles, (int)n_full);
    return hipGetLastError();
}

}  // namespace

// waves: 4 (one wavefront per SIMD) or 8 (two); row_token: 128 entries per token tile; tiled (4 wavefronts only): w and
// the tenants' signs in the serving layout
hipError_t launch_linear_prefill_big(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                     const float* alpha_by_tenant, const int32_t* row_token, const int32_t* tile_tenant,
                                     int n_mtiles, uint16_t* y, int64_t T, int64_t out, int64_t in, int waves, bool halve_last_round,
                                     bool tiled, hipStream_t st) {
    if (!prefill_big_fits(T, out, in) || (waves != 4 && waves != 8) || (tiled && waves != 4)) return hipErrorInvalidValue;
    const int n_ntiles = (int)((out + kBgN - 1) / kBgN);
    const int64_t tiles = (int64_t)n_mtiles * n_ntiles;
    if (tiles < 1 || tiles > (int64_t)1 << 30) return hipErrorInvalidValue;
    static PerDeviceOnce once4, once8, once4t;
    if (tiled)
        return launch_tiles(linear_prefill_big_kernel<1, true>, once4t, kBgLdsBytes, 256, x, w, packed_by_tenant, alpha_by_tenant,
                            row_token, tile_tenant, n_mtiles, n_ntiles, y, out, in, halve_last_round, st);
    if (waves == 4)
        return launch_tiles(linear_prefill_big_kernel<1, false>, once4, kBgLdsBytes, 256, x, w, packed_by_tenant, alpha_by_tenant,
                            row_token, tile_tenant, n_mtiles, n_ntiles, y, out, in, halve_last_round, st);
    return launch_tiles(linear_prefill_big_kernel<2, false>, once8, kBgLdsBytes, 512, x, w, packed_by_tenant, alpha_by_tenant, row_token,
                        tile_tenant, n_mtiles, n_ntiles, y, out, in, false, st);
}

// One product on W + alpha S (formed in fp16 on the way to the matrix cores); row_token: kPrefillMergedTile = 256
// entries per token tile.
hipError_t launch_linear_prefill_merged(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                        const float* alpha_by_tenant, const int32_t* row_token, const int32_t* tile_tenant,
                                        int n_mtiles, uint16_t* y, int64_t T, int64_t out, int64_t in, bool halve_last_round,
                                        bool tiled, hipStream_t st) {
    if (!prefill_big_fits(T, out, in)) return hipErrorInvalidValue;
    const int n_ntiles = (int)((out + kBgN - 1) / kBgN);
    const int64_t tiles = (int64_t)n_mtiles * n_ntiles;
    if (tiles < 1 || tiles > (int64_t)1 << 30) return hipErrorInvalidValue;
    static PerDeviceOnce once, once_t;
    if (tiled)
        return launch_tiles(linear_prefill_merged_kernel<true>, once_t, BgLds<kMergedTile>::kTotal, 256, x, w, packed_by_tenant,
                            alpha_by_tenant, row_token, tile_tenant, n_mtiles, n_ntiles, y, out, in, halve_last_round, st);
    return launch_tiles(linear_prefill_merged_kernel<false>, once, BgLds<kMergedTile>::kTotal, 256, x, w, packed_by_tenant, alpha_by_tenant,
                        row_token, tile_tenant, n_mtiles, n_ntiles, y, out, in, halve_last_round, st);
}

}  // namespace bd
