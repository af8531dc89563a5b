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
#include "bd_device.h"
#include "bd_launch.h"

namespace bd {

namespace {

constexpr int kBgM = 128, kBgN = 256, kBgK = 64;
constexpr int kBgRowBytes = kBgK * 2;                    // 128
constexpr int kBgXBytes = kBgM * kBgRowBytes;            // 16384
constexpr int kBgWBytes = kBgN * kBgRowBytes;            // 32768
constexpr int kBgSBytes = kBgN * 8;                      // 2048
constexpr int kBgBufBytes = kBgXBytes + kBgWBytes + kBgSBytes;
constexpr int kBgLutBytes = 256 * 8 * 16;
constexpr int kBgTokBytes = kBgM * 4;                    // the tile's token of every row
constexpr int kBgLdsBytes = 2 * kBgBufBytes + kBgLutBytes + kBgTokBytes;   // 135680
// Epilogue: a wavefront's rows of y as fp16, 64 features + 16 B of padding each (rows 4 apart, which one LDS
// instruction writes together, then fall into different banks), in the tile buffers, which are free by then.
constexpr int kBgOutRowBytes = 64 * 2 + 16;
static_assert(kBgM * kBgOutRowBytes * 4 <= 2 * kBgBufBytes, "the result rows of all wavefronts fit the tile buffers");
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

// One tile: TM token rows r0 .. r0 + TM of the 128-row token tile mt, output features 256 nt .. + 256.
// WM = 1: 4 wavefronts (1 x 4), each TM tokens x 64 features, alone on its SIMD; two sets of staging registers
// (loads two steps ahead).  WM = 2: 8 wavefronts (2 x 4), each TM / 2 x 64, two per SIMD; one set (one step ahead).
// TM = 128, or 64 (WM = 1 only): half a tile, for the tiles of a last round that would leave most units idle.
template <int WM, int TM>
__device__ __forceinline__ void prefill_big_tile(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, const int32_t* __restrict__ row_token, const int32_t* __restrict__ tile_tenant,
    uint16_t* __restrict__ y, const int64_t out, const int64_t in, const int mt, const int nt, const int r0) {
    extern __shared__ __align__(16) unsigned char lds[];   // [2 buffers: x, W, sign words][table][tokens]
    unsigned char* const lut = lds + 2 * kBgBufBytes;

    constexpr int kThreads = 256 * WM, kWaveM = TM / WM, MI = kWaveM / 32;
    // mfma_in_place hides the accumulators from the compiler's hazard bookkeeping, so the schedule itself has to keep
    // an accumulator's uses apart.  A k slice issues, for every (i, j), one MFMA into accb[i][j] and one into accd[i][j]:
    // 4 MI MFMAs, each accumulator once, always in the same order, so 4 MI - 1 other MFMAs (each 8 passes = 32 cycles of
    // the matrix pipe) lie between two uses of one accumulator.  The dependent-accumulate hazard of the 8-pass
    // instructions is below 20 cycles; 7 MFMAs (MI = 2: 64-row halves, or two wavefronts per SIMD) are 224.
    // The epilogue reads the accumulators with vector instructions after two `s_nop 15` (32 wait states; the rule for
    // reading the result of an 8-pass MFMA asks for 18).  Every instantiation has a full-output parity test.
    constexpr int kMfmasBetweenUses = 4 * MI - 1;
    static_assert(MI == 2 || MI == 4, "the slice schedule below is written for 2 or 4 token blocks per wavefront");
    static_assert(kMfmasBetweenUses >= 7, "an accumulator would be used again while its last MFMA may still be in the pipe");
    constexpr int kBgXPer = TM * 8 / kThreads, kBgWPer = kBgN * 8 / kThreads;   // 16-byte chunks per thread and step
    constexpr int kSets = WM == 1 ? 2 : 1;
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
    const unsigned char* const wbase = (const unsigned char*)(w + n0 * in);
    uint32_t xsrc[kBgXPer], wsrc[kBgWPer];
    lds_bytes xdst[kBgXPer], wdst[kBgWPer];   // in buffer 0
    struct Staged {
        u32x4 xg[kBgXPer], wg[kBgWPer];
        uint32_t s0, s1;
    };
    Staged set0, set1;
    const int step_b = 1 < last ? 1 : last;   // what the second set holds first
#pragma unroll
    for (int i = 0; i < kBgWPer; ++i) {
        const int q = tid + kThreads * i, row = q >> 3, c8 = q & 7;
        const int64_t wrow = n0 + row < out ? row : out - 1 - n0;
        wsrc[i] = (uint32_t)(wrow * in * 2) + c8 * 16;
        wdst[i] = lds_at(kBgXBytes + bg_off(row, c8));
        asm volatile("" : "+v"(wdst[i]));   // a register of its own: derived from xdst[i], it would cost an addition per use
        set0.wg[i] = *(const u32x4*)(wbase + wsrc[i]);
    }
    const int tenant = tile_tenant[mt];
    int tokv[kBgXPer];
#pragma unroll
    for (int i = 0; i < kBgXPer; ++i) tokv[i] = row_token[mt * kBgM + r0 + ((tid + kThreads * i) >> 3)];
    if (kSets == 2) {
#pragma unroll
        for (int i = 0; i < kBgWPer; ++i) set1.wg[i] = *(const u32x4*)(wbase + (int64_t)step_b * kBgRowBytes + wsrc[i]);
    }
    __builtin_amdgcn_sched_barrier(0);

    // byte -> 8 fp16 (+1.0 where the bit is set, else -1.0), element e = bit e; entry [byte][copy].  Consecutive lanes
    // write consecutive 16-byte copies (a wavefront 1 KiB at a stretch; a lane per entry would put its writes 128
    // bytes apart, several of them on every bank).
    for (int q = tid; q < 256 * 8; q += kThreads) {
        const uint32_t bb = (uint32_t)q >> 3;
        u32x4 e;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            e[i] = 0xBC00BC00u ^ (((bb >> (2 * i)) & 1u) << 15) ^ (((bb >> (2 * i + 1)) & 1u) << 31);
        *(u32x4*)(lut + q * 16) = e;
    }
    const lds_bytes lut_lane = lds_at(2 * kBgBufBytes + (lane & 7) * 16);
    __builtin_amdgcn_sched_barrier(0);

    const float alpha = alpha_by_tenant[tenant];
    // sign words: 256 threads take a row's two words each, 512 threads one word each
    const int s_row = WM == 1 ? tid : tid >> 1, s_word = WM == 1 ? 0 : tid & 1;
    const int64_t srow = n0 + s_row < out ? n0 + s_row : out - 1;
    const bg_global_words ssrc = (bg_global_words)(packed_by_tenant[tenant] + srow * words_per_row) + s_word;
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
    set0.s0 = ssrc[0];
    if (WM == 1) set0.s1 = ssrc[1];
    if (kSets == 2) {
        set1.s0 = ssrc[2 * step_b];
        if (WM == 1) set1.s1 = ssrc[2 * step_b + 1];
    }

    const lds_bytes sdst = lds_at(kBgXBytes + kBgWBytes + tid * (WM == 1 ? 8 : 4));
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
            st.wg[item - kBgXPer] = *(const u32x4*)(wbase + (int64_t)step * kBgRowBytes + wsrc[item - kBgXPer]);
        } else {
            st.s0 = ssrc[2 * step];
            if (WM == 1) st.s1 = ssrc[2 * step + 1];
        }
    };
    auto stage_item = [&](const Staged& st, const int buf, const int item) {
        const int b = buf * kBgBufBytes;
        if (item < kBgXPer) lds_put<u32x4>(xdst[item] + b, st.xg[item]);
        else if (item < kBgXPer + kBgWPer) lds_put<u32x4>(wdst[item - kBgXPer] + b, st.wg[item - kBgXPer]);
        else if (WM == 1) lds_put<u32x2>(sdst + b, u32x2{st.s0, st.s1});
        else lds_put<uint32_t>(sdst + b, st.s0);
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
        wrd[sl] = lds_at(kBgXBytes + (wn * 64 + r32) * kBgRowBytes + cho);
        asm volatile("" : "+v"(xrd[sl]), "+v"(wrd[sl]));
    }
    const lds_bytes srd = lds_at(kBgXBytes + kBgWBytes + (wn * 64 + r32) * 8);
    half8 a[2][MI], bw[2][2], bs[2][2];   // operands of two k slices: one being multiplied, one being read
    u32x2 sw[2];                         // this lane's row of the 2 feature blocks: the step's 8 sign bytes each
    auto read_signs = [&](const int buf) {
#pragma unroll
        for (int j = 0; j < 2; ++j) sw[j] = lds_get<u32x2>(srd + buf * kBgBufBytes + j * 32 * 8);
    };
    // The MI + 4 operand reads of a k slice, in the order the MFMAs of the slice need them.
    constexpr int kReads = MI + 4;
    const uint32_t sh[2] = {8u * hi, 16u + 8u * hi};   // bit position of the lane's sign byte in the word: slice 2 w + (0 | 1)
    auto read_item = [&](const int buf, const int sl, const int set, const int r) {
        const int b = buf * kBgBufBytes;
        // r: 0 W(0), 1 signs(0), 2 x(0), 3 W(1), 4 signs(1), 5.. x(1..)
        if (r == 0 || r == 3) {
            const int j = r / 3;
            bw[set][j] = lds_get<half8>(wrd[sl] + (b + j * 32 * kBgRowBytes));
        } else if (r == 1 || r == 4) {
            const int j = r / 3;
            const uint32_t byte = __builtin_amdgcn_ubfe(sl < 2 ? sw[j][0] : sw[j][1], sh[sl & 1], 8u);   // byte 2 sl + hi of the row's 8
            bs[set][j] = lds_get<half8>(lut_lane + (byte << 7));
        } else {
            const int i = r == 2 ? 0 : r - 4;
            a[set][i] = lds_get<half8>(xrd[sl] + (b + i * 32 * kBgRowBytes));
        }
    };
    auto read_slice = [&](const int buf, const int sl, const int set) {
#pragma unroll
        for (int r = 0; r < kReads; ++r) read_item(buf, sl, set, r);
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

    stage(set0, 0);   // both sets were requested at the top
    fetch(set0, kSets < last ? kSets : last);
    bg_barrier();       // the table and the tiles of step 0 are complete
    read_signs(0);
    read_slice(0, 0, 0);
    int step = 0;
    for (; step + 1 < n_steps; step += 2) {
        do_step(step, 0, kSets == 2 ? set1 : set0);
        do_step(step + 1, 1, set0);
    }
    if (step < n_steps) do_step(step, 0, kSets == 2 ? set1 : set0);

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
                lds_put<uint16_t>(orow + row * kBgOutRowBytes + (32 * j + r32) * 2, f2h_rne(accb[i][j][e] + alpha * accd[i][j][e]));
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
// on are run as two workgroups of half a tile each (n_full = all of them: none).
template <int WM>
__global__ __launch_bounds__(256 * WM, 1) void linear_prefill_big_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, const uint32_t* const* __restrict__ packed_by_tenant,
    const float* __restrict__ alpha_by_tenant, const int32_t* __restrict__ row_token, const int32_t* __restrict__ tile_tenant,
    uint16_t* __restrict__ y, const int64_t out, const int64_t in, const int n_mtiles, const int n_ntiles, const int n_full) {
    const int L = blockIdx.x, xcd = L % kBgXcds, slot = L / kBgXcds;
    const int chunk = (slot / kBgChunk) * kBgXcds + xcd;
    const int v = chunk * kBgChunk + slot % kBgChunk;
    const int n_tiles = n_mtiles * n_ntiles;
    if (v >= n_full + 2 * (n_tiles - n_full)) return;
    const int t = v < n_full ? v : n_full + ((v - n_full) >> 1);
    const int per_panel = n_mtiles * kBgPanel;
    const int panel = t / per_panel, tp = t - panel * per_panel;
    const int width = n_ntiles - panel * kBgPanel < kBgPanel ? n_ntiles - panel * kBgPanel : kBgPanel;
    const int mt = tp / width, nt = panel * kBgPanel + tp % width;
    if constexpr (WM == 1) {
        if (v >= n_full) {
            prefill_big_tile<1, kBgM / 2>(x, w, packed_by_tenant, alpha_by_tenant, row_token, tile_tenant, y, out, in, mt, nt,
                                          ((v - n_full) & 1) * (kBgM / 2));
            return;
        }
    }
    prefill_big_tile<WM, kBgM>(x, w, packed_by_tenant, alpha_by_tenant, row_token, tile_tenant, y, out, in, mt, nt, 0);
}

// T: rows of x (its byte offsets and those inside one 256-row band of W must fit 32 bits)
bool prefill_big_fits(int64_t T, int64_t out, int64_t in) {
    return in >= kBgK && in % kBgK == 0 && out >= 1 && (uint64_t)T * (uint64_t)in * 2 < ((uint64_t)1 << 32) &&
           (uint64_t)kBgN * (uint64_t)in * 2 < ((uint64_t)1 << 32);
}

template <int WM>
static hipError_t launch_big_t(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                               const float* alpha_by_tenant, const int32_t* row_token, const int32_t* tile_tenant,
                               int n_mtiles, int n_ntiles, uint16_t* y, int64_t out, int64_t in, bool halve_last_round,
                               hipStream_t st) {
    auto kernel = linear_prefill_big_kernel<WM>;
    static PerDeviceOnce lds_limit;
    const hipError_t ea = lds_limit.run([&] {
        hipFuncAttributes fa;
        const hipError_t e = hipFuncGetAttributes(&fa, (const void*)kernel);
        if (e != hipSuccess) return e;
        if (fa.sharedSizeBytes != 0) return hipErrorInvalidValue;   // the kernel addresses its dynamic LDS from 0
        return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kBgLdsBytes);
    });
    if (ea != hipSuccess) return ea;
    const int64_t tiles = (int64_t)n_mtiles * n_ntiles, round = (int64_t)kBgChunk * kBgXcds;
    // One workgroup per compute unit at a time: when the last round of tiles would keep at most half of the units
    // busy, its tiles are cut in two (64 token rows each), which takes little more than half the time of a round.
    int64_t n_full = tiles;
    if (WM == 1 && halve_last_round) {
        int cus = 0;
        const hipError_t ec = device_cu_count(&cus);
        if (ec != hipSuccess) return ec;
        const int64_t r = tiles % cus;
        if (r != 0 && 2 * r <= cus) n_full = tiles - r;
    }
    const int64_t n_virtual = n_full + 2 * (tiles - n_full);
    const unsigned grid = (unsigned)((n_virtual + round - 1) / round * round);   // surplus workgroups return at once
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256 * WM), kBgLdsBytes, st, x, w, packed_by_tenant, alpha_by_tenant, row_token,
                       tile_tenant, y, out, in, n_mtiles, n_ntiles, (int)n_full);
    return hipGetLastError();
}

// waves: 4 (one wavefront per SIMD) or 8 (two)
hipError_t launch_linear_prefill_big(const uint16_t* x, const uint16_t* w, const uint32_t* const* packed_by_tenant,
                                     const float* alpha_by_tenant, const int32_t* row_token, const int32_t* tile_tenant,
                                     int n_mtiles, uint16_t* y, int64_t T, int64_t out, int64_t in, int waves, bool halve_last_round,
                                     hipStream_t st) {
    if (!prefill_big_fits(T, out, in) || (waves != 4 && waves != 8)) return hipErrorInvalidValue;
    const int n_ntiles = (int)((out + kBgN - 1) / kBgN);
    const int64_t tiles = (int64_t)n_mtiles * n_ntiles;
    if (tiles < 1 || tiles > (int64_t)1 << 30) return hipErrorInvalidValue;
    if (waves == 4)
        return launch_big_t<1>(x, w, packed_by_tenant, alpha_by_tenant, row_token, tile_tenant, n_mtiles, n_ntiles, y, out, in,
                               halve_last_round, st);
    return launch_big_t<2>(x, w, packed_by_tenant, alpha_by_tenant, row_token, tile_tenant, n_mtiles, n_ntiles, y, out, in, false, st);
}

}  // namespace bd
