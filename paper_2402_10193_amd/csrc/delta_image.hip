// Delta images: one tenant's compressed model (every matrix's sign planes and scales) as a single
// relocatable block of bytes -- the on-disk format and, unchanged, the staging buffer of a hot swap
// (Sec. 3.3 of the paper: a delta is small enough to be stored per tenant and loaded on demand).
//
// Everything in this file runs on the host except bd_delta_upload / bd_delta_install, which only
// enqueue copies and the re-tiling kernel.  Layout (little-endian), also stated in bitdelta.h:
//   0   char[8]  "BDLTv001"
//   8   u32      n_mats          12  u32  planes k
//   16  u64      total bytes     24  u64  sum of the payload's 64-bit words (mod 2^64)
//   32  entry[n_mats]: i64 out, i64 in, u64 packed_offset, u64 packed_bytes, u64 alpha_offset   (40 bytes each)
//   ..  f32 alpha[n_mats][k]
//   ..  (pad to 256)  payload: for every matrix, 256-byte aligned, u32 packed[k][out][in/32]
#include "bitdelta.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>

#include "bd_tiled.h"

namespace {

constexpr char kMagic[8] = {'B', 'D', 'L', 'T', 'v', '0', '0', '1'};
constexpr size_t kHeaderBytes = 32, kEntryBytes = 40, kAlign = 256;

struct Entry {
    int64_t out, in;
    uint64_t packed_offset, packed_bytes, alpha_offset;
};
static_assert(sizeof(Entry) == kEntryBytes, "entry layout");

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline bool shape_ok(int64_t out, int64_t in) {
    return out >= 0 && in >= 0 && in % 32 == 0 && out <= ((int64_t)1 << 31) && in <= ((int64_t)1 << 31);
}

template <typename T>
inline T get(const void* image, size_t off) {
    T v;
    std::memcpy(&v, (const unsigned char*)image + off, sizeof(T));
    return v;
}
template <typename T>
inline void put(void* image, size_t off, T v) {
    std::memcpy((unsigned char*)image + off, &v, sizeof(T));
}

inline size_t payload_begin(int32_t n_mats, int32_t k) {
    return round_up(kHeaderBytes + (size_t)n_mats * kEntryBytes + (size_t)n_mats * k * sizeof(float), kAlign);
}

uint64_t word_sum(const void* image, size_t begin, size_t end) {
    uint64_t s = 0;
    const unsigned char* p = (const unsigned char*)image;
    for (size_t o = begin; o + 8 <= end; o += 8) {
        uint64_t w;
        std::memcpy(&w, p + o, 8);
        s += w;
    }
    return s;
}

// Header and entry table consistent with `bytes`?  Fills n_mats / k.
bd_status parse(const void* image, size_t bytes, int32_t* n_mats, int32_t* k) {
    if (!image) return BD_ERR_NULL;
    if (bytes < kHeaderBytes || std::memcmp(image, kMagic, 8) != 0) return BD_ERR_FORMAT;
    const uint32_t nm = get<uint32_t>(image, 8), planes = get<uint32_t>(image, 12);
    if (nm < 1 || nm > BD_DELTA_MAX_MATS || planes < 1 || planes > BD_MAX_PLANES) return BD_ERR_FORMAT;
    if (get<uint64_t>(image, 16) != bytes) return BD_ERR_FORMAT;
    size_t cursor = payload_begin((int32_t)nm, (int32_t)planes);
    if (cursor > bytes) return BD_ERR_FORMAT;
    for (uint32_t m = 0; m < nm; ++m) {
        const Entry e = get<Entry>(image, kHeaderBytes + m * kEntryBytes);
        if (!shape_ok(e.out, e.in)) return BD_ERR_FORMAT;
        const uint64_t want = (uint64_t)planes * (uint64_t)e.out * (uint64_t)(e.in / 32) * 4;
        if (e.packed_bytes != want || e.packed_offset != cursor) return BD_ERR_FORMAT;
        if (e.alpha_offset != kHeaderBytes + nm * kEntryBytes + (size_t)m * planes * sizeof(float)) return BD_ERR_FORMAT;
        cursor = round_up(cursor + want, kAlign);
        if (cursor > bytes) return BD_ERR_FORMAT;
    }
    if (cursor != bytes) return BD_ERR_FORMAT;
    *n_mats = (int32_t)nm;
    *k = (int32_t)planes;
    return BD_OK;
}

}  // namespace

extern "C" {

size_t bd_delta_image_bytes(int32_t n_mats, const int64_t* out, const int64_t* in, int32_t k) {
    if (n_mats < 1 || n_mats > BD_DELTA_MAX_MATS || k < 1 || k > BD_MAX_PLANES || !out || !in) return 0;
    size_t total = payload_begin(n_mats, k);
    for (int32_t m = 0; m < n_mats; ++m) {
        if (!shape_ok(out[m], in[m])) return 0;
        total = round_up(total + (size_t)k * (size_t)out[m] * (size_t)(in[m] / 32) * 4, kAlign);
    }
    return total;
}

bd_status bd_delta_image_build(void* image, size_t image_bytes, int32_t n_mats, const int64_t* out, const int64_t* in,
                               int32_t k, const uint32_t* const* packed, const float* const* alpha) {
    if (!image || !out || !in || !packed || !alpha) return BD_ERR_NULL;
    const size_t need = bd_delta_image_bytes(n_mats, out, in, k);
    if (need == 0) return BD_ERR_SHAPE;
    if (image_bytes != need) return BD_ERR_WORKSPACE;
    std::memset(image, 0, payload_begin(n_mats, k));
    std::memcpy(image, kMagic, 8);
    put<uint32_t>(image, 8, (uint32_t)n_mats);
    put<uint32_t>(image, 12, (uint32_t)k);
    put<uint64_t>(image, 16, (uint64_t)need);
    size_t cursor = payload_begin(n_mats, k);
    const size_t alpha0 = kHeaderBytes + (size_t)n_mats * kEntryBytes;
    for (int32_t m = 0; m < n_mats; ++m) {
        const size_t pbytes = (size_t)k * (size_t)out[m] * (size_t)(in[m] / 32) * 4;
        if (!alpha[m] || (pbytes > 0 && !packed[m])) return BD_ERR_NULL;
        Entry e{out[m], in[m], (uint64_t)cursor, (uint64_t)pbytes, (uint64_t)(alpha0 + (size_t)m * k * sizeof(float))};
        put<Entry>(image, kHeaderBytes + (size_t)m * kEntryBytes, e);
        std::memcpy((unsigned char*)image + e.alpha_offset, alpha[m], (size_t)k * sizeof(float));
        if (pbytes > 0) std::memcpy((unsigned char*)image + cursor, packed[m], pbytes);
        const size_t next = round_up(cursor + pbytes, kAlign);
        std::memset((unsigned char*)image + cursor + pbytes, 0, next - cursor - pbytes);
        cursor = next;
    }
    put<uint64_t>(image, 24, word_sum(image, payload_begin(n_mats, k), need));
    return BD_OK;
}

bd_status bd_delta_image_check(const void* image, size_t bytes, int32_t verify_checksum, int32_t* n_mats, int32_t* k) {
    int32_t nm = 0, planes = 0;
    const bd_status st = parse(image, bytes, &nm, &planes);
    if (st != BD_OK) return st;
    if (verify_checksum && word_sum(image, payload_begin(nm, planes), bytes) != get<uint64_t>(image, 24)) return BD_ERR_FORMAT;
    if (n_mats) *n_mats = nm;
    if (k) *k = planes;
    return BD_OK;
}

bd_status bd_delta_image_entry(const void* image, size_t bytes, int32_t m, int64_t* out, int64_t* in,
                               size_t* packed_offset, size_t* alpha_offset) {
    int32_t nm = 0, planes = 0;
    const bd_status st = parse(image, bytes, &nm, &planes);
    if (st != BD_OK) return st;
    if (m < 0 || m >= nm) return BD_ERR_SHAPE;
    const Entry e = get<Entry>(image, kHeaderBytes + (size_t)m * kEntryBytes);
    if (out) *out = e.out;
    if (in) *in = e.in;
    if (packed_offset) *packed_offset = (size_t)e.packed_offset;
    if (alpha_offset) *alpha_offset = (size_t)e.alpha_offset;
    return BD_OK;
}

bd_status bd_delta_file_write(const char* path, const void* image, size_t bytes) {
    if (!path || !image) return BD_ERR_NULL;
    int32_t nm = 0, planes = 0;
    const bd_status st = parse(image, bytes, &nm, &planes);
    if (st != BD_OK) return st;
    std::FILE* f = std::fopen(path, "wb");
    if (!f) return BD_ERR_IO;
    const size_t n = std::fwrite(image, 1, bytes, f);
    const int rc = std::fclose(f);
    return (n == bytes && rc == 0) ? BD_OK : BD_ERR_IO;
}

bd_status bd_delta_file_bytes(const char* path, size_t* bytes) {
    if (!path || !bytes) return BD_ERR_NULL;
    std::FILE* f = std::fopen(path, "rb");
    if (!f) return BD_ERR_IO;
    unsigned char head[kHeaderBytes];
    const size_t n = std::fread(head, 1, kHeaderBytes, f);
    std::fclose(f);
    if (n != kHeaderBytes || std::memcmp(head, kMagic, 8) != 0) return BD_ERR_FORMAT;
    *bytes = (size_t)get<uint64_t>(head, 16);
    return BD_OK;
}

bd_status bd_delta_file_read(const char* path, void* image, size_t bytes) {
    if (!path || !image) return BD_ERR_NULL;
    std::FILE* f = std::fopen(path, "rb");
    if (!f) return BD_ERR_IO;
    const size_t n = std::fread(image, 1, bytes, f);
    const bool more = std::fgetc(f) != EOF;   // the file must end where the image does
    std::fclose(f);
    if (n != bytes || more) return BD_ERR_FORMAT;
    int32_t nm = 0, planes = 0;
    return parse(image, bytes, &nm, &planes);
}

bd_status bd_delta_upload(const void* image, size_t bytes, void* arena, void* stream) {
    if (!image || !arena) return BD_ERR_NULL;
    if (((uintptr_t)arena & (kAlign - 1)) != 0) return BD_ERR_ALIGN;
    int32_t nm = 0, planes = 0;
    const bd_status st = parse(image, bytes, &nm, &planes);
    if (st != BD_OK) return st;
    return hipMemcpyAsync(arena, image, bytes, hipMemcpyHostToDevice, (hipStream_t)stream) == hipSuccess ? BD_OK
                                                                                                         : BD_ERR_DEVICE;
}

bd_status bd_delta_install(const void* image, size_t bytes, const void* arena, int32_t tenant, int32_t n_tenants,
                           uint32_t* const* tiled_dst, float* const* alpha_by_tenant, void* stream) {
    if (!image || !arena || !tiled_dst || !alpha_by_tenant) return BD_ERR_NULL;
    if (((uintptr_t)arena & (kAlign - 1)) != 0) return BD_ERR_ALIGN;
    if (tenant < 0 || tenant >= n_tenants) return BD_ERR_TENANT;
    int32_t nm = 0, planes = 0;
    bd_status st = parse(image, bytes, &nm, &planes);
    if (st != BD_OK) return st;
    for (int32_t m = 0; m < nm; ++m) {   // every argument is checked before anything is enqueued
        const Entry e = get<Entry>(image, kHeaderBytes + (size_t)m * kEntryBytes);
        if (!alpha_by_tenant[m]) return BD_ERR_NULL;
        if (e.out > 0 && e.in > 0) {
            if (bd_tiled_signs_bytes(e.out, e.in) == 0) return BD_ERR_SHAPE;
            if ((e.packed_bytes / planes) % 16 != 0) return BD_ERR_ALIGN;   // every plane starts 16-byte aligned
            for (int32_t j = 0; j < planes; ++j) {
                const uint32_t* d = tiled_dst[(size_t)m * planes + j];
                if (!d) return BD_ERR_NULL;
                if (((uintptr_t)d & 15) != 0) return BD_ERR_ALIGN;
            }
        }
    }
    for (int32_t m = 0; m < nm; ++m) {
        const Entry e = get<Entry>(image, kHeaderBytes + (size_t)m * kEntryBytes);
        // the scales come from the host copy of the image, the planes from the copy in the arena
        if (hipMemcpyAsync(alpha_by_tenant[m] + (size_t)tenant * planes, (const unsigned char*)image + e.alpha_offset,
                           (size_t)planes * sizeof(float), hipMemcpyHostToDevice, (hipStream_t)stream) != hipSuccess)
            return BD_ERR_DEVICE;
        if (e.out == 0 || e.in == 0) continue;
        const size_t plane_bytes = (size_t)(e.packed_bytes / planes);
        for (int32_t j = 0; j < planes; ++j) {
            const uint32_t* src = (const uint32_t*)((const unsigned char*)arena + e.packed_offset + (size_t)j * plane_bytes);
            st = bd_tile_signs(src, e.out, e.in, tiled_dst[(size_t)m * planes + j], stream);
            if (st != BD_OK) return st;
        }
    }
    return BD_OK;
}

}  // extern "C"
