// Host side of the packed format: size computation, bit slicing, its inverse.  No HIP calls.
// (Any-Precision LLM, Section 5.1: weights decomposed into bit-vectors, one per bit position;
// Section 5.3: the permutation inside the bitplanes is done once, as pre-processing.)
#include "pack.h"

#include <algorithm>
#include <cstring>
#include <thread>
#include <vector>

namespace apgemv {

static inline uint32_t rotl32(uint32_t v, int r) { r &= 31; return r ? (v << r) | (v >> (32 - r)) : v; }
static inline uint32_t rotr32(uint32_t v, int r) { r &= 31; return r ? (v >> r) | (v << (32 - r)) : v; }

ap_status check_shape(int M, int K, int n)
{
    if (n < AP_MIN_BITS || n > AP_MAX_BITS) return AP_ERR_BITS;
    if (M < 1 || K < kChunkSlots || K % kChunkSlots != 0) return AP_ERR_SHAPE;
    if (M > (1 << 24) || K > (1 << 24)) return AP_ERR_SHAPE;
    // the kernels address the slices of a row group with 32-bit offsets: 7 * slice_bytes < 4 GiB
    if ((unsigned long long)padded_rows(M) * (unsigned long long)K > (1ull << 32)) return AP_ERR_SHAPE;
    return AP_OK;
}

ap_status check_mask(int n, unsigned lut_mask)
{
    unsigned allowed = 0;
    for (int b = AP_MIN_BITS; b <= n; ++b) allowed |= 1u << b;
    if (lut_mask == 0 || (lut_mask & ~allowed)) return AP_ERR_BITS;
    return AP_OK;
}

ap_status check_index_range(const uint8_t *idx, int M, int K, int n)
{
    if (n >= 8) return AP_OK;
    const size_t total = (size_t)M * K;
    const unsigned limit = 1u << n;
    for (size_t i = 0; i < total; ++i)
        if (idx[i] >= limit) return AP_ERR_INDEX_RANGE;
    return AP_OK;
}

ap_status make_header(int M, int K, int n, unsigned lut_mask, BlobHeader *h)
{
    ap_status s = check_shape(M, K, n);
    if (s != AP_OK) return s;
    s = check_mask(n, lut_mask);
    if (s != AP_OK) return s;
    std::memset(h, 0, sizeof(*h));
    h->magic = kMagic;
    h->version = kLayoutVersion;
    h->M = M;
    h->K = K;
    h->n = n;
    h->lut_mask = lut_mask;
    h->slice_bytes = slice_bytes(M, K);
    size_t off = sizeof(BlobHeader);
    h->slice_off = off;
    off = align_up(off + (size_t)n * h->slice_bytes, kAlign);
    for (int b = AP_MIN_BITS; b <= n; ++b) {
        if (!(lut_mask & (1u << b))) continue;
        h->lut_off[b] = off;
        off = align_up(off + (size_t)M * ((size_t)2 << b), kAlign);
    }
    h->total_bytes = off;
    return AP_OK;
}

ap_status validate_header(const BlobHeader *h, size_t blob_bytes)
{
    if (h->magic != kMagic || h->version != kLayoutVersion) return AP_ERR_INVALID_ARG;
    BlobHeader ref;
    if (make_header(h->M, h->K, h->n, h->lut_mask, &ref) != AP_OK) return AP_ERR_INVALID_ARG;
    if (std::memcmp(&ref, h, sizeof(ref)) != 0) return AP_ERR_INVALID_ARG;
    if (blob_bytes < ref.total_bytes) return AP_ERR_BUFFER_TOO_SMALL;
    return AP_OK;
}

template <class F> static void parallel_groups(int groups, F &&fn)
{
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<unsigned>(hw ? hw : 1, 16);
    nt = std::max(1, std::min(nt, groups / 64));
    if (nt == 1) {
        fn(0, groups);
        return;
    }
    std::vector<std::thread> th;
    int per = (groups + nt - 1) / nt;
    for (int t = 0; t < nt; ++t) {
        int lo = t * per, hi = std::min(groups, lo + per);
        if (lo < hi) th.emplace_back([=, &fn] { fn(lo, hi); });
    }
    for (auto &t : th) t.join();
}

// spread[v]: bit i of v (column offset i = 2j + parity inside a run of 8 columns) moved to bit
// 8j + parity, the position of slot 8j + 2t + parity before the shift by 2t.
static const uint32_t *spread_table()
{
    static uint32_t table[256];
    static bool ready = [] {
        for (int v = 0; v < 256; ++v) {
            uint32_t w = 0;
            for (int i = 0; i < 8; ++i)
                if (v & (1 << i)) w |= 1u << (8 * (i >> 1) + (i & 1));
            table[v] = w;
        }
        return true;
    }();
    (void)ready;
    return table;
}

void pack_slices(const uint8_t *idx, const BlobHeader &h, uint8_t *blob)
{
    const int M = h.M, K = h.K, n = h.n;
    const int chunks = K / kChunkSlots;
    const int groups = padded_rows(M) / kRowsPerGroup;
    const uint32_t *spread = spread_table();
    parallel_groups(groups, [&](int g0, int g1) {
        for (int g = g0; g < g1; ++g) {
            for (int q = 0; q < chunks; ++q) {
                const int span = q / kSpanLanes, lane = q % kSpanLanes;
                const int nl = span_lanes(K, span);
                for (int r = 0; r < kRowsPerGroup; ++r) {
                    const int row = g * kRowsPerGroup + r;
                    uint32_t plain[8] = {0, 0, 0, 0, 0, 0, 0, 0}; // plain[s]: bit of slot q at bit q
                    if (row < M) {
                        const uint8_t *src = idx + (size_t)row * K;
                        // a lane's slots are four runs of 8 consecutive columns (slot_column): take a
                        // run as one 64-bit word, gather bit p of its 8 bytes into a byte with a
                        // multiply, and spread that byte to the run's slot positions
                        for (int t = 0; t < 4; ++t) {
                            uint64_t x;
                            std::memcpy(&x, src + slot_column(span, nl, lane, 2 * t), 8);
                            for (int s = 0; s < n; ++s) {
                                const int p = n - 1 - s;
                                const uint64_t bits = (x >> p) & 0x0101010101010101ull;
                                const uint32_t v = (uint32_t)((bits * 0x0102040810204080ull) >> 56);
                                plain[s] |= spread[v] << (2 * t);
                            }
                        }
                    }
                    for (int s = 0; s < n; ++s) {
                        uint32_t w = rotl32(plain[s], slice_rot(s));
                        size_t off = h.slice_off + (size_t)s * h.slice_bytes +
                                     ((size_t)g * chunks + q) * 16 + (size_t)r * 4;
                        std::memcpy(blob + off, &w, 4);
                    }
                }
            }
        }
    });
}

void unpack_slices(const uint8_t *blob, const BlobHeader &h, uint8_t *idx)
{
    const int M = h.M, K = h.K, n = h.n;
    const int chunks = K / kChunkSlots;
    const int groups = padded_rows(M) / kRowsPerGroup;
    parallel_groups(groups, [&](int g0, int g1) {
        for (int g = g0; g < g1; ++g) {
            for (int q = 0; q < chunks; ++q) {
                const int span = q / kSpanLanes, lane = q % kSpanLanes;
                const int nl = span_lanes(K, span);
                for (int r = 0; r < kRowsPerGroup; ++r) {
                    const int row = g * kRowsPerGroup + r;
                    if (row >= M) continue;
                    uint32_t plain[8];
                    for (int s = 0; s < n; ++s) {
                        uint32_t w;
                        size_t off = h.slice_off + (size_t)s * h.slice_bytes +
                                     ((size_t)g * chunks + q) * 16 + (size_t)r * 4;
                        std::memcpy(&w, blob + off, 4);
                        plain[s] = rotr32(w, slice_rot(s));
                    }
                    uint8_t *dst = idx + (size_t)row * K;
                    for (int slot = 0; slot < kChunkSlots; ++slot) {
                        unsigned v = 0;
                        for (int s = 0; s < n; ++s) v |= ((plain[s] >> slot) & 1u) << (n - 1 - s);
                        dst[slot_column(span, nl, lane, slot)] = (uint8_t)v;
                    }
                }
            }
        }
    });
}

} // namespace apgemv

using namespace apgemv;

extern "C" ap_status ap_packed_size(int M, int K, int n, unsigned lut_mask, size_t *bytes)
{
    if (!bytes) return AP_ERR_INVALID_ARG;
    BlobHeader h;
    ap_status s = make_header(M, K, n, lut_mask, &h);
    if (s != AP_OK) return s;
    *bytes = h.total_bytes;
    return AP_OK;
}

extern "C" ap_status ap_pack_host(const uint8_t *idx, int M, int K, int n,
                                  const uint16_t *const luts[9], void *blob, size_t blob_bytes)
{
    if (!idx || !luts || !blob) return AP_ERR_INVALID_ARG;
    ap_status s = check_shape(M, K, n);
    if (s != AP_OK) return s;
    unsigned mask = 0;
    for (int b = AP_MIN_BITS; b <= n; ++b)
        if (luts[b]) mask |= 1u << b;
    BlobHeader h;
    s = make_header(M, K, n, mask, &h);
    if (s != AP_OK) return s;
    if (blob_bytes < h.total_bytes) return AP_ERR_BUFFER_TOO_SMALL;
    s = check_index_range(idx, M, K, n);
    if (s != AP_OK) return s;
    uint8_t *out = static_cast<uint8_t *>(blob);
    std::memset(out, 0, h.total_bytes);
    std::memcpy(out, &h, sizeof(h));
    pack_slices(idx, h, out);
    for (int b = AP_MIN_BITS; b <= n; ++b) {
        if (!luts[b]) continue;
        const int E = 1 << b;
        std::vector<int> pos(E);
        for (int e = 0; e < E; ++e) pos[e] = lut_stored_pos(b, e);
        uint16_t *dst = reinterpret_cast<uint16_t *>(out + h.lut_off[b]);
        for (int i = 0; i < M; ++i)
            for (int e = 0; e < E; ++e) dst[(size_t)i * E + pos[e]] = luts[b][(size_t)i * E + e];
    }
    return AP_OK;
}

extern "C" ap_status ap_unpack_host(const void *blob, size_t blob_bytes, uint8_t *idx_out)
{
    if (!blob || !idx_out || blob_bytes < sizeof(BlobHeader)) return AP_ERR_INVALID_ARG;
    BlobHeader h;
    std::memcpy(&h, blob, sizeof(h));
    ap_status s = validate_header(&h, blob_bytes);
    if (s != AP_OK) return s;
    unpack_slices(static_cast<const uint8_t *>(blob), h, idx_out);
    return AP_OK;
}

extern "C" ap_status ap_blob_lut_entry(const void *blob, size_t blob_bytes, int b, int row,
                                       int entry, uint16_t *out)
{
    if (!blob || !out || blob_bytes < sizeof(BlobHeader)) return AP_ERR_INVALID_ARG;
    BlobHeader h;
    std::memcpy(&h, blob, sizeof(h));
    ap_status s = validate_header(&h, blob_bytes);
    if (s != AP_OK) return s;
    if (b < AP_MIN_BITS || b > h.n || !(h.lut_mask & (1u << b))) return AP_ERR_BITS;
    if (row < 0 || row >= h.M || entry < 0 || entry >= (1 << b)) return AP_ERR_INVALID_ARG;
    std::memcpy(out, static_cast<const uint8_t *>(blob) + h.lut_off[b] +
                         ((size_t)row << (b + 1)) + (size_t)lut_stored_pos(b, entry) * 2, 2);
    return AP_OK;
}

extern "C" ap_status ap_read_extent(int M, int K, int n, unsigned lut_mask, int b,
                                    size_t *slices_begin, size_t *slices_end, size_t *lut_begin,
                                    size_t *lut_end)
{
    BlobHeader h;
    ap_status s = make_header(M, K, n, lut_mask, &h);
    if (s != AP_OK) return s;
    if (b < AP_MIN_BITS || b > n || !(lut_mask & (1u << b))) return AP_ERR_BITS;
    if (slices_begin) *slices_begin = h.slice_off;
    if (slices_end) *slices_end = h.slice_off + (size_t)b * h.slice_bytes;
    if (lut_begin) *lut_begin = h.lut_off[b];
    if (lut_end) *lut_end = h.lut_off[b] + (size_t)M * ((size_t)2 << b);
    return AP_OK;
}

extern "C" const char *ap_strerror(ap_status s)
{
    switch (s) {
    case AP_OK: return "ok";
    case AP_ERR_INVALID_ARG: return "invalid argument";
    case AP_ERR_SHAPE: return "unsupported shape (need M >= 1, K a multiple of 32, M and K at most 2^24, at most 2^32 weights)";
    case AP_ERR_BITS: return "bit-width not supported for this matrix";
    case AP_ERR_INDEX_RANGE: return "index value does not fit the parent bit-width";
    case AP_ERR_BUFFER_TOO_SMALL: return "buffer smaller than ap_packed_size";
    case AP_ERR_BATCH: return "batch outside the supported range";
    case AP_ERR_HIP: return "HIP runtime call or kernel launch failed";
    case AP_ERR_NO_MEMORY: return "host memory could not be allocated";
    }
    return "unknown status";
}
