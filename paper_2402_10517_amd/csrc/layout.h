// Device layout of a packed any-precision matrix (shared by the host packer and the kernels).
//
// The paper stores n plain bitplanes and permutes bytes inside them so that a warp's activation
// loads coalesce (Section 5.1; Section 5.3 "Weight Bitplane Layout Optimization").  This layout
// keeps the property that matters - slice s holds index bit (n-1-s) of every weight, so a b-bit
// call reads the first b slices and nothing else - and changes everything inside a slice for
// 64-wide wavefronts and for a merge that needs no shifts:
//
//  * Rows are grouped by 4.  One 16-byte unit of a slice holds one 32-bit word for each of the
//    4 rows of a group, for one chunk of 32 weights ("slots") per row; a lane loads it with one
//    dwordx4 and reuses its 32 activations for 4 rows.
//  * A wave covers a span of 64 chunks (2048 columns) per step; the last span of a row may have
//    fewer lanes (K/32 mod 64).  Inside a span with nl lanes, lane l owns four runs of 8
//    consecutive columns, run t starting at span*2048 + t*8*nl + l*8, so each of its four 16-byte
//    activation loads is contiguous across the wave.
//  * Slot s = 8*j + u (u = s & 7, j = s >> 3) of a chunk is column offset 2*j + (u & 1) of run
//    t = u >> 1: slots u even / u+1 are adjacent columns, which lets two weights share one packed
//    binary16 activation pair.
//  * In slice s the bit of slot q sits at bit position (q + slice_rot(s)) mod 32 of the word.  With
//    these rotations, the word for the four slots {8j+u, j=0..3} of one row is obtained by
//    bit-selects with constant masks (no shifts) followed by one rotate right by u: byte j then
//    holds slice s of slot 8j+u at bit slice_rot(s).  Because the rotations 0..7 are all distinct,
//    the selects of the eight words can share a tree over the rotation value (pairs, quads, all).  Because slice_rot(0..2) are even (6,4,2) and slot
//    8j+u+1 sits one position higher, the same select for u even yields, at byte bits 2..7, the
//    six bits of the slot pair (u, u+1): the 3-bit path uses them as one index into a table of
//    centroid pairs (Section 5.3 "Merging Table Lookups", generalised to a 64-entry pair table
//    whose index bits are interleaved).
#ifndef APGEMV_LAYOUT_H
#define APGEMV_LAYOUT_H

#include <stddef.h>
#include <stdint.h>

namespace apgemv {

constexpr int kRowsPerGroup = 4;
constexpr int kChunkSlots = 32;
constexpr int kSpanLanes = 64;
constexpr int kSpanCols = kSpanLanes * kChunkSlots; // 2048
constexpr uint32_t kMagic = 0x31475041u;            // "APG1"
constexpr uint32_t kLayoutVersion = 2;
constexpr size_t kAlign = 256;

// Rotation of slice s (s = 0 is the most significant index bit).  For a b-bit call the used
// positions are slice_rot(0..b-1); for b = 4,5,6 they fall on LDS address bits 2..6 (plus bit 1),
// which spreads a row's table over distinct banks.
#if defined(__HIPCC__)
#define APGEMV_HD __host__ __device__
#else
#define APGEMV_HD
#endif
APGEMV_HD constexpr int slice_rot(int s)
{
    constexpr int rot[8] = {6, 4, 2, 3, 5, 1, 7, 0};
    return rot[s];
}

// Centroid tables are stored per row in the order of the kernel's LDS addressing, so staging is a
// plain copy.  For bit-widths that look up one weight at a time (b >= 4) the table address of an
// index is built from the index bits sitting at byte positions slice_rot(0..b-1); sorting those
// positions ascending and numbering them 0..b-1 gives the stored position of an entry:
// stored position = sum over slices s < b of (index bit of slice s) << rank_b(slice_rot(s)).
// b = 3 (pair lookups) keeps the natural order.  Natural entry e has the bit of slice s at
// bit (b-1-s).
APGEMV_HD constexpr int lut_stored_pos(int b, int e)
{
    if (b <= 3) return e;
    int pos = 0;
    for (int s = 0; s < b; ++s) {
        int rank = 0;
        for (int s2 = 0; s2 < b; ++s2)
            if (slice_rot(s2) < slice_rot(s)) ++rank;
        pos |= ((e >> (b - 1 - s)) & 1) << rank;
    }
    return pos;
}

struct BlobHeader { // first 256 bytes of the blob, little endian
    uint32_t magic;
    uint32_t version;
    int32_t M, K, n;
    uint32_t lut_mask;
    uint64_t total_bytes;
    uint64_t slice_bytes;   // bytes of one slice
    uint64_t slice_off;     // offset of slice 0; slice s at slice_off + s*slice_bytes
    uint64_t lut_off[9];    // offset of the table of bit-width b (0 = absent)
    uint8_t pad[256 - 4 * 6 - 8 * 3 - 8 * 9];
};
static_assert(sizeof(BlobHeader) == 256, "header is 256 bytes");

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int padded_rows(int M) { return (M + kRowsPerGroup - 1) / kRowsPerGroup * kRowsPerGroup; }
inline size_t slice_bytes(int M, int K) { return (size_t)padded_rows(M) * (size_t)K / 8; }

// Lanes of span `span` of a row of K columns.
inline int span_lanes(int K, int span)
{
    int chunks = K / kChunkSlots - span * kSpanLanes;
    return chunks < kSpanLanes ? chunks : kSpanLanes;
}
// Column of slot `slot` of lane `lane` in span `span` with nl lanes.
inline int slot_column(int span, int nl, int lane, int slot)
{
    int u = slot & 7, j = slot >> 3, t = u >> 1;
    return span * kSpanCols + t * 8 * nl + lane * 8 + 2 * j + (u & 1);
}

} // namespace apgemv
#endif
