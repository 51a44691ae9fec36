// Device helpers shared by the any-precision kernels for gfx950 (CDNA4, wave64): bit-select and
// SDWA wrappers, the per-bit-width table geometry, table staging, index formation (the select tree),
// table lookups and the multiply-accumulate of one unit of 4 rows x 32 columns per lane.
#ifndef APGEMV_DEVICE_COMMON_H
#define APGEMV_DEVICE_COMMON_H

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "kernels.h"
#include "layout.h"

namespace apgemv {


typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t rotl_c(uint32_t v, int r)
{
    r &= 31;
    return r ? (v << r) | (v >> (32 - r)) : v;
}
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Buffer descriptors of raw (untyped, unstrided) device memory: word 3 = 32-bit data format, no swizzle;
// weight loads do not rely on the range check (num_records = 2^32 - 1, callers clamp their own
// offsets); the tile kernel's activation loads do (a lane offset >= num_records reads zeros).
constexpr uint32_t kBufferRsrcWord3 = 0x00020000u;
constexpr int kBufferNonTemporal = 2; // cache-policy bits of a buffer load: streaming data, read once

// d = (m & a) | (~m & b) with a constant mask: one v_bfi_b32 (the mask sits in an SGPR)
__device__ __forceinline__ uint32_t bitsel(uint32_t m, uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(d) : "s"(m), "v"(a), "v"(b));
    return d;
}
// (byte J of v) & mask, and (byte J of v) << n with n in a register: one SDWA instruction each.  They turn a byte of a
// merged index word into an LDS address.
template <int J> __device__ __forceinline__ uint32_t byte_and(uint32_t v, uint32_t mask)
{
    uint32_t d;
    if constexpr (J == 0)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0 src1_sel:DWORD" : "=v"(d) : "v"(v), "s"(mask));
    else if constexpr (J == 1)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD" : "=v"(d) : "v"(v), "s"(mask));
    else if constexpr (J == 2)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2 src1_sel:DWORD" : "=v"(d) : "v"(v), "s"(mask));
    else
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3 src1_sel:DWORD" : "=v"(d) : "v"(v), "s"(mask));
    return d;
}
template <int J> __device__ __forceinline__ uint32_t byte_shl1(uint32_t v, uint32_t one)
{
    uint32_t d;
    if constexpr (J == 0)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(d) : "v"(one), "v"(v));
    else if constexpr (J == 1)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(d) : "v"(one), "v"(v));
    else if constexpr (J == 2)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(d) : "v"(one), "v"(v));
    else
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(d) : "v"(one), "v"(v));
    return d;
}
template <int B, int J> __device__ __forceinline__ uint32_t byte_to_addr(uint32_t v, uint32_t mask, uint32_t one)
{
    if constexpr (B == 8) return byte_shl1<J>(v, one);
    else return byte_and<J>(v, mask);
}

__device__ __forceinline__ uint32_t rotr_v(uint32_t v, int r)
{
    return (r & 31) ? __builtin_amdgcn_alignbit(v, v, r & 31) : v;
}

template <int B> struct Table {
    static constexpr bool kPair = (B == 3);
    // bytes of one row's table in LDS
    static constexpr int kRowBytes = B == 3 ? 256 : B <= 6 ? 128 : B == 7 ? 256 : 512;
    // Single-lookup modes: the LDS byte address of an index is the merged byte masked to the
    // positions slice_rot(0..B-1); B = 8 uses all eight byte bits and shifts left by one instead.
    __device__ static constexpr uint32_t addr_mask()
    {
        uint32_t m = 0;
        for (int s = 0; s < B; ++s) m |= 1u << slice_rot(s);
        return m;
    }
    // LDS byte address of the entry stored at position c of a row (lut_stored_pos order).
    __device__ static constexpr uint32_t stored_addr(uint32_t c)
    {
        return B == 4 ? (((c & 8u) << 3) | ((c & 7u) << 2)) : B == 5 ? (c << 2) : (c << 1);
    }
};

// The 64-entry table of centroid pairs of the 3-bit path (Section 5.3 "Merging Table Lookups"): pair
// index bit 2k is code bit k of the even slot, bit 2k+1 is code bit k of the odd slot.  Entry i6 of a
// row = (centroid of the even slot's code, centroid of the odd slot's code), from the natural row.
__device__ __forceinline__ constexpr int pair3_even(int i6) { return (i6 & 1) | ((i6 >> 1) & 2) | ((i6 >> 2) & 4); }
__device__ __forceinline__ constexpr int pair3_odd(int i6) { return ((i6 >> 1) & 1) | ((i6 >> 2) & 2) | ((i6 >> 3) & 4); }
__device__ __forceinline__ uint32_t pair_entry(const uint16_t *nat_row, int i6)
{
    return (uint32_t)nat_row[pair3_even(i6)] | ((uint32_t)nat_row[pair3_odd(i6)] << 16);
}

template <int ctrl> __device__ __forceinline__ float dpp_get(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xf, 0xf, true));
}
// Reduce the four per-row accumulators of a lane over each DPP row of 16 lanes at once.  Two
// exchange steps leave one accumulator per lane (lane bits 0,1 select which: 0 -> row 0,
// 1 -> row 2, 2 -> row 1, 3 -> row 3), two row shifts add the four quads.  On return lanes 12..15
// of every DPP row hold that row's partial sums; 11 operations instead of 4 full reductions.
__device__ __forceinline__ float reduce4_in_dpp_rows(const float (&a)[kRowsPerGroup], int lane)
{
    const bool odd = lane & 1, hi = lane & 2;
    const float keep0 = odd ? a[2] : a[0], send0 = odd ? a[0] : a[2];
    const float keep1 = odd ? a[3] : a[1], send1 = odd ? a[1] : a[3];
    const float b0 = keep0 + dpp_get<0xB1>(send0); // quad_perm [1,0,3,2]
    const float b1 = keep1 + dpp_get<0xB1>(send1);
    const float keep = hi ? b1 : b0, send = hi ? b0 : b1;
    float c = keep + dpp_get<0x4E>(send);          // quad_perm [2,3,0,1]
    c += dpp_get<0x114>(c);                        // row_shr:4 (0 shifted in)
    c += dpp_get<0x118>(c);                        // row_shr:8
    return c;
}

// Staging of the 4 rows' tables of a group, split in two so that the global loads can be issued
// before the (much larger) slice loads and the LDS writes after them: vector-memory loads return
// in order, so a table load issued last would only be usable once every slice load had landed.
template <int B> struct StagedTable {
    u32x4 v[2]; // B >= 6: up to two 16-byte pieces per thread; B <= 5: one dword in v[0].x
};

// All loads here are unconditional (indices clamped, unused results dropped or zeroed afterwards):
// with no branch between them and the slice loads the compiler can count outstanding loads
// exactly and waits for the table loads only.
// `nth` = threads that take part (thread ids 0..nth-1; a multiple of 64, at least 64).
template <int B>
__device__ __forceinline__ void stage_tables_load(StagedTable<B> &st, const uint16_t *__restrict__ lut, int row0, int M,
                                                  int nth)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    const int tid = threadIdx.x;
    const int last_row = M - 1 - row0; // >= 0
    if constexpr (B == 3) {
        // natural 8-entry rows: 4 rows x 4 dwords
        static_assert(kRowsPerGroup * 4 <= 64, "one dword per thread of the first wave");
        const int i = tid < kRowsPerGroup * 4 ? tid : kRowsPerGroup * 4 - 1;
        const int r = i >> 2;
        const int rc = r < last_row ? r : last_row;
        const uint32_t v = reinterpret_cast<const uint32_t *>(lut + (size_t)row0 * 8)[rc * 4 + (i & 3)];
        st.v[0].x = r <= last_row ? v : 0u;
    } else if constexpr (B >= 6) {
        // stored order = LDS order, rows contiguous: 16-byte pieces
        constexpr int kPerRow = TB / 16;
        constexpr int kChunks = kRowsPerGroup * kPerRow;
        static_assert(kChunks <= 2 * 64, "two rounds of at least 64 threads cover the tables");
        const u32x4 *src = reinterpret_cast<const u32x4 *>(lut + ((size_t)row0 << B));
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            int i = tid + it * nth;
            i = i < kChunks ? i : kChunks - 1;
            const int r = i / kPerRow;
            const int rc = r < last_row ? r : last_row;
            const u32x4 v = src[rc * kPerRow + i % kPerRow];
            st.v[it] = r <= last_row ? v : u32x4{0, 0, 0, 0};
        }
    } else {
        // B = 4, 5: two stored entries per dword
        constexpr int kDwordsPerRow = (1 << B) / 2;
        constexpr int kDwords = kRowsPerGroup * kDwordsPerRow;
        static_assert(kDwords <= 64, "one dword per thread of the first wave");
        const uint32_t *src = reinterpret_cast<const uint32_t *>(lut + ((size_t)row0 << B));
        const int i = tid < kDwords ? tid : kDwords - 1;
        const int r = i / kDwordsPerRow;
        const int rc = r < last_row ? r : last_row;
        const uint32_t v = src[rc * kDwordsPerRow + i % kDwordsPerRow];
        st.v[0].x = r <= last_row ? v : 0u;
    }
}

// The LDS writes are unconditional as well (threads without a piece write a 16-byte dummy area
// behind the tables): a conditional store would pull its load down into the branch, behind the
// slice loads.
template <int B, int STRIDE = Table<B>::kRowBytes>
__device__ __forceinline__ void stage_tables_store(const StagedTable<B> &st, uint8_t *tab, uint16_t *nat, int nth)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    static_assert(STRIDE >= TB, "row stride in LDS");
    constexpr int kDummy = kRowsPerGroup * STRIDE; // byte offset of the dummy area inside tab
    const int tid = threadIdx.x;
    if constexpr (B == 3) {
        // the 64-entry table of centroid pairs: pair index bit 2k is code bit k of the even slot,
        // bit 2k+1 is code bit k of the odd slot.
        uint32_t *dst = tid < kRowsPerGroup * 4 ? reinterpret_cast<uint32_t *>(nat) + tid
                                                : reinterpret_cast<uint32_t *>(tab + kDummy);
        *dst = st.v[0].x;
        __syncthreads();
        // a thread's pair index is its lane (nth is a multiple of 64); the loop only walks the rows
        const int i6 = tid & 63;
        for (int r = tid >> 6; r < kRowsPerGroup; r += nth >> 6)
            *reinterpret_cast<uint32_t *>(tab + r * STRIDE + i6 * 4) = pair_entry(nat + r * 8, i6);
    } else if constexpr (B >= 6) {
        constexpr int kPerRow = TB / 16;
        constexpr int kChunks = kRowsPerGroup * kPerRow;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int i = tid + it * nth;
            const int off = i < kChunks ? (i / kPerRow) * STRIDE + (i % kPerRow) * 16 : kDummy;
            *reinterpret_cast<u32x4 *>(tab + off) = st.v[it];
        }
    } else {
        // spread the two entries of a dword to their dword-strided LDS addresses
        constexpr int kDwordsPerRow = (1 << B) / 2;
        const int r = tid / kDwordsPerRow, k = tid % kDwordsPerRow;
        uint8_t *dst = tid < kRowsPerGroup * kDwordsPerRow ? tab + r * STRIDE + T::stored_addr(2 * k) : tab + kDummy;
        *reinterpret_cast<uint16_t *>(dst) = (uint16_t)st.v[0].x;
        *reinterpret_cast<uint16_t *>(dst + 4) = (uint16_t)(st.v[0].x >> 16);
    }
}

// Slice (0 = most significant) whose bits sit at rotation p among the first B slices, or -1.
__device__ constexpr int slice_with_rot(int B, int p)
{
    for (int s = 0; s < B; ++s)
        if (slice_rot(s) == p) return s;
    return -1;
}

// Index formation for one row (Section 5.2 step 2; Section 5.3 "Efficient Bit-transpose"): turns the
// row's B slice words into eight words W[u], u = 0..7, whose byte j holds the index of slot 8j + u
// with the bit of slice s at byte bit slice_rot(s) (other byte bits are unspecified).  In pair mode
// (B = 3) only even u are formed and byte bits 2..7 hold the interleaved indices of slots u, u + 1.
//
// Bits never move until the final rotate: slice s stores slot q at word bit q + slice_rot(s), so the
// bits wanted for class u sit at word bits 8j + u + slice_rot(s).  The selects are shared between
// classes as a three-level tree over the rotation value: level 1 joins rotations {2a, 2a+1} for the
// classes u mod 2 (the two sources occupy alternating bits), level 2 joins {4c..4c+3} for u mod 4,
// level 3 joins all eight for each u.  8 slices cost 8 + 8 + 8 selects and 7 rotates per 32 weights
// instead of 8 x 7 selects; absent rotations (B < 8) drop their selects.
// EXTRA more bits of right rotation: byte j of W[u] is then the index byte shifted right by EXTRA, with the
// low bits of byte j + 1 above it (for callers that mask the bytes afterwards).
template <int B, int EXTRA = 0>
__device__ __forceinline__ void merge_words(const uint32_t (&q)[B], uint32_t (&W)[8])
{
    constexpr bool kPair = Table<B>::kPair;
    constexpr int kStep = kPair ? 2 : 1;
    uint32_t L1[4][2];
    bool has1[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int lo = slice_with_rot(B, 2 * a), hi = slice_with_rot(B, 2 * a + 1);
        has1[a] = lo >= 0 || hi >= 0;
#pragma unroll
        for (int c = 0; c < 2; c += kStep) {
            if (lo >= 0 && hi >= 0) L1[a][c] = bitsel(rotl_c(0x55555555u, c), q[lo < 0 ? 0 : lo], q[hi < 0 ? 0 : hi]);
            else if (lo >= 0) L1[a][c] = q[lo < 0 ? 0 : lo];
            else if (hi >= 0) L1[a][c] = q[hi < 0 ? 0 : hi];
            else L1[a][c] = 0;
        }
    }
    uint32_t L2[2][4];
    bool has2[2];
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2) {
        has2[c2] = has1[2 * c2] || has1[2 * c2 + 1];
#pragma unroll
        for (int cls = 0; cls < 4; cls += kStep) {
            const uint32_t lo = L1[2 * c2][cls & 1], hi = L1[2 * c2 + 1][cls & 1];
            if (has1[2 * c2] && has1[2 * c2 + 1]) L2[c2][cls] = bitsel(rotl_c(0x33333333u, cls), lo, hi);
            else L2[c2][cls] = has1[2 * c2] ? lo : hi;
        }
    }
#pragma unroll
    for (int u = 0; u < 8; u += kStep) {
        const uint32_t lo = L2[0][u & 3], hi = L2[1][u & 3];
        uint32_t v;
        if (has2[0] && has2[1]) v = bitsel(rotl_c(0x0F0F0F0Fu, u), lo, hi);
        else v = has2[0] ? lo : hi;
        W[u] = rotr_v(v, u + EXTRA);
    }
}
template <int B>
__device__ __forceinline__ void merge_row(const u32x4 (&Q)[B], int r, uint32_t (&W)[8])
{
    uint32_t q[B];
#pragma unroll
    for (int s = 0; s < B; ++s) q[s] = Q[s][r];
    merge_words<B>(q, W);
}

// Index formation, table lookup and multiply-accumulate for the lane's 32 slots of 4 rows
// (Section 5.2 steps 2-5).
template <int B, int NB>
__device__ __forceinline__ void compute_unit(const u32x4 (&Q)[B], const u32x4 (&X)[NB][4],
                                             const uint8_t *tab, float (&acc)[NB][kRowsPerGroup])
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    uint32_t one = 1; // shift amount of the B = 8 address form, kept in a register
    asm("" : "+v"(one));
#pragma unroll
    for (int r = 0; r < kRowsPerGroup; ++r) {
        const uint8_t *trow = tab + r * TB;
        uint32_t W[8];
        merge_row<B>(Q, r, W);
        if constexpr (T::kPair) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t v = W[2 * t];
                const uint32_t a4[4] = {byte_and<0>(v, 0xFCu), byte_and<1>(v, 0xFCu), byte_and<2>(v, 0xFCu),
                                        byte_and<3>(v, 0xFCu)};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t w = *reinterpret_cast<const uint32_t *>(trow + a4[j]);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        // (copy the vector element first: a bit cast applied directly to a vector
                        // element reads element 0)
                        const uint32_t xw = X[nb][t][j];
                        acc[nb][r] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w),
                                                            __builtin_bit_cast(half2_t, xw), acc[nb][r], false);
                    }
                }
            }
        } else {
            // two merged words per activation run t: slots u = 2t (even columns) and 2t + 1 (odd)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint32_t a[2][4];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t v = W[2 * t + h];
                    a[h][0] = byte_to_addr<B, 0>(v, T::addr_mask(), one);
                    a[h][1] = byte_to_addr<B, 1>(v, T::addr_mask(), one);
                    a[h][2] = byte_to_addr<B, 2>(v, T::addr_mask(), one);
                    a[h][3] = byte_to_addr<B, 3>(v, T::addr_mask(), one);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint16_t w0 = *reinterpret_cast<const uint16_t *>(trow + a[0][j]);
                    const uint16_t w1 = *reinterpret_cast<const uint16_t *>(trow + a[1][j]);
                    if constexpr (NB == 1) {
                        const uint32_t xw = X[0][t][j];
                        const half2_t xp = __builtin_bit_cast(half2_t, xw);
                        acc[0][r] = __builtin_fmaf((float)__builtin_bit_cast(_Float16, w0), (float)xp.x, acc[0][r]);
                        acc[0][r] = __builtin_fmaf((float)__builtin_bit_cast(_Float16, w1), (float)xp.y, acc[0][r]);
                    } else {
                        // batch > 1: pack the two centroids once, one packed dot product per batch row
                        const uint32_t wp = (uint32_t)w0 | ((uint32_t)w1 << 16);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            const uint32_t xw = X[nb][t][j];
                            acc[nb][r] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, wp),
                                                                __builtin_bit_cast(half2_t, xw), acc[nb][r], false);
                        }
                    }
                }
            }
        }
    }
}

// ---- 4 bits, two weights per lookup (Section 5.3 "Merging Table Lookups", one bit-width further; used by the
// tile kernel, where a lane's row owns an LDS bank and the 256-entry table of a row gathers without the
// random bank conflicts it meets when all lanes of a wave read one row's table).  Slice 3 (rotation 3) is
// rotated to rotation 0 first, so that all four slices sit at even rotations {6, 4, 2, 0} and the bit of the
// odd slot of a pair, one position higher, never meets another slice: byte j of W[u] (u even) is the pair
// index of slots 8j + u and 8j + u + 1 with slice s of the even slot at bit 6 - 2s and of the odd slot at
// bit 7 - 2s.  Only levels 2 and 3 of the select tree are left (8 selects, 1 + 3 rotates per 32 weights).
__device__ __forceinline__ void merge_words_pair4(const uint32_t (&q)[4], uint32_t (&W)[8])
{
    const uint32_t q3 = rotr_v(q[3], 3);
    uint32_t L2[2][2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        L2[0][c] = bitsel(rotl_c(0x33333333u, 2 * c), q3, q[2]);
        L2[1][c] = bitsel(rotl_c(0x33333333u, 2 * c), q[1], q[0]);
    }
#pragma unroll
    for (int u = 0; u < 8; u += 2)
        W[u] = rotr_v(bitsel(rotl_c(0x0F0F0F0Fu, u), L2[0][(u >> 1) & 1], L2[1][(u >> 1) & 1]), u);
}
// Positions in the stored 4-bit table (slice 0, 1, 3, 2 at bits 3, 2, 1, 0) of the even and the odd slot of
// pair index p.
__device__ __forceinline__ constexpr int pair4_even(int p) { return ((p >> 3) & 8) | ((p >> 2) & 4) | ((p << 1) & 2) | ((p >> 2) & 1); }
__device__ __forceinline__ constexpr int pair4_odd(int p) { return ((p >> 4) & 8) | ((p >> 3) & 4) | (p & 2) | ((p >> 3) & 1); }

// A ragged last span of at most 32 chunks on all 64 lanes (b = 4, 5, 6): lane l works on chunk l % 32 and on
// two of its four rows, rows {0, 2} for l < 32 and {1, 3} for l >= 32, so the span costs half a wave-unit
// instead of a whole one with half of the lanes idle (rows of 5120 columns: 2.5 instead of 3 units, 11008
// columns: 5.4 instead of 6).  A row's table is 128 bytes at these bit-widths and bit 7 of an index byte is not
// an index bit: it takes the lane's half, which puts the odd rows' tables one row further without an operation
// per lookup (the even row 2 s is an immediate offset).  Per row, the products are added in the order of
// compute_unit, into the accumulator of the row this lane works on.
template <int B> constexpr bool half_unit_ok() { return B >= 4 && B <= 6; }
template <int B, int NB>
__device__ __forceinline__ void compute_unit_half(const u32x4 (&Q)[B], const u32x4 (&X)[NB][4], const uint8_t *tab,
                                                  float (&acc)[NB][kRowsPerGroup], bool upper)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    static_assert(TB == 128 && (T::addr_mask() & 0x80u) == 0, "bit 7 of an index byte is free and selects the next row");
    const uint32_t rowbit = upper ? 0x80808080u : 0u;
    uint32_t one = 1;
    asm("" : "+v"(one));
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint8_t *trow = tab + 2 * s * TB;
        uint32_t q[B];
#pragma unroll
        for (int sl = 0; sl < B; ++sl) q[sl] = upper ? Q[sl][2 * s + 1] : Q[sl][2 * s];
        uint32_t W[8];
        merge_words<B>(q, W);
#pragma unroll
        for (int u = 0; u < 8; ++u) W[u] = bitsel(0x80808080u, rowbit, W[u]);
        float a[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) a[nb] = upper ? acc[nb][2 * s + 1] : acc[nb][2 * s];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint32_t ad[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t v = W[2 * t + h];
                ad[h][0] = byte_and<0>(v, T::addr_mask() | 0x80u);
                ad[h][1] = byte_and<1>(v, T::addr_mask() | 0x80u);
                ad[h][2] = byte_and<2>(v, T::addr_mask() | 0x80u);
                ad[h][3] = byte_and<3>(v, T::addr_mask() | 0x80u);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint16_t w0 = *reinterpret_cast<const uint16_t *>(trow + ad[0][j]);
                const uint16_t w1 = *reinterpret_cast<const uint16_t *>(trow + ad[1][j]);
                if constexpr (NB == 1) {
                    const uint32_t xw = X[0][t][j];
                    const half2_t xp = __builtin_bit_cast(half2_t, xw);
                    a[0] = __builtin_fmaf((float)__builtin_bit_cast(_Float16, w0), (float)xp.x, a[0]);
                    a[0] = __builtin_fmaf((float)__builtin_bit_cast(_Float16, w1), (float)xp.y, a[0]);
                } else {
                    const uint32_t wp = (uint32_t)w0 | ((uint32_t)w1 << 16);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const uint32_t xw = X[nb][t][j];
                        a[nb] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, wp), __builtin_bit_cast(half2_t, xw), a[nb], false);
                    }
                }
            }
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            acc[nb][2 * s] = upper ? acc[nb][2 * s] : a[nb];
            acc[nb][2 * s + 1] = upper ? a[nb] : acc[nb][2 * s + 1];
        }
    }
}

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// byte J of v (already masked to table-address bits) with the lane's table row in address bits 8..9
template <int J> __device__ __forceinline__ uint32_t row_byte_addr(uint32_t v, uint32_t rowreg)
{
    return __builtin_amdgcn_perm(rowreg, v, 0x0c0c0400u | J);
}

// Tables of `ng` consecutive groups of 4 rows into LDS, row stride STRIDE (generic loop form).
template <int B, int STRIDE>
__device__ __forceinline__ void stage_tables_groups(uint8_t *tab, uint16_t *nat, const uint16_t *__restrict__ lut,
                                                    int row0, int nrows, int ng)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    const int tid = threadIdx.x, nth = blockDim.x;
    if constexpr (B == 3) {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(lut + (size_t)row0 * 8);
        for (int i = tid; i < ng * kRowsPerGroup * 4; i += nth)
            reinterpret_cast<uint32_t *>(nat)[i] = (i >> 2) < nrows ? src[i] : 0u;
        __syncthreads();
        for (int i = tid; i < ng * kRowsPerGroup * 64; i += nth) {
            const int r = i >> 6, i6 = i & 63;
            *reinterpret_cast<uint32_t *>(tab + r * STRIDE + i6 * 4) = pair_entry(nat + r * 8, i6);
        }
    } else if constexpr (B >= 6) {
        constexpr int kPerRow = TB / 16;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(lut + ((size_t)row0 << B));
        for (int i = tid; i < ng * kRowsPerGroup * kPerRow; i += nth) {
            const int r = i / kPerRow;
            *reinterpret_cast<u32x4 *>(tab + r * STRIDE + (i % kPerRow) * 16) = r < nrows ? src[i] : u32x4{0, 0, 0, 0};
        }
    } else {
        constexpr int kDwordsPerRow = (1 << B) / 2;
        const uint32_t *src = reinterpret_cast<const uint32_t *>(lut + ((size_t)row0 << B));
        for (int i = tid; i < ng * kRowsPerGroup * kDwordsPerRow; i += nth) {
            const int r = i / kDwordsPerRow, k = i % kDwordsPerRow;
            const uint32_t v = r < nrows ? src[i] : 0u;
            uint8_t *dst = tab + r * STRIDE + T::stored_addr(2 * k);
            *reinterpret_cast<uint16_t *>(dst) = (uint16_t)v;
            *reinterpret_cast<uint16_t *>(dst + 4) = (uint16_t)(v >> 16);
        }
    }
}

// Packed centroid pairs of run t of one row: element j holds columns 2j, 2j+1 (Section 5.2, steps 3-4).
template <int B>
__device__ __forceinline__ u32x4 lookup_run(const uint32_t (&W)[8], int t, const uint8_t *trow, uint32_t one)
{
    using T = Table<B>;
    u32x4 P;
    if constexpr (T::kPair) {
        const uint32_t v = W[2 * t];
        P[0] = *reinterpret_cast<const uint32_t *>(trow + byte_and<0>(v, 0xFCu));
        P[1] = *reinterpret_cast<const uint32_t *>(trow + byte_and<1>(v, 0xFCu));
        P[2] = *reinterpret_cast<const uint32_t *>(trow + byte_and<2>(v, 0xFCu));
        P[3] = *reinterpret_cast<const uint32_t *>(trow + byte_and<3>(v, 0xFCu));
    } else {
        const uint32_t v0 = W[2 * t], v1 = W[2 * t + 1];
        const uint32_t a0[4] = {byte_to_addr<B, 0>(v0, T::addr_mask(), one), byte_to_addr<B, 1>(v0, T::addr_mask(), one),
                                byte_to_addr<B, 2>(v0, T::addr_mask(), one), byte_to_addr<B, 3>(v0, T::addr_mask(), one)};
        const uint32_t a1[4] = {byte_to_addr<B, 0>(v1, T::addr_mask(), one), byte_to_addr<B, 1>(v1, T::addr_mask(), one),
                                byte_to_addr<B, 2>(v1, T::addr_mask(), one), byte_to_addr<B, 3>(v1, T::addr_mask(), one)};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t w0 = *reinterpret_cast<const uint16_t *>(trow + a0[j]);
            const uint32_t w1 = *reinterpret_cast<const uint16_t *>(trow + a1[j]);
            P[j] = w0 | (w1 << 16);
        }
    }
    return P;
}

} // namespace apgemv
#endif
