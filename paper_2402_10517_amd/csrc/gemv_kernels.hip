// Any-precision GEMV kernels for gfx950 (CDNA4, wave64) and their launcher.
//
// Steps of one call (Any-Precision LLM, Section 5.2, the five thread-level operations): load the
// first b bit slices of the lane's weights and the matching activations, turn the slices into
// table indices, fetch centroids from the table rows staged in LDS, multiply-accumulate, reduce
// over the lanes that share an output channel.  How each step is done differs from the paper's
// kernel, which was written for 32-wide warps:
//   * index formation needs no bit transpose: the slices are stored pre-rotated (layout.h), so the
//     eight words of four table indices each come out of a shared three-level tree of bit-selects
//     with constant masks (24 selects per 32 weights at 8 bits) and one rotate per word;
//   * b = 3 looks two weights up at once in a 64-entry table of centroid pairs and feeds the
//     pair to one packed dot product (Section 5.3 "Merging Table Lookups");
//   * a lane keeps its 32 activations in registers for 4 output rows;
//   * the reduction over lanes uses DPP row operations, then LDS across the waves of the group.
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

// d = (m & a) | (~m & b) with a constant mask: one v_bfi_b32 (the mask sits in an SGPR)
__device__ __forceinline__ uint32_t bitsel(uint32_t m, uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(d) : "s"(m), "v"(a), "v"(b));
    return d;
}
// (byte J of v) & mask, and (byte J of v) << 1: one SDWA instruction each.  They turn a byte of a
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
template <int B>
__device__ __forceinline__ void stage_tables_load(StagedTable<B> &st, const uint16_t *__restrict__ lut, int row0, int M)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    const int tid = threadIdx.x, nth = blockDim.x;
    const int last_row = M - 1 - row0; // >= 0
    if constexpr (B == 3) {
        // natural 8-entry rows: 4 rows x 4 dwords
        const int i = tid < kRowsPerGroup * 4 ? tid : kRowsPerGroup * 4 - 1;
        const int r = i >> 2;
        const int rc = r < last_row ? r : last_row;
        const uint32_t v = reinterpret_cast<const uint32_t *>(lut + (size_t)row0 * 8)[rc * 4 + (i & 3)];
        st.v[0].x = r <= last_row ? v : 0u;
    } else if constexpr (B >= 6) {
        // stored order = LDS order, rows contiguous: 16-byte pieces
        constexpr int kPerRow = TB / 16;
        constexpr int kChunks = kRowsPerGroup * kPerRow;
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
__device__ __forceinline__ void stage_tables_store(const StagedTable<B> &st, uint8_t *tab, uint16_t *nat)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    static_assert(STRIDE >= TB, "row stride in LDS");
    constexpr int kDummy = kRowsPerGroup * STRIDE; // byte offset of the dummy area inside tab
    const int tid = threadIdx.x, nth = blockDim.x;
    if constexpr (B == 3) {
        // the 64-entry table of centroid pairs: pair index bit 2k is code bit k of the even slot,
        // bit 2k+1 is code bit k of the odd slot.
        uint32_t *dst = tid < kRowsPerGroup * 4 ? reinterpret_cast<uint32_t *>(nat) + tid
                                                : reinterpret_cast<uint32_t *>(tab + kDummy);
        *dst = st.v[0].x;
        __syncthreads();
        // a thread's pair index is its lane (the block size is a multiple of 64): the two codes are
        // formed once, the loop only walks the rows
        const int i6 = tid & 63;
        const int a = (i6 & 1) | ((i6 >> 1) & 2) | ((i6 >> 2) & 4);
        const int c = ((i6 >> 1) & 1) | ((i6 >> 2) & 2) | ((i6 >> 3) & 4);
        for (int r = tid >> 6; r < kRowsPerGroup; r += nth >> 6) {
            const uint32_t v = (uint32_t)nat[r * 8 + a] | ((uint32_t)nat[r * 8 + c] << 16);
            *reinterpret_cast<uint32_t *>(tab + r * STRIDE + i6 * 4) = v;
        }
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
template <int B>
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
        W[u] = rotr_v(v, u);
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

// One workgroup per group of 4 rows; its waves stride over the row's spans of 2048 columns.
// The table loads go out first, then the wave's first slice loads, then the tables are written to
// LDS while the slice loads are still in flight; later
// spans are loaded after the previous one is consumed (other waves of the CU cover the latency;
// a second register set for prefetching cost more in occupancy than it gained).
template <int B, int NB, int MAXT>
__device__ __forceinline__ void gemv_group(const uint8_t *__restrict__ slices, size_t slice_bytes,
                                           const uint16_t *__restrict__ lut, const uint16_t *__restrict__ x,
                                           uint16_t *__restrict__ y, int M, int K, int batch, int g)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    __shared__ __attribute__((aligned(16))) uint8_t tab[kRowsPerGroup * TB + 16]; // + dummy area
    __shared__ __attribute__((aligned(16))) uint16_t nat[kRowsPerGroup * 8];
    __shared__ float red[MAXT / 64][NB][4][kRowsPerGroup]; // [wave][batch row][DPP row][lane & 3]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform, kept in an SGPR
    const int nwaves = blockDim.x >> 6;
    const int row0 = g * kRowsPerGroup;
    const int chunks = K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;

    u32x4 Q[B];
    u32x4 X[NB][4];
    // Loads of the lane's slice words and activations for one span (Section 5.2 step 1).
    auto issue_loads = [&](int span) {
        const int rem = chunks - span * kSpanLanes;
        const int nl = rem < kSpanLanes ? rem : kSpanLanes;
        {
            // Lanes past the end of a ragged last span load what the last valid lane loads (and are
            // masked out of the compute): no branch around the loads.
            // wave-uniform base + 32-bit lane offset: the loads use the scalar-base address form
            const uint8_t *sbase = slices + ((size_t)g * chunks + (size_t)span * kSpanLanes) * 16;
            const uint32_t loff = (uint32_t)(lane < nl ? lane : nl - 1) * 16u;
#pragma unroll
            for (int s = 0; s < B; ++s)
                Q[s] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(sbase + (size_t)s * slice_bytes + loff));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int xr = nb < batch ? nb : batch - 1;
                const uint8_t *xbase =
                    reinterpret_cast<const uint8_t *>(x + (size_t)xr * K + (size_t)span * kSpanCols);
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    X[nb][t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)(t * 16 * nl) + loff);
            }
        }
    };
    auto active = [&](int span) { return lane < chunks - span * kSpanLanes; };

    float acc[NB][kRowsPerGroup];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < kRowsPerGroup; ++r) acc[nb][r] = 0.f;

    int span = wave; // the launcher guarantees nwaves <= nspans
    StagedTable<B> st;
    stage_tables_load<B>(st, lut, row0, M);
    issue_loads(span);
    stage_tables_store<B>(st, tab, nat); // waits for the table loads only
    __syncthreads();
    while (true) {
        if (active(span)) compute_unit<B, NB>(Q, X, tab, acc);
        span += nwaves;
        if (span >= nspans) break;
        issue_loads(span);
    }

    // ---- reduce over lanes, then over the waves of the group (fixed order: deterministic)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float c = reduce4_in_dpp_rows(acc[nb], lane);
        if ((lane & 15) >= 12) red[wave][nb][lane >> 4][lane & 3] = c;
    }
    __syncthreads();
    if (threadIdx.x < kRowsPerGroup * NB) {
        const int nb = threadIdx.x / kRowsPerGroup, r = threadIdx.x % kRowsPerGroup;
        const int cls = ((r & 1) << 1) | (r >> 1); // lane & 3 that holds row r
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w)
            for (int d = 0; d < 4; ++d) s += red[w][nb][d][cls];
        const int row = row0 + r;
        if (row < M && nb < batch) {
            const __half h = __float2half_rn(s);
            y[(size_t)nb * M + row] = __builtin_bit_cast(uint16_t, h);
        }
    }
}

template <int B, int NB, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(2, (B <= 4 && NB == 1) ? 8 : 6))) void gemv_kernel(
    const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
    const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int M, int K, int batch)
{
    gemv_group<B, NB, MAXT>(slices, slice_bytes, lut, x, y, M, K, batch, blockIdx.x);
}

// Several matrices with the same row length in one launch (the q/k/v or gate/up projections of
// a decoder layer): workgroup -> (matrix, group of 4 rows) through the prefix sums of the group
// counts.  Each matrix keeps its own activations and outputs; the work per group is that of
// gemv_kernel, so results are bit-identical to separate calls that use it.
template <int B, int NB, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(2, 6))) void gemv_multi_kernel(MultiArgs a)
{
    int m = 0;
#pragma unroll
    for (int i = 1; i < kMaxMulti; ++i)
        if (i < a.count && (int)blockIdx.x >= a.group_begin[i]) m = i;
    gemv_group<B, NB, MAXT>(a.slices[m], a.slice_bytes[m], a.lut[m], a.x[m], a.y[m], a.M[m], a.K, a.batch,
                            (int)blockIdx.x - a.group_begin[m]);
}

// Variant for matrices with many rows and for batches: one workgroup owns up to kMaxRowGroups
// consecutive groups of 4 rows and each wave keeps its activations (one span, all batch rows) in
// registers across them, so activation traffic through the caches drops by that factor and the
// per-wave set-up is paid once.  The slice words of the next group are loaded while the current
// group is processed.  Requires one wave per span (the launcher checks).
constexpr int kMaxRowGroups = 4;

template <int B, int NB, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(1, 6))) void gemv_rows_kernel(
    const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
    const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int M, int K, int batch, int rg_per_wg)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    constexpr int kGroupBytes = kRowsPerGroup * TB;
    __shared__ __attribute__((aligned(16))) uint8_t tab[kMaxRowGroups * kGroupBytes];
    __shared__ __attribute__((aligned(16))) uint16_t nat[kMaxRowGroups * kRowsPerGroup * 8];
    __shared__ float red[MAXT / 64][kMaxRowGroups][NB][4][kRowsPerGroup];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform, kept in an SGPR
    const int nwaves = blockDim.x >> 6;
    const int tid = threadIdx.x, nth = blockDim.x;
    const int groups = (M + kRowsPerGroup - 1) / kRowsPerGroup;
    const int g0 = blockIdx.x * rg_per_wg;
    const int ng = groups - g0 < rg_per_wg ? groups - g0 : rg_per_wg;
    const int row0 = g0 * kRowsPerGroup;
    const int nrows = M - row0 < ng * kRowsPerGroup ? M - row0 : ng * kRowsPerGroup; // valid rows here
    const int chunks = K / kChunkSlots;
    const int span = wave; // one wave per span
    const int rem = chunks - span * kSpanLanes;
    const int nl = rem < kSpanLanes ? rem : kSpanLanes;
    const bool active = lane < nl;
    const uint32_t loff = (uint32_t)(active ? lane : nl - 1) * 16u;

    auto load_q = [&](u32x4 (&Q)[B], int rg) {
        const uint8_t *sbase = slices + ((size_t)(g0 + rg) * chunks + (size_t)span * kSpanLanes) * 16;
#pragma unroll
        for (int s = 0; s < B; ++s)
            Q[s] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4 *>(sbase + (size_t)s * slice_bytes + loff));
    };

    u32x4 X[NB][4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int xr = nb < batch ? nb : batch - 1;
        const uint8_t *xbase = reinterpret_cast<const uint8_t *>(x + (size_t)xr * K + (size_t)span * kSpanCols);
#pragma unroll
        for (int t = 0; t < 4; ++t)
            X[nb][t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)(t * 16 * nl) + loff);
    }
    u32x4 QA[B], QB[B];
    load_q(QA, 0);

    // ---- tables of all the groups of this workgroup (rows are contiguous in the stored tables)
    if constexpr (B == 3) {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(lut + (size_t)row0 * 8);
        for (int i = tid; i < ng * kRowsPerGroup * 4; i += nth)
            reinterpret_cast<uint32_t *>(nat)[i] = (i >> 2) < nrows ? src[i] : 0u;
        __syncthreads();
        for (int i = tid; i < ng * kRowsPerGroup * 64; i += nth) {
            const int r = i >> 6, i6 = i & 63;
            const int a = (i6 & 1) | ((i6 >> 1) & 2) | ((i6 >> 2) & 4);
            const int c = ((i6 >> 1) & 1) | ((i6 >> 2) & 2) | ((i6 >> 3) & 4);
            const uint32_t v = (uint32_t)nat[r * 8 + a] | ((uint32_t)nat[r * 8 + c] << 16);
            *reinterpret_cast<uint32_t *>(tab + r * TB + i6 * 4) = v;
        }
    } else if constexpr (B >= 6) {
        constexpr int kPerRow = TB / 16;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(lut + ((size_t)row0 << B));
        for (int i = tid; i < ng * kRowsPerGroup * kPerRow; i += nth)
            reinterpret_cast<u32x4 *>(tab)[i] = i / kPerRow < nrows ? src[i] : u32x4{0, 0, 0, 0};
    } else {
        constexpr int kDwordsPerRow = (1 << B) / 2;
        const uint32_t *src = reinterpret_cast<const uint32_t *>(lut + ((size_t)row0 << B));
        for (int i = tid; i < ng * kRowsPerGroup * kDwordsPerRow; i += nth) {
            const int r = i / kDwordsPerRow, k = i % kDwordsPerRow;
            const uint32_t v = r < nrows ? src[i] : 0u;
            uint8_t *dst = tab + r * TB + T::stored_addr(2 * k);
            *reinterpret_cast<uint16_t *>(dst) = (uint16_t)v;
            *reinterpret_cast<uint16_t *>(dst + 4) = (uint16_t)(v >> 16);
        }
    }
    __syncthreads();

    auto process = [&](const u32x4 (&Q)[B], int rg) {
        float acc[NB][kRowsPerGroup];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < kRowsPerGroup; ++r) acc[nb][r] = 0.f;
        if (active) compute_unit<B, NB>(Q, X, tab + rg * kGroupBytes, acc);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const float c = reduce4_in_dpp_rows(acc[nb], lane);
            if ((lane & 15) >= 12) red[wave][rg][nb][lane >> 4][lane & 3] = c;
        }
    };
    for (int rg = 0; rg < ng; rg += 2) {
        if (rg + 1 < ng) load_q(QB, rg + 1);
        process(QA, rg);
        if (rg + 1 >= ng) break;
        if (rg + 2 < ng) load_q(QA, rg + 2);
        process(QB, rg + 1);
    }
    __syncthreads();
    for (int i = tid; i < ng * kRowsPerGroup * NB; i += nth) {
        const int rg = i / (kRowsPerGroup * NB), nb = (i / kRowsPerGroup) % NB, r = i % kRowsPerGroup;
        const int cls = ((r & 1) << 1) | (r >> 1); // lane & 3 that holds row r
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w)
            for (int d = 0; d < 4; ++d) s += red[w][rg][nb][d][cls];
        const int row = row0 + rg * kRowsPerGroup + r;
        if (row < M && nb < batch) {
            const __half h = __float2half_rn(s);
            y[(size_t)nb * M + row] = __builtin_bit_cast(uint16_t, h);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Small-batch variant on the matrix cores (batch 3..8).  The paper's kernel runs batches on the
// ordinary ALUs and slows down by up to 2x at batch 8 (Section 6.2; Appendix C.3); here the
// multiply-accumulates of a batch go to v_mfma_f32_4x4x4_16B_f16, whose 16 independent 4x4x4
// blocks fit the layout's groups of 4 rows: block = 4 adjacent lanes, lane q of a block supplies
// A row q (4 consecutive weights of output row q) and B column q (the same 4 columns of batch row
// q), and receives D column q (4 output rows x batch row q).  For that a lane owns ONE row of the
// group and 4 chunks of the span (4 dword loads per slice instead of one 16-byte load), and
// the 4 rows' tables sit 256 (b <= 7) or 512 bytes apart so that the row is part of the LDS
// address.  Requires K % 128 == 0 (every block of 4 chunks is entirely inside or outside a span).
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
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
            const int a = (i6 & 1) | ((i6 >> 1) & 2) | ((i6 >> 2) & 4);
            const int c = ((i6 >> 1) & 1) | ((i6 >> 2) & 2) | ((i6 >> 3) & 4);
            const uint32_t v = (uint32_t)nat[r * 8 + a] | ((uint32_t)nat[r * 8 + c] << 16);
            *reinterpret_cast<uint32_t *>(tab + r * STRIDE + i6 * 4) = v;
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

// R = consecutive groups of 4 rows per workgroup: a lane's activations of a chunk are loaded once
// and used for R groups (activation traffic through the caches drops R-fold; at batch 8 it is
// otherwise 8 KB of activations per KB of 3-bit weights).
template <int B, int NBH, int R>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 6))) void gemv_mfma_kernel(
    const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
    const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int M, int K, int batch)
{
    using T = Table<B>;
    constexpr int STRIDE = B == 8 ? 512 : 256;
    constexpr int kGroupBytes = kRowsPerGroup * STRIDE;
    __shared__ __attribute__((aligned(16))) uint8_t tab[R * kGroupBytes];
    __shared__ __attribute__((aligned(16))) uint16_t nat[R * kRowsPerGroup * 8];
    __shared__ float red[8][R][NBH][4][4][4]; // [wave][group][batch half][output row][DPP row][batch row in half]

    const int lane = threadIdx.x & 63;
    const int q = lane & 3;      // row of a group this lane dequantises; batch row (in a half) it feeds
    const int quad = lane >> 2;  // block of the matrix instruction
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int groups = (M + kRowsPerGroup - 1) / kRowsPerGroup;
    const int g0 = blockIdx.x * R;
    const int ng = groups - g0 < R ? groups - g0 : R;
    const int row0 = g0 * kRowsPerGroup;
    const int nrows = M - row0 < ng * kRowsPerGroup ? M - row0 : ng * kRowsPerGroup;
    const int chunks = K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;

    stage_tables_groups<B, STRIDE>(tab, nat, lut, row0, nrows, ng);
    __syncthreads();

    float4_t D[R][NBH];
#pragma unroll
    for (int rg = 0; rg < R; ++rg)
#pragma unroll
        for (int h = 0; h < NBH; ++h) D[rg][h] = float4_t{0.f, 0.f, 0.f, 0.f};
    const uint32_t rowreg = (uint32_t)q;                  // B <= 7: row in address bits 8..9 via v_perm
    const uint32_t rowbase = (uint32_t)q * (uint32_t)STRIDE;
    const uint8_t *xrow[NBH];
#pragma unroll
    for (int h = 0; h < NBH; ++h) {
        const int br = 4 * h + q < batch ? 4 * h + q : batch - 1; // rows past the batch repeat the last one
        xrow[h] = reinterpret_cast<const uint8_t *>(x + (size_t)br * K);
    }

    // One span of 2048 columns: acc[rg][h] += partial products of this lane's block.
    auto run_span = [&](float4_t (&acc)[R][NBH], int span, int nl, int nq, int cq) {
        const uint8_t *sbase = slices + ((size_t)g0 * chunks + (size_t)span * kSpanLanes) * 16 + q * 4;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t c = (uint32_t)(p * nq + cq); // chunk inside the span
            u32x4 X[NBH][4];
#pragma unroll
            for (int h = 0; h < NBH; ++h)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    X[h][t] = *reinterpret_cast<const u32x4 *>(
                        xrow[h] + ((size_t)span * kSpanCols + (size_t)(t * 8 * nl) + c * 8u) * 2);
#pragma unroll
            for (int rg = 0; rg < R; ++rg) {
                if (rg >= ng) break;
                const uint8_t *tg = tab + rg * kGroupBytes;
                uint32_t Qw[B];
#pragma unroll
                for (int s = 0; s < B; ++s)
                    Qw[s] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(
                        sbase + (size_t)rg * chunks * 16 + (size_t)s * slice_bytes + c * 16u));
                uint32_t W[8];
                merge_words<B>(Qw, W);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    uint32_t P[4]; // packed centroid pairs of columns 2j, 2j+1 of run t
                    if constexpr (T::kPair) {
                        const uint32_t v = W[2 * t] & 0xFCFCFCFCu;
                        P[0] = *reinterpret_cast<const uint32_t *>(tg + row_byte_addr<0>(v, rowreg));
                        P[1] = *reinterpret_cast<const uint32_t *>(tg + row_byte_addr<1>(v, rowreg));
                        P[2] = *reinterpret_cast<const uint32_t *>(tg + row_byte_addr<2>(v, rowreg));
                        P[3] = *reinterpret_cast<const uint32_t *>(tg + row_byte_addr<3>(v, rowreg));
                    } else {
                        uint32_t a[2][4];
#pragma unroll
                        for (int hh = 0; hh < 2; ++hh) {
                            uint32_t v = W[2 * t + hh];
                            if constexpr (B == 8) {
#pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    a[hh][j] = (((v >> (8 * j)) & 0xFFu) << 1) | rowbase;
                            } else {
                                v &= T::addr_mask() * 0x01010101u;
                                a[hh][0] = row_byte_addr<0>(v, rowreg);
                                a[hh][1] = row_byte_addr<1>(v, rowreg);
                                a[hh][2] = row_byte_addr<2>(v, rowreg);
                                a[hh][3] = row_byte_addr<3>(v, rowreg);
                            }
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const uint32_t w0 = *reinterpret_cast<const uint16_t *>(tg + a[0][j]);
                            const uint32_t w1 = *reinterpret_cast<const uint16_t *>(tg + a[1][j]);
                            P[j] = w0 | (w1 << 16);
                        }
                    }
#pragma unroll
                    for (int kq = 0; kq < 2; ++kq) {
                        const u32x2 aw = {P[2 * kq], P[2 * kq + 1]};
#pragma unroll
                        for (int h = 0; h < NBH; ++h) {
                            const u32x2 bw = {X[h][t][2 * kq], X[h][t][2 * kq + 1]};
                            acc[rg][h] = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4_t, aw),
                                                                            __builtin_bit_cast(half4_t, bw),
                                                                            acc[rg][h], 0, 0, 0);
                        }
                    }
                }
            }
        }
    };

    for (int span = wave; span < nspans; span += nwaves) {
        const int rem = chunks - span * kSpanLanes;
        const int nl = rem < kSpanLanes ? rem : kSpanLanes;
        const int nq = nl >> 2; // blocks in use; block b owns chunks p*nq + b, p = 0..3, so that the
                                // blocks' loads of one p are adjacent in memory
        if (nq == kSpanLanes / 4) {
            run_span(D, span, nl, nq, quad);
        } else {
            // ragged last span: blocks past its end run on repeated data and their sums are dropped
            const bool active = quad < nq;
            float4_t Ds[R][NBH];
#pragma unroll
            for (int rg = 0; rg < R; ++rg)
#pragma unroll
                for (int h = 0; h < NBH; ++h) Ds[rg][h] = float4_t{0.f, 0.f, 0.f, 0.f};
            run_span(Ds, span, nl, nq, active ? quad : nq - 1);
#pragma unroll
            for (int rg = 0; rg < R; ++rg)
#pragma unroll
                for (int h = 0; h < NBH; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i) D[rg][h][i] += active ? Ds[rg][h][i] : 0.f;
        }
    }

    // D[rg][h][i] of lane (block, q): output row i of group rg, batch row 4h+q, summed over the block's
    // columns.  Add the 4 blocks of a DPP row (lanes with equal q), then waves and DPP rows through LDS.
#pragma unroll
    for (int rg = 0; rg < R; ++rg)
#pragma unroll
        for (int h = 0; h < NBH; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float c = D[rg][h][i];
                c += dpp_get<0x114>(c); // row_shr:4
                c += dpp_get<0x118>(c); // row_shr:8
                if ((lane & 15) >= 12) red[wave][rg][h][i][lane >> 4][q] = c;
            }
    __syncthreads();
    for (int o = threadIdx.x; o < ng * NBH * 16; o += blockDim.x) {
        const int rg = o / (NBH * 16), h = (o / 16) % NBH, i = (o >> 2) & 3, j = o & 3;
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w)
            for (int d = 0; d < 4; ++d) s += red[w][rg][h][i][d][j];
        const int row = row0 + rg * kRowsPerGroup + i, br = 4 * h + j;
        if (row < M && br < batch) {
            const __half hv = __float2half_rn(s);
            y[(size_t)br * M + row] = __builtin_bit_cast(uint16_t, hv);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Small-batch variant on the matrix cores that keeps the ALU kernels' lane ownership (a lane
// dequantises 4 rows x 32 columns, so every table lookup instruction reads ONE row's table and stays
// free of bank conflicts at b <= 6).  The matrix instruction wants the opposite: the 4 lanes of a
// block share 4 columns and hold one row each.  The packed centroid pairs are therefore exchanged
// between lanes through a 4 KB per-wave LDS buffer, one run of 8 columns per lane at a time: lane L
// writes row r at slot L ^ 2r of row r's 64 slots of 16 bytes; for its s-th instruction of a run,
// block n (lanes 4n..4n+3) takes the columns of source lane s*nq + n (nq = blocks in the span), so
// lane 4n+i reads row i from slot (s*nq + n) ^ 2i.  Both directions touch 8 different 16-byte bank
// groups per 8 lanes, and the activation loads of one instruction are contiguous across the blocks
// (256 bytes per batch row).  The multiply-accumulate cost no longer grows with the batch: per 128
// weights of a lane, 32 matrix instructions per half batch instead of 64 packed dot products per
// batch row.  Requires K % 128 == 0 (a block is entirely inside or outside a ragged last span).
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

// R consecutive groups of 4 rows per workgroup; the waves stride over the spans.  A wave's
// activations of a span (its batch rows x 2048 columns, 64 registers per half batch) are loaded once
// and reused for the R groups: without the reuse every group re-reads batch x 4 KB of activations
// per 2048 columns through the caches, which at batch 8 is 8 times the 3-bit weight bytes and
// bounds the kernel.  The slice words of the next unit are requested as soon as the current unit's
// index words are formed.  Per-span sums are reduced over the blocks and accumulated in LDS.
// LOOP = false: one wave per span (the launcher checks), straight-line code.
template <int B, int NBH, int R, bool LOOP>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 4))) void gemv_xmfma_kernel(
    const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
    const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int M, int K, int batch)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    constexpr int kGroupBytes = kRowsPerGroup * TB;
    __shared__ __attribute__((aligned(16))) uint8_t tab[R * kGroupBytes];
    __shared__ __attribute__((aligned(16))) uint16_t nat[R * kRowsPerGroup * 8];
    __shared__ __attribute__((aligned(16))) u32x4 xp[8][kRowsPerGroup][kSpanLanes];
    __shared__ float red[8][R][NBH][4][4][4]; // [wave][group][batch half][output row][DPP row][batch row in half]

    const int lane = threadIdx.x & 63;
    const int q = lane & 3;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int groups = (M + kRowsPerGroup - 1) / kRowsPerGroup;
    const int g0 = blockIdx.x * R;
    const int ng = groups - g0 < R ? groups - g0 : R;
    const int row0 = g0 * kRowsPerGroup;
    const int nrows = M - row0 < ng * kRowsPerGroup ? M - row0 : ng * kRowsPerGroup;
    const int chunks = K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;

    const uint8_t *xrow[NBH];
#pragma unroll
    for (int h = 0; h < NBH; ++h) {
        const int br = 4 * h + q < batch ? 4 * h + q : batch - 1; // rows past the batch repeat the last one
        xrow[h] = reinterpret_cast<const uint8_t *>(x + (size_t)br * K);
    }
    u32x4 Q[B];
    // lanes past the end of a ragged last span load what its last lane loads
    auto load_q = [&](int span, int rg) {
        const int rem = chunks - span * kSpanLanes;
        const int nl = rem < kSpanLanes ? rem : kSpanLanes;
        const uint32_t loff = (uint32_t)(lane < nl ? lane : nl - 1) * 16u;
        const uint8_t *sbase = slices + ((size_t)(g0 + rg) * chunks + (size_t)span * kSpanLanes) * 16;
#pragma unroll
        for (int s = 0; s < B; ++s)
            Q[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(sbase + (size_t)s * slice_bytes + loff));
    };
    load_q(wave, 0); // the launcher guarantees nwaves <= nspans
    stage_tables_groups<B, TB>(tab, nat, lut, row0, nrows, ng);
    __syncthreads();

    uint32_t one = 1;
    asm("" : "+v"(one));
    u32x4 *buf = &xp[wave][0][0];
    for (int span = wave; span < nspans; span += nwaves) {
        const int rem = chunks - span * kSpanLanes;
        const int nl = rem < kSpanLanes ? rem : kSpanLanes;
        const int nq = nl >> 2;
        const bool active = lane < nl;
        const int blk = active ? lane >> 2 : nq - 1;
        const bool first = !LOOP || span == wave;
        if (!first) load_q(span, 0);
        // activations: block blk takes the columns of source lane s*nq + blk for its s-th instruction
        u32x4 XB[NBH][4][4]; // [batch half][run t][instruction s]: 8 columns of this lane's batch row
        {
            const size_t span_col = (size_t)span * kSpanCols;
#pragma unroll
            for (int h = 0; h < NBH; ++h)
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        XB[h][t][s] = *reinterpret_cast<const u32x4 *>(
                            xrow[h] + (span_col + (size_t)(t * 8 * nl) + (size_t)((s * nq + blk) * 8)) * 2);
        }
        // unrolled over the groups: the table base of a group is then an immediate offset of the lookups
#pragma unroll
        for (int rg = 0; rg < R; ++rg) {
            if (rg >= ng) break;
            uint32_t W[kRowsPerGroup][8];
#pragma unroll
            for (int r = 0; r < kRowsPerGroup; ++r) merge_row<B>(Q, r, W[r]);
            if (rg + 1 < ng) load_q(span, rg + 1);
            float4_t D[NBH];
#pragma unroll
            for (int h = 0; h < NBH; ++h) D[h] = float4_t{0.f, 0.f, 0.f, 0.f};
            const uint8_t *tg = tab + rg * kGroupBytes;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int r = 0; r < kRowsPerGroup; ++r)
                    buf[r * kSpanLanes + (lane ^ (2 * r))] = lookup_run<B>(W[r], t, tg + r * TB, one);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const u32x4 A = buf[q * kSpanLanes + ((s * nq + blk) ^ (2 * q))];
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        const u32x2 aw = {A[2 * kk], A[2 * kk + 1]};
#pragma unroll
                        for (int h = 0; h < NBH; ++h) {
                            const u32x4 xb = XB[h][t][s];
                            const u32x2 bw = {xb[2 * kk], xb[2 * kk + 1]};
                            D[h] = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4_t, aw),
                                                                      __builtin_bit_cast(half4_t, bw), D[h], 0, 0, 0);
                        }
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            // D[h][i] of lane (block, q): output row i, batch row 4h+q, summed over the block's columns;
            // blocks past the end of a ragged span ran on repeated data and are dropped.  Add the 4
            // blocks of a DPP row (lanes with equal q) and accumulate over the wave's spans in LDS.
#pragma unroll
            for (int h = 0; h < NBH; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float c = active ? D[h][i] : 0.f;
                    c += dpp_get<0x114>(c); // row_shr:4
                    c += dpp_get<0x118>(c); // row_shr:8
                    if ((lane & 15) >= 12) {
                        float *dst = &red[wave][rg][h][i][lane >> 4][q];
                        *dst = first ? c : *dst + c;
                    }
                }
        }
        if (!LOOP) break;
    }
    __syncthreads();
    for (int o = threadIdx.x; o < ng * NBH * 16; o += blockDim.x) {
        const int rg = o / (NBH * 16), h = (o / 16) % NBH, i = (o >> 2) & 3, j = o & 3;
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w)
            for (int d = 0; d < 4; ++d) s += red[w][rg][h][i][d][j];
        const int row = row0 + rg * kRowsPerGroup + i, br = 4 * h + j;
        if (row < M && br < batch) {
            const __half hv = __float2half_rn(s);
            y[(size_t)br * M + row] = __builtin_bit_cast(uint16_t, hv);
        }
    }
}

template <int B, int NBH> static hipError_t launch_xmfma(const GemvArgs &a, hipStream_t stream)
{
    constexpr int kMaxWaves = 8;
    const int groups = padded_rows(a.M) / kRowsPerGroup;
    const int chunks = a.K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;
    // equal number of spans per wave where possible (14 spans: 7 waves x 2)
    const int rounds = (nspans + kMaxWaves - 1) / kMaxWaves;
    int nw = (nspans + rounds - 1) / rounds;
    if (a.waves_per_group > 0 && a.waves_per_group < nw) nw = a.waves_per_group;
    int rg = a.row_groups_per_wg;
    if (rg < 0) rg = groups >= 2048 ? 4 : 1;
    const bool loop = nw < nspans;
#define APGEMV_LAUNCH_X(RR, LL)                                                                              \
    hipLaunchKernelGGL((gemv_xmfma_kernel<B, NBH, RR, LL>), dim3((groups + RR - 1) / RR), dim3(64 * nw), 0, \
                       stream, a.slices, a.slice_bytes, a.lut, a.x, a.y, a.M, a.K, a.batch)
    if (rg >= 4) {
        if (loop) APGEMV_LAUNCH_X(4, true); else APGEMV_LAUNCH_X(4, false);
    } else if (rg >= 2) {
        if (loop) APGEMV_LAUNCH_X(2, true); else APGEMV_LAUNCH_X(2, false);
    } else {
        if (loop) APGEMV_LAUNCH_X(1, true); else APGEMV_LAUNCH_X(1, false);
    }
#undef APGEMV_LAUNCH_X
    return hipGetLastError();
}

template <int B, int NB>
static hipError_t launch_one(const GemvArgs &a, hipStream_t stream)
{
    // Up to 8 waves per group at batch 1 and 2 (measured best across the Llama shapes: long rows
    // then take two spans per wave); batch 4 and 8 hold 4 or 8 activation rows in registers and
    // are capped at 4 waves.
    constexpr int kMaxWaves = NB <= 4 ? 8 : 4;
    constexpr int kMaxThreads = 64 * kMaxWaves;
    const int groups = padded_rows(a.M) / kRowsPerGroup;
    const int chunks = a.K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;
    int nw = kMaxWaves;
    if (a.waves_per_group > 0 && a.waves_per_group < nw) nw = a.waves_per_group;
    if (nw > nspans) nw = nspans;
    // several row groups per workgroup at batch 5..8 when every span has its own wave and there are
    // enough groups to keep the device full (at batch 2..4 the plain kernel measured faster)
    int rg = a.row_groups_per_wg;
    if (rg < 0) rg = (nspans <= kMaxWaves && groups >= 2048 && NB >= 8) ? kMaxRowGroups : 1;
    if (rg > kMaxRowGroups) rg = kMaxRowGroups;
    if (rg > 1 && nspans <= kMaxWaves) {
        hipLaunchKernelGGL((gemv_rows_kernel<B, NB, kMaxThreads>), dim3((groups + rg - 1) / rg),
                           dim3(64 * nspans), 0, stream, a.slices, a.slice_bytes, a.lut, a.x, a.y, a.M,
                           a.K, a.batch, rg);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((gemv_kernel<B, NB, kMaxThreads>), dim3(groups), dim3(64 * nw), 0, stream,
                       a.slices, a.slice_bytes, a.lut, a.x, a.y, a.M, a.K, a.batch);
    return hipGetLastError();
}

template <int B, int NBH> static hipError_t launch_mfma(const GemvArgs &a, hipStream_t stream)
{
    const int groups = padded_rows(a.M) / kRowsPerGroup;
    const int chunks = a.K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;
    int nw = 8;
    if (a.waves_per_group > 0 && a.waves_per_group < nw) nw = a.waves_per_group;
    if (nw > nspans) nw = nspans;
    int rg = a.row_groups_per_wg;
    if (rg < 0) rg = groups >= 2048 ? 4 : 1;
    if (rg >= 4)
        hipLaunchKernelGGL((gemv_mfma_kernel<B, NBH, 4>), dim3((groups + 3) / 4), dim3(64 * nw), 0, stream,
                           a.slices, a.slice_bytes, a.lut, a.x, a.y, a.M, a.K, a.batch);
    else if (rg >= 2)
        hipLaunchKernelGGL((gemv_mfma_kernel<B, NBH, 2>), dim3((groups + 1) / 2), dim3(64 * nw), 0, stream,
                           a.slices, a.slice_bytes, a.lut, a.x, a.y, a.M, a.K, a.batch);
    else
        hipLaunchKernelGGL((gemv_mfma_kernel<B, NBH, 1>), dim3(groups), dim3(64 * nw), 0, stream, a.slices,
                           a.slice_bytes, a.lut, a.x, a.y, a.M, a.K, a.batch);
    return hipGetLastError();
}

template <int B> static hipError_t launch_b(const GemvArgs &a, hipStream_t stream)
{
    // Batch 3..8 at b >= 6 goes to the matrix cores when the row length allows it: measured 7-18 %
    // faster than the ALU kernels there, slower at b <= 5, where the four rows' small tables of a
    // block share LDS banks (mfma_min_batch: tuning override; a negative value also lifts the b limit)
    // Which kernel for batch >= 2 was settled by measurement on the 70B shapes (8192x8192, 28672x8192,
    // 8192x28672; all b):
    //  * batch 2: the plain kernel (one group of rows per workgroup) wins everywhere;
    //  * batch 5..8 with >= 2048 groups of rows: the matrix-core kernel with in-wave exchange, every b
    //    (up to 24 % faster than the ALU kernels at b <= 5, level at b = 8);
    //  * batch 3..4: that kernel for b >= 6 and, on the tallest matrices (>= 4096 groups), for b = 4, 5,
    //    when every span has its own wave; b = 3 and short matrices stay on the plain kernel, long
    //    rows at b >= 6 on the first matrix-core kernel.
    // variant: 1 = never the in-wave-exchange kernel, 3 = whenever the shape allows (tuning overrides).
    if (a.batch >= 2 && a.K % 128 == 0 && a.variant != 1) {
        const int groups = padded_rows(a.M) / kRowsPerGroup;
        const int nspans = (a.K / kChunkSlots + kSpanLanes - 1) / kSpanLanes;
        const bool one_wave_per_span = nspans <= 8;
        bool pays = false;
        if (groups >= 2048 && a.row_groups_per_wg < 0 && a.mfma_min_batch == 0) {
            if (a.batch >= 5) pays = true;
            else if (a.batch >= 3 && one_wave_per_span) pays = B >= 6 || (B >= 4 && groups >= 4096);
        }
        if (a.variant == 3 || pays)
            return a.batch <= 4 ? launch_xmfma<B, 1>(a, stream) : launch_xmfma<B, 2>(a, stream);
    }
    const int min_batch = a.mfma_min_batch > 0 ? a.mfma_min_batch : a.mfma_min_batch < 0 ? -a.mfma_min_batch : 3;
    if (a.batch >= min_batch && a.K % 128 == 0 && (B >= 6 || a.mfma_min_batch < 0))
        return a.batch <= 4 ? launch_mfma<B, 1>(a, stream) : launch_mfma<B, 2>(a, stream);
    if (a.batch == 1) return launch_one<B, 1>(a, stream);
    if (a.batch == 2) return launch_one<B, 2>(a, stream);
    if (a.batch <= 4) return launch_one<B, 4>(a, stream);
    return launch_one<B, 8>(a, stream);
}

// Dequantise kernel (Section 6.2, "Matrix-Matrix Multiplication Performance": above a batch
// threshold the engine dequantises the weights with a separate kernel and hands them to a dense
// FP16 GEMM).  Same unit walk as the GEMV: a lane forms the table indices of its 32 slots of 4
// rows and, instead of multiplying, writes the centroids as dense binary16: 8 consecutive columns
// (16 bytes) per row and run, 1 KB contiguous per wave and row.
template <int B>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 6))) void dequant_kernel(
    const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
    uint16_t *__restrict__ w, int M, int K)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    __shared__ __attribute__((aligned(16))) uint8_t tab[kRowsPerGroup * TB + 16];
    __shared__ __attribute__((aligned(16))) uint16_t nat[kRowsPerGroup * 8];
    const int g = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int row0 = g * kRowsPerGroup;
    const int chunks = K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;

    StagedTable<B> st;
    stage_tables_load<B>(st, lut, row0, M);
    stage_tables_store<B>(st, tab, nat);
    __syncthreads();
    uint32_t one = 1;
    asm("" : "+v"(one));
    for (int span = wave; span < nspans; span += nwaves) {
        const int rem = chunks - span * kSpanLanes;
        const int nl = rem < kSpanLanes ? rem : kSpanLanes;
        if (lane >= nl) continue;
        const uint8_t *sbase = slices + ((size_t)g * chunks + (size_t)span * kSpanLanes) * 16;
        u32x4 Q[B];
#pragma unroll
        for (int s = 0; s < B; ++s)
            Q[s] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4 *>(sbase + (size_t)s * slice_bytes + (uint32_t)lane * 16u));
#pragma unroll
        for (int r = 0; r < kRowsPerGroup; ++r) {
            const uint8_t *trow = tab + r * TB;
            u32x4 out[4]; // out[t][j] = columns 2j, 2j+1 of run t
            uint32_t W[8];
            merge_row<B>(Q, r, W);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if constexpr (T::kPair) {
                    const uint32_t v = W[2 * t];
                    out[t][0] = *reinterpret_cast<const uint32_t *>(trow + byte_and<0>(v, 0xFCu));
                    out[t][1] = *reinterpret_cast<const uint32_t *>(trow + byte_and<1>(v, 0xFCu));
                    out[t][2] = *reinterpret_cast<const uint32_t *>(trow + byte_and<2>(v, 0xFCu));
                    out[t][3] = *reinterpret_cast<const uint32_t *>(trow + byte_and<3>(v, 0xFCu));
                } else {
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
                        const uint32_t w0 = *reinterpret_cast<const uint16_t *>(trow + a[0][j]);
                        const uint32_t w1 = *reinterpret_cast<const uint16_t *>(trow + a[1][j]);
                        out[t][j] = w0 | (w1 << 16);
                    }
                }
            }
            const int row = row0 + r;
            if (row < M) {
                uint16_t *wrow = w + (size_t)row * K + (size_t)span * kSpanCols + lane * 8;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    __builtin_nontemporal_store(out[t], reinterpret_cast<u32x4 *>(wrow + t * 8 * nl));
            }
        }
    }
}

template <int B> static hipError_t launch_dequant_b(const GemvArgs &a, hipStream_t stream)
{
    const int groups = padded_rows(a.M) / kRowsPerGroup;
    const int chunks = a.K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;
    const int nw = nspans < 8 ? nspans : 8;
    hipLaunchKernelGGL((dequant_kernel<B>), dim3(groups), dim3(64 * nw), 0, stream, a.slices,
                       a.slice_bytes, a.lut, a.y, a.M, a.K);
    return hipGetLastError();
}

// a.y is the dense output (M*K binary16, row-major); a.x and a.batch are unused
hipError_t launch_dequantize(const GemvArgs &a, hipStream_t stream)
{
    switch (a.b) {
    case 3: return launch_dequant_b<3>(a, stream);
    case 4: return launch_dequant_b<4>(a, stream);
    case 5: return launch_dequant_b<5>(a, stream);
    case 6: return launch_dequant_b<6>(a, stream);
    case 7: return launch_dequant_b<7>(a, stream);
    case 8: return launch_dequant_b<8>(a, stream);
    }
    return hipErrorInvalidValue;
}

// Plain read of known size with the slice loads' instruction and access shape (calibration of
// profiling counters); each lane reads 4 x 16 bytes, a wave 4 x 1 KB.
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4 *__restrict__ p, uint32_t *sink)
{
    const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    uint32_t a = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const u32x4 v = __builtin_nontemporal_load(p + (wave * 4 + k) * 64 + lane);
        a ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (a == 0x9e3779b9u && sink) *sink = a; // keeps the loads alive; sink is null in practice
}

hipError_t launch_probe_read(const void *dev_buf, size_t bytes, hipStream_t stream)
{
    const size_t blocks = bytes / 16384; // 256 threads x 64 bytes
    hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<const u32x4 *>(dev_buf), static_cast<uint32_t *>(nullptr));
    return hipGetLastError();
}

template <int B, int NB> static hipError_t launch_multi_one(const MultiArgs &a, int total_groups, hipStream_t stream)
{
    constexpr int kMaxWaves = NB <= 4 ? 8 : 4;
    const int chunks = a.K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;
    const int nw = nspans < kMaxWaves ? nspans : kMaxWaves;
    hipLaunchKernelGGL((gemv_multi_kernel<B, NB, 64 * kMaxWaves>), dim3(total_groups), dim3(64 * nw), 0, stream, a);
    return hipGetLastError();
}

template <int B> static hipError_t launch_multi_b(const MultiArgs &a, int total_groups, hipStream_t stream)
{
    if (a.batch == 1) return launch_multi_one<B, 1>(a, total_groups, stream);
    if (a.batch == 2) return launch_multi_one<B, 2>(a, total_groups, stream);
    if (a.batch <= 4) return launch_multi_one<B, 4>(a, total_groups, stream);
    return launch_multi_one<B, 8>(a, total_groups, stream);
}

hipError_t launch_gemv_multi(const MultiArgs &a, int b, int total_groups, hipStream_t stream)
{
    switch (b) {
    case 3: return launch_multi_b<3>(a, total_groups, stream);
    case 4: return launch_multi_b<4>(a, total_groups, stream);
    case 5: return launch_multi_b<5>(a, total_groups, stream);
    case 6: return launch_multi_b<6>(a, total_groups, stream);
    case 7: return launch_multi_b<7>(a, total_groups, stream);
    case 8: return launch_multi_b<8>(a, total_groups, stream);
    }
    return hipErrorInvalidValue;
}

// Bit-width dispatch: one stored matrix, the kernel and the table are chosen per call
// (Section 5.2: only the first b slices and the b-bit table are touched).
hipError_t launch_gemv(const GemvArgs &a, hipStream_t stream)
{
    switch (a.b) {
    case 3: return launch_b<3>(a, stream);
    case 4: return launch_b<4>(a, stream);
    case 5: return launch_b<5>(a, stream);
    case 6: return launch_b<6>(a, stream);
    case 7: return launch_b<7>(a, stream);
    case 8: return launch_b<8>(a, stream);
    }
    return hipErrorInvalidValue;
}

} // namespace apgemv
