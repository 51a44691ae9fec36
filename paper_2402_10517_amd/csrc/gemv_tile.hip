// Small-batch kernel (batch 2..8) that feeds v_mfma_f32_16x16x32_f16 from the dequantising lanes
// (Section 6.2 "Matrix-Matrix Multiplication Performance": the paper's kernel runs batches on the
// ordinary ALUs and slows down by up to 2x at batch 8).
//
// In that instruction lane l supplies A[l % 16][8 (l / 16) .. + 7] and B[8 (l / 16) .. + 7][l % 16] and
// receives D[4 (l / 16) .. + 3][l % 16].  With A = weights and B = activations this fixes who owns
// what: lane (i, kg) = (l % 16, l / 16) dequantises row i of a tile of 16 rows, 8 columns per
// instruction; the multiply-accumulate cost does not depend on the batch.
//   * A wave works on octets of chunks (8 chunks = 256 columns of the tile's 16 rows): two quads of
//     chunks, lane group kg taking chunk kg of the first and chunk 4 + kg of the second.
//   * Every load instruction reads whole 128-byte lines in lane order.  A slice load covers 2 row groups
//     x 8 chunks x 4 rows (lane 32 p + 4 c + r: group p, chunk c ^ 2 p, row r), two loads per slice and
//     tile; one v_permlane16_swap turns the pair into the words of the first and of the second quad (all
//     4 row groups each), and one ds_bpermute per word moves a word to the lane that dequantises it
//     (lane 16 kg + 4 g + r: group g, row r).  Loaded directly in that order, every 4 lanes would touch
//     another cache line and a line would be requested again while it is still in flight.
//   * The activations of a run of an octet are 128 contiguous bytes per batch row: lane 8 n + p loads
//     16 bytes of batch row n (chunk p ^ 2 (n / 4)), so one instruction covers 8 batch rows line by line
//     (a lane-per-row order costs one cache access per lane).  Four ds_bpermute per run move them to the
//     lanes of the matrix instruction: lane (i, kg) takes batch row i % 8, chunk 4 (i / 8) + kg.  The
//     chunk exchanges (^ 2 p, ^ 2 (n / 4)) make the 32 source lanes of each half of a ds_bpermute
//     different mod 32, which is what that instruction needs to run without bank conflicts.  Both
//     quads of the octet use that register as B: output columns 0..7 of the first quad's instruction
//     and columns 8..15 of the second's are the products wanted (batch rows 0..7 each), the other
//     halves multiply one quad's weights with the other quad's activations and are dropped, so each
//     quad has its own accumulator and the final sum takes column n of one and n + 8 of the other.
//     Batch rows that do not exist read zeros (their buffer offset is out of range: no memory traffic).
//   * One instruction takes one run of 8 consecutive columns: their indices are the bytes of the
//     merged words of the run's even and odd slots, the activations the lane's 16 bytes of that run.
//   * The LDS serves 32 lanes per clock, here 16 rows x 2 lane groups, so every (row, lane group
//     parity) gets a bank of its own: each row's table is stored twice, entry v of row i for lane
//     groups of parity c is the low half of the dword at (v << s) | (c << 6) | (i << 2); no two lanes
//     of a clock share a bank.  For b <= 7, s = 8 and v = the index byte shifted down to its lowest
//     used bit (the index words are rotated that much further and masked, once per 4 lookups), so
//     that one v_perm_b32 per lookup builds the address from the word's byte and the lane's base; for
//     b = 8 that would need 64 KB per tile, so s = 7 and the address takes two operations (a byte
//     select and a shift-or).  The 3-bit path keeps its 64-entry table of centroid pairs, one pair
//     per dword.  The 4-bit path looks pairs up as well: slice 3 is rotated to rotation 0 so that a
//     merged byte is the 8-bit index of a column pair (8 selects and 4 rotates per 32 weights instead
//     of 14 and 7, no clean-up), a row's 256 pair entries are built in LDS from its 16 stored
//     centroids, two copies, entry p of row i at (p << 7) | (c << 6) | (i << 2) (two operations per
//     address, but per pair, and no pack before the matrix instruction).  Here that pays (same box,
//     alternating runs at batch 8: 28672 x 8192 46 -> 39 us, 8192 x 8192 16 -> 13.5, 8192 x 28672
//     46 -> 36), once the table build is cheap (below); in the batch-1 kernel, where all 64 lanes gather
//     from one row's 256 dwords, the bank conflicts eat the gain.
// Requires K % 256 == 0 (an octet is entirely inside or outside a ragged last span) and batch <= 8.
#include <type_traits>
#include "device_common.h"
#include "launchers.h"

namespace apgemv {

template <int B> struct TileTable {
    static constexpr bool kPair = (B == 3);
    // 4 bits: a 256-entry table of centroid pairs per row, two copies like the other tables: entry p of row i
    // for lane groups of parity c at (p << 7) | (c << 6) | (i << 2)
    static constexpr bool kPair4 = (B == 4);
    static constexpr uint32_t kMask = kPair ? 0xFCu : Table<B>::addr_mask(); // index bits inside a merged byte
    static constexpr int kLow = (kMask & 1) ? 0 : (kMask & 2) ? 1 : 2;       // lowest of them
    static constexpr bool kPerm = (B <= 7);                                  // address by one v_perm_b32
    static constexpr int kExtra = kPerm ? kLow : 0;                          // extra rotation of the index words
    static constexpr uint32_t kClean = (kMask >> kExtra) * 0x01010101u;      // index bits of the rotated words
    static constexpr int kShift = kPerm ? 8 : 7 - kLow;                      // entry value -> address
    static constexpr int kTileBytes = kPair4 ? 256 * 128 : (int)((kMask >> kLow) + 1) << (kPerm ? 8 : 7); // 16 rows x 2 copies x 4 bytes per entry (x 2 unused)
    // value in a (rotated) index byte of the entry stored at position p of a row (lut_stored_pos order; pair index for B = 3)
    __device__ static constexpr uint32_t byte_of(uint32_t p)
    {
        return (kPair ? p << 2 : B == 4 ? (((p & 8u) << 3) | ((p & 7u) << 2)) : p << kLow) >> kExtra;
    }
    // LDS address of the entry selected by byte J of the index word w, for a lane with base `rowbase` (< 128)
    template <int J> __device__ static __forceinline__ uint32_t addr(uint32_t w, uint32_t rowbase)
    {
        if constexpr (kPerm) return __builtin_amdgcn_perm(rowbase, w, 0x0c0c0004u | ((uint32_t)J << 8));
        else return (byte_and<J>(w, kMask) << kShift) | rowbase;
    }
};

// `wg` = index of the workgroup within its matrix (R tiles each).
template <int B, int R, int MAXT>
__device__ __forceinline__ void gemv_tile_body(const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
                                               const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int M, int K, int batch,
                                               int wg)
{
    using TT = TileTable<B>;
    constexpr int kTileRows = 16, kTileGroups = kTileRows / kRowsPerGroup;
    // the tables during the main loop, then the waves' partial sums [wave][tile][row][batch row]
    constexpr int kTabBytes = R * TT::kTileBytes, kRedBytes = (MAXT / 64) * R * kTileRows * 16 * 4;
    __shared__ __attribute__((aligned(16))) uint8_t smem[kTabBytes > kRedBytes ? kTabBytes : kRedBytes];
    uint8_t *tab = smem;
    __shared__ __attribute__((aligned(16))) uint16_t nat[TT::kPair ? R * kTileRows * 10 : TT::kPair4 ? R * kTileRows * 18 : 8]; // the rows as stored (pair paths)
    float(*red)[R][kTileRows][16] = reinterpret_cast<float(*)[R][kTileRows][16]>(smem);

    const int tid = threadIdx.x, nth = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = nth >> 6;
    const int i = lane & 15;  // row of a tile this lane dequantises; output column (batch row) it receives
    const int kg = lane >> 4; // its 8 columns of every instruction; its chunk of every quad of chunks
    const int groups = (M + kRowsPerGroup - 1) / kRowsPerGroup;
    const int g0 = wg * (R * kTileGroups);
    const int row0 = g0 * kRowsPerGroup;
    const int chunks = K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;

    // ---- per-lane offsets of the slice loads: lane 32 p + 4 c + r loads row r of row group 2 half + p of
    // the tile, chunk c ^ 2 p of the octet (16 lanes still read 64 contiguous bytes; the exchange of the
    // chunk pairs in the odd row groups keeps the lane exchange below free of bank conflicts)
    const int lp = lane >> 5, lc = ((lane >> 2) & 7) ^ (lp << 1), lr = lane & 3;
    const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(slices + (size_t)g0 * chunks * 16), 0, 0xffffffffu, kBufferRsrcWord3);
    uint32_t soff_lane[R][2];
#pragma unroll
    for (int tile = 0; tile < R; ++tile)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            int rg = tile * kTileGroups + 2 * half + lp;
            if (g0 + rg >= groups) rg = groups - 1 - g0; // past the matrix: the last group again (never stored)
            soff_lane[tile][half] = (uint32_t)(rg * chunks + lc) * 16u + (uint32_t)lr * 4u;
        }
    // After the swap of 16-lane rows, lane 16 p + 4 c + r of the first (second) word holds row r, chunk
    // c ^ 2 (g & 1) (plus 4) of the row group g at position p of the order 0, 2, 1, 3; this lane
    // dequantises row i & 3 of row group i >> 2, chunk kg (4 + kg).  ds_bpermute serves 32 lanes a clock
    // and two of them conflict when their source lanes are equal mod 32: with the chunk exchange the 32
    // sources of either half of the wave are all different (without it every exchange took two clocks
    // more).
    const int bperm_src = (((((i >> 2) & 1) << 1 | (i >> 3)) << 4) | ((kg ^ (((i >> 2) & 1) << 1)) << 2) | (i & 3)) << 2; // byte address of the source lane
    // activations: lane 8 n + p loads batch row n, chunk p ^ 2 (n / 4) of the octet (8 lanes = one 128-byte
    // line; the exchange for the same reason as above); the descriptor ends with the last batch row, and
    // lanes of rows past the batch carry an offset beyond it (batch * K * 2 < 2^31; valid lanes stay below
    // the end with any scalar offset).  This lane then takes batch row i & 7, chunk 4 (i >> 3) + kg.
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(x), 0, (uint32_t)batch * (uint32_t)K * 2u, kBufferRsrcWord3);
    const uint32_t xoff_lane = (lane >> 3) < batch ? (uint32_t)(lane >> 3) * (uint32_t)K * 2u +
                                                         (uint32_t)((lane & 7) ^ ((lane >> 5) << 1)) * 16u
                                                   : 0x80000000u;
    const int xperm_src = (((i & 7) << 3) | ((i >> 3) << 2) | (kg ^ (((i >> 2) & 1) << 1))) << 2; // byte address of the source lane
    const uint32_t rowbase = ((uint32_t)i << 2) | ((uint32_t)(kg & 1) << 6);
    uint32_t seven = 7; // shift amount of the 4-bit pair path's addresses, kept in a register (SDWA operand)
    asm("" : "+v"(seven));

    float4_t acc[R][2]; // one accumulator per quad of an octet: independent chains of matrix instructions
#pragma unroll
    for (int tile = 0; tile < R; ++tile) acc[tile][0] = acc[tile][1] = float4_t{0.f, 0.f, 0.f, 0.f};

    // Octet o of a row = chunks 8 o .. 8 o + 7 (span o / 8); the waves split the row's pairs of octets
    // evenly.  The loads of an octet are issued before the arithmetic of the octet before it (two
    // register sets).  Every pass of the loop issues the same loads and has no exit in the middle, so the
    // wait before the arithmetic leaves exactly the newer loads in flight: a row with an odd number of
    // octets gets one more whose activations are read as zeros (offset out of range), and the loads
    // issued in the last pass for the pass after it repeat a valid octet and are dropped.
    auto issue = [&](int o, bool real, u32x4 (&X)[4], uint32_t (&Q)[R][2][B]) {
        const int span = o >> 3, oi = o & 7;
        const int rem = chunks - span * kSpanLanes;
        const int nl = rem < kSpanLanes ? rem : kSpanLanes;
        const uint32_t xs = (uint32_t)span * (kSpanCols * 2u) + (uint32_t)oi * 128u;
        const uint32_t xoff = real ? xoff_lane : 0x80000000u;
#pragma unroll
        for (int t = 0; t < 4; ++t) X[t] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, xoff, xs + (uint32_t)(t * 16 * nl), 0);
        const uint32_t soct = (uint32_t)o * 128u;
#pragma unroll
        for (int tile = 0; tile < R; ++tile)
#pragma unroll
            for (int s = 0; s < B; ++s)
#pragma unroll
                for (int half = 0; half < 2; ++half)
                    Q[tile][half][s] = __builtin_amdgcn_raw_buffer_load_b32(srsrc, soff_lane[tile][half],
                                                                            soct + (uint32_t)s * (uint32_t)slice_bytes, kBufferNonTemporal);
    };
    auto compute = [&](const u32x4 (&Xl)[4], const uint32_t (&Q)[R][2][B]) {
        u32x4 X[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int d = 0; d < 4; ++d) X[t][d] = (uint32_t)__builtin_amdgcn_ds_bpermute(xperm_src, (int)Xl[t][d]);
#pragma unroll
        for (int tile = 0; tile < R; ++tile) {
            const uint8_t *tt = tab + tile * TT::kTileBytes;
            uint32_t W[2][8]; // [quad of the octet]
            {
                uint32_t q[2][B];
#pragma unroll
                for (int s = 0; s < B; ++s) {
                    const auto sw = __builtin_amdgcn_permlane16_swap(Q[tile][0][s], Q[tile][1][s], false, false);
                    q[0][s] = (uint32_t)__builtin_amdgcn_ds_bpermute(bperm_src, (int)sw[0]);
                    q[1][s] = (uint32_t)__builtin_amdgcn_ds_bpermute(bperm_src, (int)sw[1]);
                }
                if constexpr (TT::kPair4) {
                    merge_words_pair4(q[0], W[0]);
                    merge_words_pair4(q[1], W[1]);
                } else {
                    merge_words<B, TT::kExtra>(q[0], W[0]);
                    merge_words<B, TT::kExtra>(q[1], W[1]);
                }
                if constexpr (TT::kPerm && !TT::kPair4) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int u = 0; u < 8; u += TT::kPair ? 2 : 1) W[h][u] &= TT::kClean;
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint32_t P[2][4]; // packed centroid pairs: P[h][j] = columns 2j, 2j + 1 of run t, quad h
                if constexpr (TT::kPair || TT::kPair4) {
                    uint32_t ad[2][4];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t v = W[h][2 * t];
                        if constexpr (TT::kPair4) {
                            ad[h][0] = byte_shl1<0>(v, seven) | rowbase;
                            ad[h][1] = byte_shl1<1>(v, seven) | rowbase;
                            ad[h][2] = byte_shl1<2>(v, seven) | rowbase;
                            ad[h][3] = byte_shl1<3>(v, seven) | rowbase;
                        } else {
                            ad[h][0] = TT::template addr<0>(v, rowbase);
                            ad[h][1] = TT::template addr<1>(v, rowbase);
                            ad[h][2] = TT::template addr<2>(v, rowbase);
                            ad[h][3] = TT::template addr<3>(v, rowbase);
                        }
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int j = 0; j < 4; ++j) P[h][j] = *reinterpret_cast<const uint32_t *>(tt + ad[h][j]);
                } else {
                    uint32_t ae[2][4], ao[2][4];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t ve = W[h][2 * t], vo = W[h][2 * t + 1];
                        ae[h][0] = TT::template addr<0>(ve, rowbase);
                        ae[h][1] = TT::template addr<1>(ve, rowbase);
                        ae[h][2] = TT::template addr<2>(ve, rowbase);
                        ae[h][3] = TT::template addr<3>(ve, rowbase);
                        ao[h][0] = TT::template addr<0>(vo, rowbase);
                        ao[h][1] = TT::template addr<1>(vo, rowbase);
                        ao[h][2] = TT::template addr<2>(vo, rowbase);
                        ao[h][3] = TT::template addr<3>(vo, rowbase);
                    }
                    uint32_t we[2][4], wo[2][4];
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            we[h][j] = *reinterpret_cast<const uint16_t *>(tt + ae[h][j]);
                            wo[h][j] = *reinterpret_cast<const uint16_t *>(tt + ao[h][j]);
                        }
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int j = 0; j < 4; ++j) P[h][j] = we[h][j] | (wo[h][j] << 16);
                }
                // both quads against the same B: columns 0..7 of the first product and 8..15 of the second count
                const u32x4 a0 = {P[0][0], P[0][1], P[0][2], P[0][3]}, a1 = {P[1][0], P[1][1], P[1][2], P[1][3]};
                acc[tile][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a0), __builtin_bit_cast(half8_t, X[t]),
                                                                      acc[tile][0], 0, 0, 0);
                acc[tile][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a1), __builtin_bit_cast(half8_t, X[t]),
                                                                      acc[tile][1], 0, 0, 0);
            }
        }
    };

    const int nocts = chunks >> 3; // K % 256 == 0
    const int npairs = (nocts + 1) >> 1;
    const int p1 = (int)((long long)npairs * (wave + 1) / nwaves);
    u32x4 XA[4], XB[4];
    uint32_t QA[R][2][B], QB[R][2][B];
    int p = (int)((long long)npairs * wave / nwaves); // < p1: the launcher starts no more waves than pairs
    // ---- tables of the R tiles into LDS (rows past the matrix repeat the last row; never stored).
    // Thread (row = tid % 16, copy = (tid / 16) % 2, part = tid / 32) writes the entries of the pieces
    // part, part + nparts, ... of its row and copy: the 32 lanes of an LDS clock hit 32 different banks
    // (with one row per wave every lane of a store would land in the same bank).  A thread loads 16
    // bytes at a time and issues its loads before the first store that depends on them (one dword load
    // per loop pass cost a memory round trip per pass and one cache access per lane: 4 to 7 us per
    // workgroup).  The loads of the wave's first octet go out between the table loads and the table
    // stores, so that they are in flight during the stores and do not delay the tables (loads return in
    // order).
    {
        const int srow = tid & 15, scopy = (tid >> 4) & 1, part = tid >> 5, nparts = nth >> 5;
        if constexpr (TT::kPair4) {
            // the rows as stored (16 entries = 32 bytes each; 36 bytes apart in LDS, so that the rows fall on
            // different banks) first, then the 256 pair entries of every row and copy: thread (row, copy, part) writes
            // entries part + k * parts, 16 rows x 2 copies = 32 banks a clock.  With 256 or 512 threads the loop over k
            // is unrolled: the even and odd table positions are then the thread's own (from `part`) plus a
            // constant, i.e. an immediate offset of the LDS read, and an entry costs two reads, one pack and one
            // write.
            constexpr int kNatDwords = 9;
            for (int e = tid; e < R * kTileRows * 8; e += nth) {
                const int r = e >> 3;
                const int row = row0 + r < M ? row0 + r : M - 1;
                reinterpret_cast<uint32_t *>(nat)[r * kNatDwords + (e & 7)] = reinterpret_cast<const uint32_t *>(lut + (size_t)row * 16)[e & 7];
            }
            issue(2 * p, true, XA, QA);
            __syncthreads();
            auto build = [&](auto log2_parts) {
                constexpr int L = decltype(log2_parts)::value;
                const uint16_t *even = nat + srow * (2 * kNatDwords) + pair4_even(part);
                const uint16_t *odd = nat + srow * (2 * kNatDwords) + pair4_odd(part);
                uint8_t *base = tab + ((srow << 2) | (scopy << 6)) + (part << 7);
#pragma unroll
                for (int tile = 0; tile < R; ++tile)
#pragma unroll
                    for (int k = 0; k < (256 >> L); ++k)
                        *reinterpret_cast<uint32_t *>(base + tile * TT::kTileBytes + (k << (L + 7))) =
                            (uint32_t)even[tile * kTileRows * 2 * kNatDwords + pair4_even(k << L)] |
                            ((uint32_t)odd[tile * kTileRows * 2 * kNatDwords + pair4_odd(k << L)] << 16);
            };
            if (nth == 256) build(std::integral_constant<int, 3>{});
            else if (nth == 512) build(std::integral_constant<int, 4>{});
            else {
#pragma unroll
                for (int tile = 0; tile < R; ++tile) {
                    const uint16_t *src = nat + (tile * kTileRows + srow) * (2 * kNatDwords);
                    uint8_t *base = tab + tile * TT::kTileBytes + ((srow << 2) | (scopy << 6));
                    for (int d = part; d < 256; d += nparts)
                        *reinterpret_cast<uint32_t *>(base + (d << 7)) = (uint32_t)src[pair4_even(d)] | ((uint32_t)src[pair4_odd(d)] << 16);
                }
            }
        } else if constexpr (TT::kPair) {
            // natural rows (8 entries = 16 bytes each, 20 bytes apart in LDS: 16 rows on 16 banks) first, then the
            // pair entries from LDS; unrolled like the 4-bit build above (entries part + k * parts of a thread's
            // row and copy: the even and odd centroid of an entry sit at the thread's own offset + a constant)
            constexpr int kNatDwords = 5;
            for (int e = tid; e < R * kTileRows * 4; e += nth) {
                const int r = e >> 2;
                const int row = row0 + r < M ? row0 + r : M - 1;
                reinterpret_cast<uint32_t *>(nat)[r * kNatDwords + (e & 3)] = reinterpret_cast<const uint32_t *>(lut + (size_t)row * 8)[e & 3];
            }
            issue(2 * p, true, XA, QA);
            __syncthreads();
            auto build = [&](auto log2_parts) {
                constexpr int L = decltype(log2_parts)::value;
                const uint16_t *even = nat + srow * (2 * kNatDwords) + pair3_even(part);
                const uint16_t *odd = nat + srow * (2 * kNatDwords) + pair3_odd(part);
                uint8_t *base = tab + ((srow << 2) | (scopy << 6)) + (TT::byte_of(part) << TT::kShift);
#pragma unroll
                for (int tile = 0; tile < R; ++tile)
#pragma unroll
                    for (int k = 0; k < (64 >> L); ++k)
                        *reinterpret_cast<uint32_t *>(base + tile * TT::kTileBytes + (TT::byte_of(k << L) << TT::kShift)) =
                            (uint32_t)even[tile * kTileRows * 2 * kNatDwords + pair3_even(k << L)] |
                            ((uint32_t)odd[tile * kTileRows * 2 * kNatDwords + pair3_odd(k << L)] << 16);
            };
            if (nth == 256) build(std::integral_constant<int, 3>{});
            else if (nth == 512) build(std::integral_constant<int, 4>{});
            else {
#pragma unroll
                for (int tile = 0; tile < R; ++tile) {
                    uint8_t *base = tab + tile * TT::kTileBytes + ((srow << 2) | (scopy << 6));
                    for (int d = part; d < 64; d += nparts)
                        *reinterpret_cast<uint32_t *>(base + (TT::byte_of(d) << TT::kShift)) =
                            pair_entry(nat + (tile * kTileRows + srow) * (2 * kNatDwords), d);
                }
            }
        } else {
            constexpr int kPieces = (2 << B) / 16; // 16-byte pieces (8 entries) of a row's table
            constexpr int kBurst = 4;              // pieces per thread in the first pass: all of them from 4 waves on
            auto store_piece = [&](uint8_t *base, int pc, const u32x4 &v) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    *reinterpret_cast<uint16_t *>(base + (TT::byte_of(8 * pc + 2 * e) << TT::kShift)) = (uint16_t)v[e];
                    *reinterpret_cast<uint16_t *>(base + (TT::byte_of(8 * pc + 2 * e + 1) << TT::kShift)) = (uint16_t)(v[e] >> 16);
                }
            };
            const u32x4 *src[R];
            uint8_t *base[R];
            u32x4 v[R][kBurst];
#pragma unroll
            for (int tile = 0; tile < R; ++tile) {
                const int row = row0 + tile * kTileRows + srow < M ? row0 + tile * kTileRows + srow : M - 1;
                src[tile] = reinterpret_cast<const u32x4 *>(lut + ((size_t)row << B));
                base[tile] = tab + tile * TT::kTileBytes + ((srow << 2) | (scopy << 6));
#pragma unroll
                for (int j = 0; j < kBurst; ++j) {
                    const int pc = part + j * nparts;
                    v[tile][j] = src[tile][pc < kPieces ? pc : kPieces - 1];
                }
            }
            issue(2 * p, true, XA, QA);
#pragma unroll
            for (int tile = 0; tile < R; ++tile) {
#pragma unroll
                for (int j = 0; j < kBurst; ++j) {
                    const int pc = part + j * nparts;
                    if (pc < kPieces) store_piece(base[tile], pc, v[tile][j]);
                }
                // workgroups of fewer than 4 waves (rows of less than 2048 columns) at b >= 7: the rest
                for (int pc = part + kBurst * nparts; pc < kPieces; pc += nparts) store_piece(base[tile], pc, src[tile][pc]);
            }
        }
    }
    __syncthreads();

    for (; p < p1; ++p) {
        const bool second = 2 * p + 1 < nocts;
        issue(second ? 2 * p + 1 : 2 * p, second, XB, QB);
        __builtin_amdgcn_sched_barrier(0); // keep the loads ahead of the arithmetic they overlap with
        compute(XA, QA);
        issue(p + 1 < p1 ? 2 * p + 2 : 2 * p, true, XA, QA);
        __builtin_amdgcn_sched_barrier(0);
        compute(XB, QB);
    }

    // ---- acc[tile][h][r] of lane (i, kg): output row 4 kg + r of the tile over the wave's columns of quad
    //      h; column i of the h = 0 accumulator is batch row i for i < 8, column i of the h = 1 accumulator
    //      is batch row i - 8 for i >= 8.  Waves are added in fixed order
    __syncthreads(); // every wave is done with the tables, whose memory now takes the partial sums
#pragma unroll
    for (int tile = 0; tile < R; ++tile)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][tile][4 * kg + r][i] = i < 8 ? acc[tile][0][r] : acc[tile][1][r];
    __syncthreads();
    for (int o = tid; o < R * kTileRows * 8; o += nth) {
        const int n = o & 7, r = o >> 3; // r = row inside the workgroup's R tiles
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w) s += red[w][r >> 4][r & 15][n] + red[w][r >> 4][r & 15][n + 8];
        const int row = row0 + r;
        if (row < M && n < batch) {
            const __half hv = __float2half_rn(s);
            y[(size_t)n * M + row] = __builtin_bit_cast(uint16_t, hv);
        }
    }
}

template <int B, int R, int MAXT>
__global__ __launch_bounds__(MAXT) void gemv_tile_kernel(const uint8_t *__restrict__ slices, size_t slice_bytes,
                                                         const uint16_t *__restrict__ lut, const uint16_t *__restrict__ x,
                                                         uint16_t *__restrict__ y, int M, int K, int batch)
{
    gemv_tile_body<B, R, MAXT>(slices, slice_bytes, lut, x, y, M, K, batch, (int)blockIdx.x);
}

// Several matrices of equal row length at one bit-width and batch in one launch (the projections of a
// decoder layer that share their input): workgroup -> (matrix, tile) through the prefix sums of the
// tile counts, which the launcher puts into group_begin.
template <int B, int MAXT>
__global__ __launch_bounds__(MAXT) void gemv_tile_multi_kernel(MultiArgs a)
{
    int m = 0;
#pragma unroll
    for (int i = 1; i < kMaxMulti; ++i)
        if (i < a.count && (int)blockIdx.x >= a.group_begin[i]) m = i;
    gemv_tile_body<B, 1, MAXT>(a.slices[m], a.slice_bytes[m], a.lut[m], a.x[m], a.y[m], a.M[m], a.K, a.batch,
                               (int)blockIdx.x - a.group_begin[m]);
}

// A work list of matrices of any shapes (rows of one class of length) at one bit-width and batch.
template <int B, int MAXT>
__global__ __launch_bounds__(MAXT) void gemv_tile_list_kernel(ListArgs a, int batch)
{
    int it = 0;
#pragma unroll
    for (int i = 1; i < kMaxListItems; ++i)
        if (i < a.count && (int)blockIdx.x >= a.group_begin[i]) it = i;
    const ListItem &I = a.item[it];
    gemv_tile_body<B, 1, MAXT>(I.slices, I.slice_bytes, I.lut, I.x, I.y, I.M, I.K, batch, (int)blockIdx.x - a.group_begin[it]);
}

template <int B, int R> static hipError_t launch_tile_r(const GemvArgs &a, hipStream_t stream)
{
    constexpr int kMaxWaves = 8;
    const int npairs = (a.K / (8 * kChunkSlots) + 1) / 2;
    // short rows: 4 waves, so that a wave still runs several passes of its loop
    int nw = a.waves_per_group > 0 ? a.waves_per_group : a.K >= 12288 ? kMaxWaves : 4;
    if (nw > npairs) nw = npairs;
    const int tiles = (a.M + 15) / 16;
    hipLaunchKernelGGL((gemv_tile_kernel<B, R, 64 * kMaxWaves>), dim3((tiles + R - 1) / R), dim3(64 * nw), 0, stream, a.slices,
                       a.slice_bytes, a.lut, a.x, a.y, a.M, a.K, a.batch);
    return hipGetLastError();
}

template <int B> static hipError_t launch_tile_b(const GemvArgs &a, hipStream_t stream)
{
    // two tiles per workgroup re-read and re-arrange the activations half as often, at more registers:
    // measured faster on rows of 16384 columns or more, and at 3 bits (where the loads outweigh the
    // arithmetic) on matrices tall enough to fill the device with half as many workgroups (28672 x 8192 at
    // batch 4 and 8: 29-34 -> 28 us; 8192 x 8192: 11.8 -> 12.5, so not there)
    const int tiles = (a.M + 15) / 16;
    const int r = a.variant == 9 ? 1 : a.variant == 10 ? 2 : (a.K >= 16384 || (B == 3 && tiles >= 1536)) ? 2 : 1;
    if (r == 2) return launch_tile_r<B, 2>(a, stream);
    return launch_tile_r<B, 1>(a, stream);
}

template <int B> static hipError_t launch_tile_multi_b(MultiArgs &m, int total_tiles, hipStream_t stream)
{
    constexpr int kMaxWaves = 8;
    const int npairs = (m.K / (8 * kChunkSlots) + 1) / 2;
    int nw = m.K >= 12288 ? kMaxWaves : 4;
    if (nw > npairs) nw = npairs;
    hipLaunchKernelGGL((gemv_tile_multi_kernel<B, 64 * kMaxWaves>), dim3(total_tiles), dim3(64 * nw), 0, stream, m);
    return hipGetLastError();
}

// batch 2..8, K % 256 == 0 (the caller checks); one tile per workgroup
hipError_t launch_matrix_tile_multi(const MultiArgs &a, int b, hipStream_t stream)
{
    MultiArgs m = a;
    int total = 0;
    for (int i = 0; i < m.count; ++i) {
        m.group_begin[i] = total;
        total += (m.M[i] + 15) / 16;
    }
    switch (b) {
    case 3: return launch_tile_multi_b<3>(m, total, stream);
    case 4: return launch_tile_multi_b<4>(m, total, stream);
    case 5: return launch_tile_multi_b<5>(m, total, stream);
    case 6: return launch_tile_multi_b<6>(m, total, stream);
    case 7: return launch_tile_multi_b<7>(m, total, stream);
    case 8: return launch_tile_multi_b<8>(m, total, stream);
    }
    return hipErrorInvalidValue;
}

template <int B> static hipError_t launch_tile_list_b(const ListArgs &a, int total_tiles, int nw, int batch, hipStream_t stream)
{
    hipLaunchKernelGGL((gemv_tile_list_kernel<B, 512>), dim3(total_tiles), dim3(64 * nw), 0, stream, a, batch);
    return hipGetLastError();
}

hipError_t launch_matrix_tile_list(ListArgs &a, int b, int batch, hipStream_t stream)
{
    int total = 0, min_pairs = 1 << 30;
    bool long_rows = false;
    for (int i = 0; i < a.count; ++i) {
        a.group_begin[i] = total;
        total += (a.item[i].M + 15) / 16;
        const int npairs = (a.item[i].K / (8 * kChunkSlots) + 1) / 2;
        if (npairs < min_pairs) min_pairs = npairs;
        long_rows = a.item[i].K >= 12288;
    }
    for (int i = a.count; i < kMaxListItems; ++i) a.group_begin[i] = 0x7fffffff;
    int nw = long_rows ? 8 : 4; // as in single calls; no more waves than the shortest row has pairs of octets
    if (nw > min_pairs) nw = min_pairs;
    switch (b) {
    case 3: return launch_tile_list_b<3>(a, total, nw, batch, stream);
    case 4: return launch_tile_list_b<4>(a, total, nw, batch, stream);
    case 5: return launch_tile_list_b<5>(a, total, nw, batch, stream);
    case 6: return launch_tile_list_b<6>(a, total, nw, batch, stream);
    case 7: return launch_tile_list_b<7>(a, total, nw, batch, stream);
    case 8: return launch_tile_list_b<8>(a, total, nw, batch, stream);
    }
    return hipErrorInvalidValue;
}

// batch <= 8, K % 256 == 0 (the dispatcher checks)
hipError_t launch_matrix_tile(const GemvArgs &a, hipStream_t stream)
{
    switch (a.b) {
    case 3: return launch_tile_b<3>(a, stream);
    case 4: return launch_tile_b<4>(a, stream);
    case 5: return launch_tile_b<5>(a, stream);
    case 6: return launch_tile_b<6>(a, stream);
    case 7: return launch_tile_b<7>(a, stream);
    case 8: return launch_tile_b<8>(a, stream);
    }
    return hipErrorInvalidValue;
}

} // namespace apgemv
