// Small-batch kernels on the matrix cores (v_mfma_f32_4x4x4_16B_f16) for gfx950 and their launchers.
#include "device_common.h"
#include "launchers.h"

namespace apgemv {

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

#define APGEMV_SWITCH_B(FN)                                                            \
    switch (a.b) {                                                                     \
    case 3: return a.batch <= 4 ? FN<3, 1>(a, stream) : FN<3, 2>(a, stream);           \
    case 4: return a.batch <= 4 ? FN<4, 1>(a, stream) : FN<4, 2>(a, stream);           \
    case 5: return a.batch <= 4 ? FN<5, 1>(a, stream) : FN<5, 2>(a, stream);           \
    case 6: return a.batch <= 4 ? FN<6, 1>(a, stream) : FN<6, 2>(a, stream);           \
    case 7: return a.batch <= 4 ? FN<7, 1>(a, stream) : FN<7, 2>(a, stream);           \
    case 8: return a.batch <= 4 ? FN<8, 1>(a, stream) : FN<8, 2>(a, stream);           \
    }                                                                                  \
    return hipErrorInvalidValue
hipError_t launch_matrix_row_per_lane(const GemvArgs &a, hipStream_t stream) { APGEMV_SWITCH_B(launch_mfma); }
hipError_t launch_matrix_exchange(const GemvArgs &a, hipStream_t stream) { APGEMV_SWITCH_B(launch_xmfma); }
#undef APGEMV_SWITCH_B

} // namespace apgemv
