// Batch-1 GEMV for the two widest bit-widths (b = 7, 8) with conflict-free table lookups.
//
// With 128 or 256 entries a row's table covers every LDS bank several times, so a wave whose 64
// lanes look into ONE table (gemv_kernel) loses half to two thirds of its lookup rate to bank
// conflicts.  Here every lane owns one LDS bank: the steps are those of Section 5.2 (load slices
// and activations, form indices, fetch centroids, multiply-accumulate, reduce), but
//   * a lane owns ONE row of the group and 4 chunks of 32 weights of the span (4 dword loads per
//     slice); the 4 lanes of a quad own the 4 rows of the same 128 columns;
//   * the group's tables are staged as 8 copies per row: entry p of bank column k (row k & 3) is
//     the low half of the dword at p * 128 + k * 4, and lane l only ever reads column l & 31, so
//     the 32 lanes the LDS serves per clock hit 32 different banks whatever their indices;
//   * a quad's activations are loaded once (lane m of the quad holds those of chunk m) and reach
//     the other three lanes through the DPP operand of v_dot2c_f32_f16: a 16-bit lookup returns
//     (centroid, 0), so one packed dot product against (x_even, x_odd) or its half-swapped copy
//     multiplies one weight, and no instruction is spent on moving activations between lanes.
#include "device_common.h"
#include "launchers.h"

namespace apgemv {

template <int B> struct QuadTable {
    static_assert(B == 7 || B == 8, "the bank-per-lane kernel serves b = 7 and 8");
    static constexpr int kEntries = 1 << B;
    static constexpr int kBytes = kEntries * 128; // one dword per entry and bank column
    static constexpr int kPieces = kEntries / 8;  // 16-byte pieces of a stored table row
};

// LDS byte offset (without the lane's column) of the entry selected by byte J of a merged word.
template <int B, int J> __device__ __forceinline__ uint32_t quad_entry_offset(uint32_t v, uint32_t seven)
{
    if constexpr (B == 8) return byte_shl1<J>(v, seven);  // byte << 7: all eight bits are index bits
    else return byte_and<J>(v, 0xFEu) << 6;               // bit 0 belongs to the absent eighth slice
}

// acc += x_lo * w_lo + x_hi * w_hi with x taken from lane SRC of the quad.
template <int SRC> __device__ __forceinline__ void mac8(float &acc0, float &acc1, const u32x4 &xe, const u32x4 &xo,
                                                        const uint32_t (&we)[4], const uint32_t (&wo)[4])
{
#define APGEMV_MAC8(P)                                                                                      \
    asm volatile("s_nop 1\n\t"                                                                              \
                 "v_dot2c_f32_f16_dpp %0, %2, %10 quad_perm:" P " row_mask:0xf bank_mask:0xf\n\t"           \
                 "v_dot2c_f32_f16_dpp %1, %6, %14 quad_perm:" P " row_mask:0xf bank_mask:0xf\n\t"           \
                 "v_dot2c_f32_f16_dpp %0, %3, %11 quad_perm:" P " row_mask:0xf bank_mask:0xf\n\t"           \
                 "v_dot2c_f32_f16_dpp %1, %7, %15 quad_perm:" P " row_mask:0xf bank_mask:0xf\n\t"           \
                 "v_dot2c_f32_f16_dpp %0, %4, %12 quad_perm:" P " row_mask:0xf bank_mask:0xf\n\t"           \
                 "v_dot2c_f32_f16_dpp %1, %8, %16 quad_perm:" P " row_mask:0xf bank_mask:0xf\n\t"           \
                 "v_dot2c_f32_f16_dpp %0, %5, %13 quad_perm:" P " row_mask:0xf bank_mask:0xf\n\t"           \
                 "v_dot2c_f32_f16_dpp %1, %9, %17 quad_perm:" P " row_mask:0xf bank_mask:0xf"               \
                 : "+v"(acc0), "+v"(acc1)                                                                   \
                 : "v"(xe[0]), "v"(xe[1]), "v"(xe[2]), "v"(xe[3]), "v"(xo[0]), "v"(xo[1]), "v"(xo[2]), "v"(xo[3]), \
                   "v"(we[0]), "v"(we[1]), "v"(we[2]), "v"(we[3]), "v"(wo[0]), "v"(wo[1]), "v"(wo[2]), "v"(wo[3]))
    if constexpr (SRC == 0) APGEMV_MAC8("[0,0,0,0]");
    else if constexpr (SRC == 1) APGEMV_MAC8("[1,1,1,1]");
    else if constexpr (SRC == 2) APGEMV_MAC8("[2,2,2,2]");
    else APGEMV_MAC8("[3,3,3,3]");
#undef APGEMV_MAC8
}

// One workgroup per group of 4 rows; its waves stride over the row's spans of 2048 columns.
// R = 16-byte table pieces each thread stages (the launcher picks it from the wave count).
template <int B, int R, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(2, 4))) void gemv_quad_kernel(
    const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
    const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int M, int K)
{
    using T = QuadTable<B>;
    __shared__ __attribute__((aligned(16))) uint8_t tab[T::kBytes];
    __shared__ float red[MAXT / 64][4][kRowsPerGroup]; // [wave][DPP row][row of the group]

    const int tid = threadIdx.x, nth = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = nth >> 6;
    const int q = lane & 3;  // row of the group
    const int c = lane >> 2; // quad: chunks c, c + 16, c + 32, c + 48 of a span
    const int g = blockIdx.x;
    const int row0 = g * kRowsPerGroup;
    const int chunks = K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;

    // ---- table pieces first (vector-memory loads return in order): thread -> bank column tid & 31,
    //      pieces (tid >> 5) + i * (nth >> 5); indices past the end repeat the last piece (the copy
    //      is then written twice with the same bytes)
    const int col = tid & 31;
    const int last_row = M - 1 - row0;
    const int trow = (col & 3) < last_row ? (col & 3) : last_row;
    const u32x4 *tsrc = reinterpret_cast<const u32x4 *>(lut + ((size_t)(row0 + trow) << B));
    u32x4 st[R];
    int piece[R];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int p = (tid >> 5) + i * (nth >> 5);
        piece[i] = p < T::kPieces ? p : T::kPieces - 1;
        st[i] = tsrc[piece[i]];
    }

    uint32_t Q[B][4];
    u32x4 XE[4];
    int nl = 0;
    auto issue_loads = [&](int span) {
        const int rem = chunks - span * kSpanLanes;
        nl = rem < kSpanLanes ? rem : kSpanLanes;
        const uint8_t *sbase = slices + ((size_t)g * chunks + (size_t)span * kSpanLanes) * 16;
        uint32_t voff[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int ch = c + 16 * m;
            voff[m] = (uint32_t)(ch < nl ? ch : nl - 1) * 16u + (uint32_t)q * 4u;
        }
#pragma unroll
        for (int s = 0; s < B; ++s)
#pragma unroll
            for (int m = 0; m < 4; ++m)
                Q[s][m] = __builtin_nontemporal_load(
                    reinterpret_cast<const uint32_t *>(sbase + (size_t)s * slice_bytes + voff[m]));
        // lane q of a quad holds the activations of chunk c + 16 q
        const int xch = c + 16 * q;
        const uint32_t xoff = (uint32_t)(xch < nl ? xch : nl - 1) * 16u;
        const uint8_t *xbase = reinterpret_cast<const uint8_t *>(x + (size_t)span * kSpanCols);
#pragma unroll
        for (int t = 0; t < 4; ++t)
            XE[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)(t * 16 * nl) + xoff);
    };

    int span = wave; // the launcher guarantees nwaves <= nspans
    issue_loads(span);

    // ---- tables into LDS while the slice loads are in flight
#pragma unroll
    for (int i = 0; i < R; ++i) {
        uint8_t *dst = tab + piece[i] * (8 * 128) + col * 4;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            *reinterpret_cast<uint16_t *>(dst + k * 128) = (uint16_t)(st[i][k >> 1] >> ((k & 1) * 16));
    }
    __syncthreads();

    float acc0 = 0.f, acc1 = 0.f;
    uint32_t seven = 7;
    asm("" : "+v"(seven));
    const uint32_t colbase = (uint32_t)col * 4u;
    while (true) {
        // half-swapped copy of the activations for the odd columns
        u32x4 XO[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) XO[t][j] = __builtin_amdgcn_alignbit(XE[t][j], XE[t][j], 16);
        auto chunk = [&](auto mtag) {
            constexpr int m = decltype(mtag)::value;
            if (c + 16 * m < nl) {
                uint32_t qw[B];
#pragma unroll
                for (int s = 0; s < B; ++s) qw[s] = Q[s][m];
                uint32_t W[8];
                merge_words<B>(qw, W);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t ve = W[2 * t], vo = W[2 * t + 1];
                    const uint32_t ae[4] = {quad_entry_offset<B, 0>(ve, seven) | colbase, quad_entry_offset<B, 1>(ve, seven) | colbase,
                                            quad_entry_offset<B, 2>(ve, seven) | colbase, quad_entry_offset<B, 3>(ve, seven) | colbase};
                    const uint32_t ao[4] = {quad_entry_offset<B, 0>(vo, seven) | colbase, quad_entry_offset<B, 1>(vo, seven) | colbase,
                                            quad_entry_offset<B, 2>(vo, seven) | colbase, quad_entry_offset<B, 3>(vo, seven) | colbase};
                    uint32_t we[4], wo[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        we[j] = *reinterpret_cast<const uint16_t *>(tab + ae[j]);
                        wo[j] = *reinterpret_cast<const uint16_t *>(tab + ao[j]);
                    }
                    mac8<m>(acc0, acc1, XE[t], XO[t], we, wo);
                }
            }
        };
        chunk(std::integral_constant<int, 0>{});
        chunk(std::integral_constant<int, 1>{});
        chunk(std::integral_constant<int, 2>{});
        chunk(std::integral_constant<int, 3>{});
        span += nwaves;
        if (span >= nspans) break;
        issue_loads(span);
    }

    // ---- reduce: the 16 quads of a wave (two row shifts inside each DPP row of 16 lanes leave the
    //      sums of rows 0..3 in lanes 12..15), then the DPP rows and waves in fixed order
    asm volatile("s_nop 3" : "+v"(acc0), "+v"(acc1)); // a packed-dot result needs 3 wait states before another ALU op reads it
    float a = acc0 + acc1;
    a += dpp_get<0x114>(a); // row_shr:4 (0 shifted in)
    a += dpp_get<0x118>(a); // row_shr:8
    if ((lane & 15) >= 12) red[wave][lane >> 4][lane & 3] = a;
    __syncthreads();
    if (tid < kRowsPerGroup) {
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w)
            for (int d = 0; d < 4; ++d) s += red[w][d][tid];
        const int row = row0 + tid;
        if (row < M) {
            const __half h = __float2half_rn(s);
            y[row] = __builtin_bit_cast(uint16_t, h);
        }
    }
}

template <int B, int R> static hipError_t launch_quad_r(const GemvArgs &a, int groups, int nw, hipStream_t stream)
{
    hipLaunchKernelGGL((gemv_quad_kernel<B, R, 512>), dim3(groups), dim3(64 * nw), 0, stream, a.slices,
                       a.slice_bytes, a.lut, a.x, a.y, a.M, a.K);
    return hipGetLastError();
}

template <int B> static hipError_t launch_quad_b(const GemvArgs &a, hipStream_t stream)
{
    constexpr int kMaxWaves = 8;
    const int groups = padded_rows(a.M) / kRowsPerGroup;
    const int chunks = a.K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;
    int nw = kMaxWaves;
    if (a.waves_per_group > 0 && a.waves_per_group < nw) nw = a.waves_per_group;
    if (nw > nspans) nw = nspans;
    // pieces per thread: all kPieces * 32 copies of a 16-byte piece over 64 * nw threads
    const int need = (QuadTable<B>::kPieces + 2 * nw - 1) / (2 * nw);
    if (need <= 1) return launch_quad_r<B, 1>(a, groups, nw, stream);
    if (need <= 2) return launch_quad_r<B, 2>(a, groups, nw, stream);
    if (need <= 4) return launch_quad_r<B, 4>(a, groups, nw, stream);
    if (need <= 8) return launch_quad_r<B, 8>(a, groups, nw, stream);
    return launch_quad_r<B, 16>(a, groups, nw, stream);
}

// batch 1, b = 7 or 8 (the dispatcher checks)
hipError_t launch_quad(const GemvArgs &a, hipStream_t stream)
{
    if (a.batch != 1) return hipErrorInvalidValue;
    if (a.b == 7) return launch_quad_b<7>(a, stream);
    if (a.b == 8) return launch_quad_b<8>(a, stream);
    return hipErrorInvalidValue;
}

} // namespace apgemv
