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
#include "device_common.h"
#include "launchers.h"

namespace apgemv {

// Waves per group of 4 rows at batch 1 and 2 for a row of `nspans` spans of 2048 columns: one per span up to 4 spans
// and 8 from 9 spans on, but rows of 5 to 8 spans take half as many waves, two spans each.  Measured, us per
// single call, one wave per span -> half: 4096 x 11008 (6 spans) b = 3 7.2 -> 6.9, b = 5 10.7 -> 9.3, b = 6
// 11.8 -> 10.1, b = 7 12.0 -> 11.2, level at b = 4 and 8; 5120 x 13824 (7 spans) b = 5 14.8 -> 12.4, b = 6
// 16.2 -> 14.0, b = 7 18.0 -> 16.1, b = 8 19.9 -> 18.4, level at b = 3, 4; the headline list of 18 products
// gains 10 % (same box, alternating runs).  The last wave of such a row is mostly empty, and set-up, barrier
// and reduction are shared by fewer waves.  Not so on shorter rows (4 spans as 2 waves: level on 8192 x 8192 and
// 28672 x 8192, 30 % slower on 1024 x 8192; 3 spans as 2 waves: 15 % slower) nor on 14 spans (7, 5 or 4 waves:
// level).  Single calls and work lists use the same rule, so their outputs stay bit-identical.
static inline int batch1_waves(int nspans)
{
    if (nspans >= 5 && nspans <= 8) return (nspans + 1) / 2;
    return nspans < 8 ? nspans : 8;
}

// One workgroup per group of 4 rows; its waves stride over the row's spans of 2048 columns.
// The table loads go out first, then the wave's first slice loads, then the tables are written to
// LDS while the slice loads are still in flight; later
// spans are loaded after the previous one is consumed (other waves of the CU cover the latency;
// a second register set for prefetching cost more in occupancy than it gained).
template <int B, int NB, int MAXT>
__device__ __forceinline__ void gemv_group(const uint8_t *__restrict__ slices, size_t slice_bytes,
                                           const uint16_t *__restrict__ lut, const uint16_t *__restrict__ x,
                                           uint16_t *__restrict__ y, int M, int K, int batch, int g, int nwaves)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    __shared__ __attribute__((aligned(16))) uint8_t tab[kRowsPerGroup * TB + 16]; // + dummy area
    __shared__ __attribute__((aligned(16))) uint16_t nat[kRowsPerGroup * 8];
    __shared__ float red[MAXT / 64][NB][4][kRowsPerGroup]; // [wave][batch row][DPP row][lane & 3]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform, kept in an SGPR
    const int row0 = g * kRowsPerGroup;
    const int chunks = K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;

    u32x4 Q[B];
    u32x4 X[NB][4];
    // Loads of the lane's slice words and activations for one span (Section 5.2 step 1), as buffer
    // loads: wave-uniform base and offset in scalar registers, one per-lane byte offset for all of
    // them, so that no vector operation is spent on addresses.  The slice descriptor starts at this
    // group's first unit of slice 0; slice s is s * slice_bytes further (below 4 GiB: the packed
    // format limits a matrix to 2^32 weights).
    const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(slices + (size_t)g * chunks * 16), 0, 0xffffffffu, kBufferRsrcWord3);
    // A ragged last span of at most 32 chunks runs on both halves of the wave at b = 4, 5, 6 (compute_unit_half):
    // lane l then takes chunk l % 32.
    auto halved = [&](int span) { return half_unit_ok<B>() && chunks - span * kSpanLanes <= 32; };
    auto issue_loads = [&](int span) {
        const int rem = chunks - span * kSpanLanes;
        const int nl = rem < kSpanLanes ? rem : kSpanLanes;
        // Lanes past the end of a ragged last span load what the last valid lane loads (and are
        // masked out of the compute): no branch around the loads.
        const int cl = halved(span) ? (lane & 31) : lane;
        const uint32_t loff = (uint32_t)(cl < nl ? cl : nl - 1) * 16u;
        const uint32_t sspan = (uint32_t)span * (kSpanLanes * 16u);
#pragma unroll
        for (int s = 0; s < B; ++s)
            Q[s] = __builtin_amdgcn_raw_buffer_load_b128(srsrc, loff, sspan + (uint32_t)s * (uint32_t)slice_bytes, kBufferNonTemporal);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int xr = nb < batch ? nb : batch - 1;
            const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint16_t *>(x + (size_t)xr * K + (size_t)span * kSpanCols), 0, 0xffffffffu, kBufferRsrcWord3);
#pragma unroll
            for (int t = 0; t < 4; ++t)
                X[nb][t] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, loff, (uint32_t)(t * 16 * nl), 0);
        }
    };
    auto active = [&](int span) { return (halved(span) ? (lane & 31) : lane) < chunks - span * kSpanLanes; };

    float acc[NB][kRowsPerGroup];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < kRowsPerGroup; ++r) acc[nb][r] = 0.f;

    int span = wave; // the launcher guarantees nwaves <= nspans
    StagedTable<B> st;
    // A wave issues all its requests in one burst at raised priority: the memory pipeline serves a
    // compute unit's requests in order, so waves whose bursts do not interleave receive their data
    // one after the other and start computing while the later ones are still being served, instead
    // of all finishing their last slice at the end of the stream together.
    __builtin_amdgcn_s_setprio(3);
    stage_tables_load<B>(st, lut, row0, M, nwaves * 64);
    issue_loads(span);
    __builtin_amdgcn_s_setprio(0);
    stage_tables_store<B>(st, tab, nat, nwaves * 64); // waits for the table loads only
    __syncthreads();
    while (true) {
        if constexpr (half_unit_ok<B>()) {
            if (halved(span)) {
                if (active(span)) compute_unit_half<B, NB>(Q, X, tab, acc, lane >= 32);
            } else if (active(span)) compute_unit<B, NB>(Q, X, tab, acc);
        } else if (active(span)) compute_unit<B, NB>(Q, X, tab, acc);
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

// Two consecutive groups of 4 rows per workgroup, batch 1, one wave per span: every wave requests the
// slice words of both groups up front (twice the bytes in flight per wave slot: at 3 to 5 bits one
// group per wave leaves HBM waiting at full occupancy), loads its activations once for both, and the
// table staging and the two barriers are shared.  Per row the arithmetic and its order are those of
// gemv_group, so the outputs are bit-identical.  `gp` = index of the pair; with an odd number of
// groups the last workgroup computes the last group twice and stores it once.
template <int B, int MAXT>
__device__ __forceinline__ void gemv_group_pair(const uint8_t *__restrict__ slices, size_t slice_bytes,
                                                const uint16_t *__restrict__ lut, const uint16_t *__restrict__ x,
                                                uint16_t *__restrict__ y, int M, int K, int gp, int nwaves)
{
    using T = Table<B>;
    constexpr int TB = T::kRowBytes;
    constexpr int R = 2;
    __shared__ __attribute__((aligned(16))) uint8_t tab[R][kRowsPerGroup * TB + 16]; // + dummy area
    __shared__ __attribute__((aligned(16))) uint16_t nat[R][kRowsPerGroup * 8];
    __shared__ float red[MAXT / 64][R][4][kRowsPerGroup]; // [wave][group][DPP row][lane & 3]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int groups = (M + kRowsPerGroup - 1) / kRowsPerGroup;
    const int g0 = gp * R;
    const bool both = g0 + 1 < groups;
    const int gofs = both ? 1 : 0; // second group of the pair, as an offset from the first
    const int chunks = K / kChunkSlots;
    const int span = wave; // the launcher gives every span its own wave
    const int rem = chunks - span * kSpanLanes;
    const int nl = rem < kSpanLanes ? rem : kSpanLanes;
    const bool active = lane < nl;
    const uint32_t loff = (uint32_t)(active ? lane : nl - 1) * 16u;

    const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(slices + (size_t)g0 * chunks * 16), 0, 0xffffffffu, kBufferRsrcWord3);
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(x + (size_t)span * kSpanCols), 0, 0xffffffffu, kBufferRsrcWord3);
    StagedTable<B> st[R];
    u32x4 Q[R][B];
    u32x4 X[1][4];
    __builtin_amdgcn_s_setprio(3); // one uninterrupted burst of requests per wave (see gemv_group)
#pragma unroll
    for (int rg = 0; rg < R; ++rg) stage_tables_load<B>(st[rg], lut, (g0 + rg * gofs) * kRowsPerGroup, M, nwaves * 64);
#pragma unroll
    for (int rg = 0; rg < R; ++rg) {
        const uint32_t sunit = (uint32_t)(rg * gofs) * (uint32_t)chunks * 16u + (uint32_t)span * (kSpanLanes * 16u);
#pragma unroll
        for (int s = 0; s < B; ++s)
            Q[rg][s] = __builtin_amdgcn_raw_buffer_load_b128(srsrc, loff, sunit + (uint32_t)s * (uint32_t)slice_bytes, kBufferNonTemporal);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) X[0][t] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, loff, (uint32_t)(t * 16 * nl), 0);
    __builtin_amdgcn_s_setprio(0);
#pragma unroll
    for (int rg = 0; rg < R; ++rg) stage_tables_store<B>(st[rg], tab[rg], nat[rg], nwaves * 64);
    __syncthreads();
#pragma unroll
    for (int rg = 0; rg < R; ++rg) {
        float acc[1][kRowsPerGroup] = {{0.f, 0.f, 0.f, 0.f}};
        if (active) compute_unit<B, 1>(Q[rg], X, tab[rg], acc);
        const float c = reduce4_in_dpp_rows(acc[0], lane);
        if ((lane & 15) >= 12) red[wave][rg][lane >> 4][lane & 3] = c;
    }
    __syncthreads();
    if (threadIdx.x < R * kRowsPerGroup) {
        const int rg = threadIdx.x / kRowsPerGroup, r = threadIdx.x % kRowsPerGroup;
        const int cls = ((r & 1) << 1) | (r >> 1); // lane & 3 that holds row r
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w)
            for (int d = 0; d < 4; ++d) s += red[w][rg][d][cls];
        const int row = (g0 + rg) * kRowsPerGroup + r;
        if ((rg == 0 || both) && row < M) {
            const __half h = __float2half_rn(s);
            y[row] = __builtin_bit_cast(uint16_t, h);
        }
    }
}

template <int B, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(2, B <= 4 ? 8 : 6))) void gemv_pair_kernel(
    const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
    const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int M, int K)
{
    gemv_group_pair<B, MAXT>(slices, slice_bytes, lut, x, y, M, K, blockIdx.x, blockDim.x >> 6);
}

template <int B, int NB, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(2, (B <= 4 && NB == 1) ? 8 : 6))) void gemv_kernel(
    const uint8_t *__restrict__ slices, size_t slice_bytes, const uint16_t *__restrict__ lut,
    const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int M, int K, int batch)
{
    gemv_group<B, NB, MAXT>(slices, slice_bytes, lut, x, y, M, K, batch, blockIdx.x, blockDim.x >> 6);
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
                            (int)blockIdx.x - a.group_begin[m], blockDim.x >> 6);
}

// A list of batch-1 products in one launch: matrices of any shapes, each with its own bit-width (the
// projections of a decoder layer, possibly at per-layer mixed precision; Section 6.3 measures whole-model
// decoding, where a launch per matrix costs more than the small matrices' own traffic).  Workgroup ->
// (item, group of 4 rows) through the prefix sums of the group counts; the workgroup has as many waves
// as the longest row of the list needs (at most 8), and waves beyond an item's span count retire before
// the first barrier (a barrier counts the surviving waves only).  The work per group is that of
// gemv_kernel with the same number of waves, so every output is bit-identical to a separate call.
// B = the bit-width of every item, or 0 for a list of mixed bit-widths (one kernel then holds all six
// code paths and the registers of the widest; lists of one bit-width get that bit-width's own kernel).
template <int B, int NB, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(2, ((B == 3 || B == 4) && NB == 1) ? 8 : 6))) void gemv_list_kernel(ListArgs a)
{
    int it = 0;
#pragma unroll
    for (int i = 1; i < kMaxListItems; ++i)
        if (i < a.count && (int)blockIdx.x >= a.group_begin[i]) it = i;
    const ListItem &I = a.item[it];
    const int K = I.K;
    const int nspans = (K / kChunkSlots + kSpanLanes - 1) / kSpanLanes;
    const int launched = blockDim.x >> 6;
    const int nwaves = nspans < launched ? nspans : launched;
    if ((int)(threadIdx.x >> 6) >= nwaves) return;
    const int g = (int)blockIdx.x - a.group_begin[it];
    if constexpr (B != 0) {
        gemv_group<B, NB, MAXT>(I.slices, I.slice_bytes, I.lut, I.x, I.y, I.M, K, NB, g, nwaves);
    } else {
        switch (I.b) {
        case 3: gemv_group<3, NB, MAXT>(I.slices, I.slice_bytes, I.lut, I.x, I.y, I.M, K, NB, g, nwaves); break;
        case 4: gemv_group<4, NB, MAXT>(I.slices, I.slice_bytes, I.lut, I.x, I.y, I.M, K, NB, g, nwaves); break;
        case 5: gemv_group<5, NB, MAXT>(I.slices, I.slice_bytes, I.lut, I.x, I.y, I.M, K, NB, g, nwaves); break;
        case 6: gemv_group<6, NB, MAXT>(I.slices, I.slice_bytes, I.lut, I.x, I.y, I.M, K, NB, g, nwaves); break;
        case 7: gemv_group<7, NB, MAXT>(I.slices, I.slice_bytes, I.lut, I.x, I.y, I.M, K, NB, g, nwaves); break;
        default: gemv_group<8, NB, MAXT>(I.slices, I.slice_bytes, I.lut, I.x, I.y, I.M, K, NB, g, nwaves); break;
        }
    }
}

// One launch for the items of `a` whose rows need `nw` waves.
template <int NB> static hipError_t launch_list_class(const ListArgs &a, int nw, hipStream_t stream)
{
    constexpr int kMaxWaves = 8;
    constexpr int T = 64 * kMaxWaves;
    ListArgs sub;
    sub.count = 0;
    int total = 0, b = -1, max_nw = 1;
    for (int i = 0; i < a.count; ++i) {
        const int spans = (a.item[i].K / kChunkSlots + kSpanLanes - 1) / kSpanLanes;
        const int w = batch1_waves(spans);
        if (w != nw) continue;
        sub.item[sub.count] = a.item[i];
        sub.group_begin[sub.count] = total;
        ++sub.count;
        total += padded_rows(a.item[i].M) / kRowsPerGroup;
        if (w > max_nw) max_nw = w;
        b = b < 0 || b == a.item[i].b ? a.item[i].b : 0;
    }
    if (sub.count == 0) return hipSuccess;
    for (int i = sub.count; i < kMaxListItems; ++i) sub.group_begin[i] = 0x7fffffff;
    const dim3 grid(total), block(64 * max_nw);
    switch (b) {
    case 3: hipLaunchKernelGGL((gemv_list_kernel<3, NB, T>), grid, block, 0, stream, sub); break;
    case 4: hipLaunchKernelGGL((gemv_list_kernel<4, NB, T>), grid, block, 0, stream, sub); break;
    case 5: hipLaunchKernelGGL((gemv_list_kernel<5, NB, T>), grid, block, 0, stream, sub); break;
    case 6: hipLaunchKernelGGL((gemv_list_kernel<6, NB, T>), grid, block, 0, stream, sub); break;
    case 7: hipLaunchKernelGGL((gemv_list_kernel<7, NB, T>), grid, block, 0, stream, sub); break;
    case 8: hipLaunchKernelGGL((gemv_list_kernel<8, NB, T>), grid, block, 0, stream, sub); break;
    default: hipLaunchKernelGGL((gemv_list_kernel<0, NB, T>), grid, block, 0, stream, sub); break;
    }
    return hipGetLastError();
}

// The caller has checked every item (3 <= b <= 8; every item at batch `batch`, 1 or 2).  Items are launched
// together per number of waves their rows take (batch1_waves): a workgroup sized for the longest row would hold
// wave slots for short rows that retire at once.
hipError_t launch_gemv_list(ListArgs &a, int batch, hipStream_t stream)
{
    if (batch != 1 && batch != 2) return hipErrorInvalidValue;
    bool seen[9] = {};
    for (int i = 0; i < a.count; ++i) {
        const int spans = (a.item[i].K / kChunkSlots + kSpanLanes - 1) / kSpanLanes;
        const int w = batch1_waves(spans);
        if (seen[w]) continue;
        seen[w] = true;
        const hipError_t e = batch == 1 ? launch_list_class<1>(a, w, stream) : launch_list_class<2>(a, w, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
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
            *reinterpret_cast<uint32_t *>(tab + r * TB + i6 * 4) = pair_entry(nat + r * 8, i6);
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
    if (NB <= 2 && a.waves_per_group == 0) nw = batch1_waves(nspans); // batch 2 gains the same (5 to 14 %)
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
    // Two row groups per workgroup at batch 1: on request only.  On 28672x8192 it measured within the
    // run-to-run spread of the kernel with one group per workgroup (+-5 % either way, by bit-width), and
    // smaller matrices need every workgroup they can get (11008x4096: 10 to 30 % slower).
    if constexpr (NB == 1) {
        if (nw == nspans && nspans >= 2 && a.waves_per_group == 0 && a.row_groups_per_wg < 0 && a.variant == 7) {
            hipLaunchKernelGGL((gemv_pair_kernel<B, kMaxThreads>), dim3((groups + 1) / 2), dim3(64 * nw), 0, stream,
                               a.slices, a.slice_bytes, a.lut, a.x, a.y, a.M, a.K);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((gemv_kernel<B, NB, kMaxThreads>), dim3(groups), dim3(64 * nw), 0, stream,
                       a.slices, a.slice_bytes, a.lut, a.x, a.y, a.M, a.K, a.batch);
    return hipGetLastError();
}

// The ALU kernels for one call: template instance by bit-width and by batch rounded up to 1, 2, 4, 8.
template <int B> static hipError_t launch_alu_b(const GemvArgs &a, hipStream_t stream)
{
    if (a.batch == 1) return launch_one<B, 1>(a, stream);
    if (a.batch == 2) return launch_one<B, 2>(a, stream);
    if (a.batch <= 4) return launch_one<B, 4>(a, stream);
    return launch_one<B, 8>(a, stream);
}
hipError_t launch_alu(const GemvArgs &a, hipStream_t stream)
{
    switch (a.b) {
    case 3: return launch_alu_b<3>(a, stream);
    case 4: return launch_alu_b<4>(a, stream);
    case 5: return launch_alu_b<5>(a, stream);
    case 6: return launch_alu_b<6>(a, stream);
    case 7: return launch_alu_b<7>(a, stream);
    case 8: return launch_alu_b<8>(a, stream);
    }
    return hipErrorInvalidValue;
}

template <int B, int NB> static hipError_t launch_multi_one(const MultiArgs &a, int total_groups, hipStream_t stream)
{
    constexpr int kMaxWaves = NB <= 4 ? 8 : 4;
    const int chunks = a.K / kChunkSlots;
    const int nspans = (chunks + kSpanLanes - 1) / kSpanLanes;
    const int nw = NB <= 2 ? batch1_waves(nspans) : nspans < kMaxWaves ? nspans : kMaxWaves; // as single calls do
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

} // namespace apgemv
