// Large-batch path for callers that cannot allocate device memory: ap_gemm with its dense-weight
// workspace in a static device array and the dense product in a kernel of this library.
//
// ap_gemm takes the workspace from the caller and hands the product to rocBLAS, whose first use
// allocates.  Code under HIP graph capture, tight serving loops and harnesses that forbid
// hipMalloc need an entry point that allocates nothing at all: the dequantised weights go to
// `scratch` below (one copy per GPU, held until the process ends) and the product is computed by
// dense_gemm_kernel (v_mfma_f32_16x16x16_f16, binary32 accumulation).
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/apgemv.h"
#include "handle.h"
#include "kernels.h"

namespace apgemv {

// Dense binary16 weights of one matrix.  In host code this name is only a stand-in for the device
// symbol: the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) uint8_t scratch[AP_GEMM_STATIC_MAX_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices]; // device address of `scratch` on each device, 0 = not asked yet

// Address of this device's copy of `scratch` (each GPU holds its own copy at its own address).
void *scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// y[t][i] = sum_k w[i][k] * x[t][k]: one wave per tile of 16 output rows x 16 batch rows.  In
// v_mfma_f32_16x16x16_f16 lane l supplies A[l % 16][4 (l / 16) .. + 3] and B[4 (l / 16) .. + 3][l % 16]
// and receives D[4 (l / 16) .. + 3][l % 16].  Which four k a lane group contributes is free as long
// as A and B agree, so group g takes the 8 consecutive k of a 16-byte load in two instructions.
// K % 32 == 0 (guaranteed by the packed format).
__global__ __launch_bounds__(256) void dense_gemm_kernel(const uint16_t *__restrict__ w, const uint16_t *__restrict__ x,
                                                         uint16_t *__restrict__ y, int M, int K, int batch, int row_tiles,
                                                         int tiles)
{
    const int tile = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (tile >= tiles) return; // whole waves
    const int rt = tile % row_tiles, bt = tile / row_tiles;
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    const int row = rt * 16 + r, t = bt * 16 + r;
    const u32x4 *wp = reinterpret_cast<const u32x4 *>(w + (size_t)(row < M ? row : M - 1) * K) + g;
    const u32x4 *xp = reinterpret_cast<const u32x4 *>(x + (size_t)(t < batch ? t : batch - 1) * K) + g;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < K / 8; k += 4) {
        const u32x4 a = wp[k], b = xp[k];
        const u32x2 a0 = {a[0], a[1]}, a1 = {a[2], a[3]}, b0 = {b[0], b[1]}, b1 = {b[2], b[3]};
        acc = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a0), __builtin_bit_cast(f16x4, b0), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a1), __builtin_bit_cast(f16x4, b1), acc, 0, 0, 0);
    }
    if (t < batch) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int orow = rt * 16 + 4 * g + j;
            if (orow < M) {
                const _Float16 h = (_Float16)acc[j];
                y[(size_t)t * M + orow] = __builtin_bit_cast(uint16_t, h);
            }
        }
    }
}

} // namespace

bool static_scratch_setup() { return scratch_on_current_device() != nullptr; }

} // namespace apgemv

using namespace apgemv;

extern "C" ap_status ap_gemm_static(const ap_matrix *h, int b, const void *x_dev, void *y_dev, int batch,
                                    void *stream)
{
    if (!handle_ok(h) || !x_dev || !y_dev) return AP_ERR_INVALID_ARG;
    if (b < AP_MIN_BITS || b > h->hdr.n || !(h->hdr.lut_mask & (1u << b))) return AP_ERR_BITS;
    if (batch < 1 || batch > (1 << 20)) return AP_ERR_BATCH;
    if (reinterpret_cast<uintptr_t>(x_dev) % 16 || reinterpret_cast<uintptr_t>(y_dev) % 2) return AP_ERR_INVALID_ARG;
    const size_t need = (size_t)h->hdr.M * (size_t)h->hdr.K * 2;
    if (need > (size_t)AP_GEMM_STATIC_MAX_BYTES) return AP_ERR_BUFFER_TOO_SMALL;
    void *work = scratch_on_current_device();
    if (!work) return AP_ERR_HIP;

    GemvArgs a;
    a.slices = h->dev + h->hdr.slice_off;
    a.slice_bytes = h->hdr.slice_bytes;
    a.lut = reinterpret_cast<const uint16_t *>(h->dev + h->hdr.lut_off[b]);
    a.x = nullptr;
    a.y = static_cast<uint16_t *>(work);
    a.M = h->hdr.M;
    a.K = h->hdr.K;
    a.b = b;
    a.batch = 1;
    a.waves_per_group = 0;
    a.row_groups_per_wg = -1;
    a.mfma_min_batch = 0;
    a.variant = 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // every element of the M x K dense matrix is rewritten before it is read: nothing to clear
    if (launch_dequantize(a, st) != hipSuccess) return AP_ERR_HIP;
    const int row_tiles = (a.M + 15) / 16, batch_tiles = (batch + 15) / 16;
    const long long tiles = (long long)row_tiles * batch_tiles;
    if (tiles > 0x7fffffffLL / 64) return AP_ERR_BATCH;
    const unsigned blocks = (unsigned)((tiles + 3) / 4);
    hipLaunchKernelGGL(dense_gemm_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const uint16_t *>(work),
                       static_cast<const uint16_t *>(x_dev), static_cast<uint16_t *>(y_dev), a.M, a.K, batch, row_tiles,
                       (int)tiles);
    return hipGetLastError() == hipSuccess ? AP_OK : AP_ERR_HIP;
}
