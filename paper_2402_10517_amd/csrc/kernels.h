// Internal interface between the C-ABI entry points and the HIP kernels.
#ifndef APGEMV_KERNELS_H
#define APGEMV_KERNELS_H

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace apgemv {

struct GemvArgs {
    const uint8_t *slices; // device: slice 0 of the packed matrix
    size_t slice_bytes;
    const uint16_t *lut;   // device: table of bit-width b, M * 2^b binary16
    const uint16_t *x;     // device: batch * K binary16
    uint16_t *y;           // device: batch * M binary16
    int M, K, b, batch;
    int waves_per_group;   // 0 = choose from the shape
    int row_groups_per_wg; // -1 = choose from the shape; 1 = one group of 4 rows per workgroup
    int mfma_min_batch;    // 0 = default (3); batches below it use the ALU kernels; 9 = never
    int variant;           // AP_VARIANT_*: 0 = choose; 1 = never the matrix-core kernel with in-wave exchange;
                           // 3 = that kernel whenever the shape allows it (batch >= 2, K % 128 == 0);
                           // 5 = the bank-per-lane kernel at batch 1, b >= 7;
                           // 7 / 8 = two row groups per workgroup at batch 1 whenever possible / never;
                           // 9 / 10 = the 16-row-tile matrix-core kernel (batch >= 2, K % 256 == 0) with one /
                           //          two tiles per workgroup
};

constexpr int kMaxMulti = 8;
struct MultiArgs { // passed by value as the kernel argument of a fused launch
    const uint8_t *slices[kMaxMulti];
    size_t slice_bytes[kMaxMulti];
    const uint16_t *lut[kMaxMulti];
    const uint16_t *x[kMaxMulti];
    uint16_t *y[kMaxMulti];
    int M[kMaxMulti];
    int group_begin[kMaxMulti]; // first workgroup of matrix i
    int count, K, batch;
};

// Work list of gemv_list_kernel, passed by value as its kernel argument (batch 1).
constexpr int kMaxListItems = 32;
struct ListItem {
    const uint8_t *slices;
    size_t slice_bytes;
    const uint16_t *lut; // table of this item's bit-width
    const uint16_t *x;
    uint16_t *y;
    int M, K, b;
    int pad;
};
struct ListArgs {
    ListItem item[kMaxListItems];
    int group_begin[kMaxListItems]; // first workgroup of item i (filled in by the launcher)
    int count;
};

hipError_t launch_gemv(const GemvArgs &a, hipStream_t stream);
// a work list on the batch-1/2 kernel: every item at batch `batch` (1 or 2); group_begin is filled in there
hipError_t launch_gemv_list(ListArgs &a, int batch, hipStream_t stream);
hipError_t launch_gemv_multi(const MultiArgs &a, int b, int total_groups, hipStream_t stream);
// the same launch on the matrix-core kernel over tiles of 16 rows (batch 2..8, K % 256 == 0)
hipError_t launch_matrix_tile_multi(const MultiArgs &a, int b, hipStream_t stream);
// a work list on that kernel: every item at bit-width b, K % 256 == 0, all rows in the same class of length
// (below / from 12288 columns); group_begin is filled in here
hipError_t launch_matrix_tile_list(ListArgs &a, int b, int batch, hipStream_t stream);
hipError_t launch_dequantize(const GemvArgs &a, hipStream_t stream);
hipError_t launch_probe_read(const void *dev_buf, size_t bytes, hipStream_t stream);
hipError_t launch_probe_issue(int kind, int passes, hipStream_t stream);
// Looks up, once per device, the device address of the static array ap_gemm_static writes the dense
// weights to (the current device's copy); called where a matrix is set up on a device.
bool static_scratch_setup();

} // namespace apgemv
#endif
