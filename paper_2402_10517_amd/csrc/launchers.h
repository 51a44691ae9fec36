// Launchers of the kernel families (each defined next to its kernels); launch_gemv chooses between them.
#ifndef APGEMV_LAUNCHERS_H
#define APGEMV_LAUNCHERS_H

#include "kernels.h"

namespace apgemv {

hipError_t launch_alu(const GemvArgs &a, hipStream_t stream);                 // gemv_kernel / gemv_rows_kernel
hipError_t launch_quad(const GemvArgs &a, hipStream_t stream);                // gemv_quad_kernel (batch 1, b = 7, 8)
hipError_t launch_matrix_row_per_lane(const GemvArgs &a, hipStream_t stream); // gemv_mfma_kernel (batch >= 3, K % 128 == 0)
hipError_t launch_matrix_exchange(const GemvArgs &a, hipStream_t stream);     // gemv_xmfma_kernel (batch >= 2, K % 128 == 0)
hipError_t launch_matrix_tile(const GemvArgs &a, hipStream_t stream);         // gemv_tile_kernel (batch >= 2, K % 256 == 0)

} // namespace apgemv
#endif
