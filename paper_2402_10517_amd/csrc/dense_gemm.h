// Dense FP16 GEMM used by the large-batch path: a plain library GEMM (rocBLAS), bound at run time.
#ifndef APGEMV_DENSE_GEMM_H
#define APGEMV_DENSE_GEMM_H

#include <hip/hip_runtime_api.h>

namespace apgemv {

// y[batch x M] = x[batch x K] * w[M x K]^T, all binary16 row-major, binary32 accumulation.
// Returns false if rocBLAS cannot be loaded or reports an error.
bool dense_gemm_f16(const void *w_dev, const void *x_dev, void *y_dev, int M, int K, int batch,
                    hipStream_t stream);

} // namespace apgemv
#endif
