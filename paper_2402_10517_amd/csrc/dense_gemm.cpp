// Dense FP16 GEMM through rocBLAS, loaded with dlopen on first use so that the library has no
// link-time dependency on it (the GEMV path never touches it).
#include "dense_gemm.h"

#include <dlfcn.h>
#include <rocblas/rocblas.h>

#include <mutex>

namespace apgemv {

namespace {

struct Blas {
    void *lib = nullptr;
    rocblas_handle handle = nullptr;
    decltype(&rocblas_create_handle) create = nullptr;
    decltype(&rocblas_set_stream) set_stream = nullptr;
    decltype(&rocblas_gemm_ex) gemm_ex = nullptr;
    bool ok = false;
};

Blas &blas()
{
    static Blas b;
    static std::once_flag once;
    std::call_once(once, [] {
        const char *names[] = {"librocblas.so.5", "librocblas.so"};
        for (const char *n : names) {
            b.lib = dlopen(n, RTLD_NOW | RTLD_GLOBAL);
            if (b.lib) break;
        }
        if (!b.lib) return;
        b.create = reinterpret_cast<decltype(b.create)>(dlsym(b.lib, "rocblas_create_handle"));
        b.set_stream = reinterpret_cast<decltype(b.set_stream)>(dlsym(b.lib, "rocblas_set_stream"));
        b.gemm_ex = reinterpret_cast<decltype(b.gemm_ex)>(dlsym(b.lib, "rocblas_gemm_ex"));
        if (!b.create || !b.set_stream || !b.gemm_ex) return;
        if (b.create(&b.handle) != rocblas_status_success) return;
        b.ok = true;
    });
    return b;
}

} // namespace

bool dense_gemm_f16(const void *w_dev, const void *x_dev, void *y_dev, int M, int K, int batch,
                    hipStream_t stream)
{
    Blas &b = blas();
    if (!b.ok) return false;
    // one rocBLAS handle for the process: the stream it is bound to and the call that uses it must not
    // be separated by another thread's call
    static std::mutex call_lock;
    std::lock_guard<std::mutex> guard(call_lock);
    if (b.set_stream(b.handle, stream) != rocblas_status_success) return false;
    // Column-major view: Y^T (M x batch, ld M) = W (op T on the K x M view, ld K) * X^T (K x batch, ld K)
    const float alpha = 1.0f, beta = 0.0f;
    rocblas_status st = b.gemm_ex(b.handle, rocblas_operation_transpose, rocblas_operation_none, M, batch,
                                  K, &alpha, w_dev, rocblas_datatype_f16_r, K, x_dev,
                                  rocblas_datatype_f16_r, K, &beta, y_dev, rocblas_datatype_f16_r, M,
                                  y_dev, rocblas_datatype_f16_r, M, rocblas_datatype_f32_r,
                                  rocblas_gemm_algo_standard, 0, 0);
    return st == rocblas_status_success;
}

} // namespace apgemv
