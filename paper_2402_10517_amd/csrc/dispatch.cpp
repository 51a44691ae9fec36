// Bit-width and kernel-family dispatch of one ap_gemv call: one stored matrix, the kernel and the
// table are chosen per call (Section 5.2: only the first b slices and the b-bit table are touched).
#include "launchers.h"
#include "layout.h"

namespace apgemv {

hipError_t launch_gemv(const GemvArgs &a, hipStream_t stream)
{
    if (a.b < 3 || a.b > 8) return hipErrorInvalidValue;
    const int B = a.b;
    // Bank-per-lane lookups at batch 1, b = 7, 8: conflict-free, but two operations per table address
    // and 8 copies of every table; measured slower than the shared-table kernel on every Llama shape
    // (b = 8: 8.2 / 17.7 / 19.6 us against 6.8 / 12.0 / 12.7 us on the 7B shapes), so only on request.
    if (a.batch == 1 && B >= 7 && a.variant == 5) return launch_quad(a, stream);
    // The matrix-core kernel on tiles of 16 rows (K % 256 == 0).  Measured on the 7B, 13B and 70B shapes at
    // batch 2, 3, 4, 6, 8 against the kernels below: at batch >= 5 it wins on every matrix with at least
    // 1024 groups of rows (5 to 60 %, most at small b and long rows); at batch 3 and 4 it wins by 5 to
    // 40 % on matrices with at least 2048 groups of rows and on rows of 16384 columns or more (level at
    // b = 5, 6 on 28672 x 8192) and loses on smaller ones; at batch 2, and on 1024 x 8192 at every
    // batch, the ALU kernels are faster.
    // variant: 9 / 10 = this kernel with one / two tiles per workgroup whenever the shape allows; any
    // other tuning override keeps the call away from it.
    if (a.batch >= 2 && a.K % 256 == 0) {
        const int groups = padded_rows(a.M) / kRowsPerGroup;
        const bool tuned = a.row_groups_per_wg >= 0 || a.mfma_min_batch != 0 || a.waves_per_group != 0;
        const bool pays = a.variant == 0 && !tuned && groups >= 1024 &&
                          (a.batch >= 5 || (a.batch >= 3 && (a.K >= 16384 || groups >= 2048)));
        if (a.variant == 9 || a.variant == 10 || pays) return launch_matrix_tile(a, stream);
    }
    // What is left for batch >= 2 (K not a multiple of 256, smaller matrices, batch 2..4) was settled by
    // measurement on the 70B shapes (8192x8192, 28672x8192, 8192x28672; all b):
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
            return launch_matrix_exchange(a, stream);
    }
    // The first matrix-core kernel (one row per lane): batch 3..8 at b >= 6 when the row length allows
    // it; at b <= 5 the four rows' small tables of a block share LDS banks and it is slower.  Matrices
    // with fewer than 2048 groups of rows stay on the ALU kernels: measured on 4096x4096 and 4096x11008
    // at batch 3, 4, 8 the ALU kernels are level or up to 30 % faster there (the device is not full,
    // and a call is bound by latency, not by the multiply-accumulates the matrix cores take over).
    // (mfma_min_batch: tuning override, also of the size rule; a negative value lifts the b limit too.)
    const int min_batch = a.mfma_min_batch > 0 ? a.mfma_min_batch : a.mfma_min_batch < 0 ? -a.mfma_min_batch : 3;
    const bool big_enough = a.mfma_min_batch != 0 || padded_rows(a.M) / kRowsPerGroup >= 2048;
    if (a.batch >= min_batch && a.K % 128 == 0 && big_enough && (B >= 6 || a.mfma_min_batch < 0))
        return launch_matrix_row_per_lane(a, stream);
    return launch_alu(a, stream);
}

} // namespace apgemv
