/*
 * CPU oracle for the any-precision matrix-vector product.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's cpu_baseline
 * leg, never by the product path, and it shares no code with the HIP library.
 *
 * What it computes is the plain definition of the operation (Any-Precision LLM,
 * Section 3.3 "Concept" and Section 5.2 "System Overview"): one stored n-bit index per
 * weight; the b-bit model uses the b most significant bits of that index (Section 4.1:
 * every upscale appends one bit at the end, so earlier bits are the more significant
 * ones; Section 5.2: a 4-bit run of an 8-bit parent reads bitplanes 4..7) and looks
 * them up in the output channel's own table of 2^b centroids (Section 5.2: one table
 * row per output channel, 2^k values per row); the result is the dot product of the
 * dequantised row with the activations (Section 5.2, thread-level steps 4 and 5).
 *
 * Precision: centroids and activations are IEEE binary16 bit patterns, decoded exactly
 * to double; products and sums are carried in double, summed in column order.
 * No blocking, no SIMD, no reordering.
 *
 * Pins (tests/test_oracle_pins.py): brute-force dense dequantise-then-matmul in numpy
 * float64 (numpy's own binary16 decode), one-hot activations reproducing single table
 * entries exactly, integer tables giving exact integer sums, the MSB-nesting invariant,
 * and the storage closed form against the footprints printed in Table 1.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the row loop of oracle_gemv will use (reported beside timings; no arithmetic here). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* IEEE 754 binary16 bit pattern -> double, exact (subnormals, signed zero, inf, nan). */
double oracle_fp16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);                 /* subnormal or zero: frac * 2^-24 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp((double)(frac | 0x400), expo - 25); /* (1024+frac) * 2^(expo-15-10)   */
    return sign ? -v : v;
}

/* The b-bit model's index of a weight whose stored n-bit index is idx_n:
 * its b most significant bits (Section 3.3; Section 4.1). */
unsigned oracle_truncate_index(unsigned idx_n, int n, int b)
{
    return idx_n >> (n - b);
}

/*
 * y[t*M + i]   = sum_j  C_b[i][ idx[i][j] >> (n-b) ] * x[t][j]
 * mag[t*M + i] = sum_j |C_b[i][ idx[i][j] >> (n-b) ]| * |x[t][j]|     (for the tolerance)
 *
 * idx : M*K bytes, row-major (row = output channel), each value < 2^n
 * lut : M * 2^b binary16 bit patterns, row-major: entry e of row i at lut[i*2^b + e]
 * x   : batch*K binary16 bit patterns, row-major
 * y, mag : batch*M doubles, row-major (either may be NULL)
 * Returns 0, or -1 on an argument the definition does not cover.
 */
int oracle_gemv(const uint8_t *idx, int M, int K, int n,
                const uint16_t *lut, int b,
                const uint16_t *x, int batch,
                double *y, double *mag)
{
    if (!idx || !lut || !x || M < 0 || K < 0 || batch < 0) return -1;
    if (n < 1 || n > 8 || b < 1 || b > n) return -1;
    const size_t entries = (size_t)1 << b;
    for (int t = 0; t < batch; ++t) {
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
        for (int i = 0; i < M; ++i) {
            double acc = 0.0, m = 0.0;
            for (int j = 0; j < K; ++j) {
                unsigned e = oracle_truncate_index(idx[(size_t)i * K + j], n, b);
                double w = oracle_fp16_to_double(lut[(size_t)i * entries + e]);
                double xv = oracle_fp16_to_double(x[(size_t)t * K + j]);
                acc += w * xv;
                m += fabs(w) * fabs(xv);
            }
            if (y) y[(size_t)t * M + i] = acc;
            if (mag) mag[(size_t)t * M + i] = m;
        }
    }
    return 0;
}

/* Dense dequantised matrix of the b-bit model: W[i*K + j] = C_b[i][idx[i][j] >> (n-b)]. */
int oracle_dequantize(const uint8_t *idx, int M, int K, int n,
                      const uint16_t *lut, int b, double *W)
{
    if (!idx || !lut || !W || n < 1 || n > 8 || b < 1 || b > n) return -1;
    const size_t entries = (size_t)1 << b;
    for (int i = 0; i < M; ++i)
        for (int j = 0; j < K; ++j)
            W[(size_t)i * K + j] = oracle_fp16_to_double(
                lut[(size_t)i * entries + oracle_truncate_index(idx[(size_t)i * K + j], n, b)]);
    return 0;
}

/*
 * Storage closed form of an any-precision deployment (Section 3.3, Table 1): the parent
 * model's n-bit indices for every quantised weight, one binary16 centroid table of 2^b
 * entries per output channel for every supported bit-width b, plus whatever stays
 * unquantised (other_bytes).  bit_mask has bit b set when b is supported; n is the
 * largest supported b.
 */
double oracle_anyprecision_bytes(double n_weights, double n_rows, unsigned bit_mask, double other_bytes)
{
    int n = 0;
    double table_bytes = 0.0;
    for (int b = 1; b <= 8; ++b)
        if (bit_mask & (1u << b)) { n = b; table_bytes += (double)(1u << b) * 2.0; }
    return n_weights * n / 8.0 + n_rows * table_bytes + other_bytes;
}
