// Any-precision quantisation by incremental upscaling on the host (Any-Precision LLM, Section 4):
// a seed model of n_seed bits per weight from a sensitivity-weighted clustering of every output
// channel (Section 4.2: SqueezeLLM-style non-uniform quantisation), then one bit at a time: every
// cluster is divided in two by a weighted 2-means over its members, the new bit is appended at
// the end of the index (Section 4.1), and the table of the wider model holds the sub-cluster
// centroids.  Produces the parent index matrix and one centroid table per bit-width - the inputs
// of ap_pack.  CPU only (the paper runs this step on a CPU, Section 6.1).
//
// Where the paper is silent, the choices are: clustering is per output channel and one-dimensional;
// Lloyd iterations start from centroids at the weighted quantiles (q + 0.5)/k, run a fixed number of
// rounds (early exit when no assignment changes), assign to the nearest centroid with ties to the
// lower one, and keep the previous centroid of an empty cluster; the sub-cluster with the lower
// centroid gets bit 0; a cluster that cannot be divided (fewer than two distinct values) passes its
// centroid to both children and its members to child 0.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <thread>
#include <vector>

#include "../../include/apgemv.h"

#pragma clang fp contract(off) // sums must round like the plain reference loops

namespace {

// binary64 -> binary16 bit pattern, round to nearest even (overflow -> infinity)
uint16_t double_to_half_bits(double d)
{
    uint64_t u;
    std::memcpy(&u, &d, 8);
    const uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
    const double a = std::fabs(d);
    if (std::isnan(d)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);
    if (a < 5.9604644775390625e-8 * 0.5) return sign;                 // below half the smallest subnormal
    int e;
    std::frexp(a, &e);                                                // a = m * 2^e, m in [0.5, 1)
    int exp16 = e - 1 + 15;                                           // biased exponent if normal
    double scaled;
    if (exp16 >= 1) scaled = std::ldexp(a, 10 - (e - 1));             // in [1024, 2048)
    else { scaled = std::ldexp(a, 24); exp16 = 0; }                   // subnormal: units of 2^-24
    double r = std::nearbyint(scaled);                                // ties to even (default mode)
    uint32_t mant = (uint32_t)r;
    if (exp16 >= 1) {
        if (mant == 2048) { mant = 1024; ++exp16; }
        if (exp16 >= 31) return (uint16_t)(sign | 0x7c00u);
        return (uint16_t)(sign | (exp16 << 10) | (mant - 1024));
    }
    return (uint16_t)(sign | mant);                                   // mant == 1024 becomes the smallest normal
}

struct Cluster {
    std::vector<double> centroids;  // k
    std::vector<int> assign;        // per member
};

// Weighted one-dimensional k-means over v[0..m) with weights s.
void kmeans_1d(const double *v, const double *s, int m, int k, int iters, Cluster &out)
{
    out.centroids.assign(k, 0.0);
    out.assign.assign(m, 0);
    if (m == 0) return;
    std::vector<int> order(m);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return v[a] < v[b]; });
    double total = 0.0;
    for (int i = 0; i < m; ++i) total += s[order[i]];
    // initial centroids: values at the weighted quantiles (q + 0.5) / k
    {
        int pos = 0;
        double cum = s[order[0]];
        for (int q = 0; q < k; ++q) {
            const double target = (q + 0.5) / k * total;
            while (cum < target && pos + 1 < m) cum += s[order[++pos]];
            out.centroids[q] = v[order[pos]];
        }
    }
    std::vector<double> num(k), den(k);
    for (int it = 0; it <= iters; ++it) {
        bool changed = false;
        for (int i = 0; i < m; ++i) {
            int best = 0;
            double bd = std::fabs(v[i] - out.centroids[0]);
            for (int q = 1; q < k; ++q) {
                const double d = std::fabs(v[i] - out.centroids[q]);
                if (d < bd) { bd = d; best = q; }
            }
            if (best != out.assign[i]) { out.assign[i] = best; changed = true; }
        }
        if (it == iters || (!changed && it > 0)) break;
        std::fill(num.begin(), num.end(), 0.0);
        std::fill(den.begin(), den.end(), 0.0);
        for (int i = 0; i < m; ++i) {
            const double p = s[i] * v[i];
            num[out.assign[i]] += p;
            den[out.assign[i]] += s[i];
        }
        for (int q = 0; q < k; ++q)
            if (den[q] > 0.0) out.centroids[q] = num[q] / den[q];
    }
}

void quantize_row(const float *w, const float *sens, int K, int n_seed, int n, int iters, uint8_t *idx,
                  uint16_t *const luts[9], int row)
{
    std::vector<double> v(K), s(K);
    for (int j = 0; j < K; ++j) {
        v[j] = (double)w[j];
        s[j] = sens ? (double)sens[j] : 1.0;
    }
    Cluster seed;
    kmeans_1d(v.data(), s.data(), K, 1 << n_seed, iters, seed);
    // order the seed clusters by centroid so that the seed table ascends
    std::vector<int> rank(1 << n_seed), by(1 << n_seed);
    std::iota(by.begin(), by.end(), 0);
    std::stable_sort(by.begin(), by.end(), [&](int a, int b) { return seed.centroids[a] < seed.centroids[b]; });
    for (int q = 0; q < (1 << n_seed); ++q) rank[by[q]] = q;
    std::vector<int> code(K);
    std::vector<double> cent(1 << n_seed);
    for (int q = 0; q < (1 << n_seed); ++q) cent[rank[q]] = seed.centroids[q];
    for (int j = 0; j < K; ++j) code[j] = rank[seed.assign[j]];
    if (luts[n_seed])
        for (int q = 0; q < (1 << n_seed); ++q) luts[n_seed][((size_t)row << n_seed) + q] = double_to_half_bits(cent[q]);

    std::vector<double> mv, ms;
    std::vector<int> members;
    for (int b = n_seed; b < n; ++b) {
        std::vector<double> next(2 << b);
        std::vector<int> next_code(K);
        for (int c = 0; c < (1 << b); ++c) {
            members.clear();
            mv.clear();
            ms.clear();
            for (int j = 0; j < K; ++j)
                if (code[j] == c) { members.push_back(j); mv.push_back(v[j]); ms.push_back(s[j]); }
            Cluster two;
            kmeans_1d(mv.data(), ms.data(), (int)members.size(), 2, iters, two);
            bool divisible = false;
            for (size_t i = 0; i < members.size(); ++i)
                if (two.assign[i] != two.assign[0]) divisible = true;
            if (!divisible) {
                next[2 * c] = next[2 * c + 1] = cent[c];
                for (int j : members) next_code[j] = 2 * c;
            } else {
                const bool swap = two.centroids[1] < two.centroids[0];
                next[2 * c] = two.centroids[swap ? 1 : 0];
                next[2 * c + 1] = two.centroids[swap ? 0 : 1];
                for (size_t i = 0; i < members.size(); ++i)
                    next_code[members[i]] = 2 * c + (two.assign[i] ^ (swap ? 1 : 0));
            }
        }
        cent.swap(next);
        code.swap(next_code);
        if (luts[b + 1])
            for (int q = 0; q < (2 << b); ++q) luts[b + 1][((size_t)row << (b + 1)) + q] = double_to_half_bits(cent[q]);
    }
    for (int j = 0; j < K; ++j) idx[j] = (uint8_t)code[j];
}

} // namespace

extern "C" ap_status ap_quantize(const float *w, const float *sens, int M, int K, int n_seed, int n, int iters,
                                 uint8_t *idx_out, uint16_t *const luts_out[9])
{
    if (!w || !idx_out || !luts_out) return AP_ERR_INVALID_ARG;
    if (M < 1 || K < 1) return AP_ERR_SHAPE;
    if (n_seed < 1 || n > AP_MAX_BITS || n_seed > n) return AP_ERR_BITS;
    if (iters < 1) return AP_ERR_INVALID_ARG;
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<unsigned>(hw ? hw : 1, 16);
    nt = std::max(1, std::min(nt, M));
    std::vector<std::thread> th;
    for (int t = 0; t < nt; ++t)
        th.emplace_back([=] {
            for (int i = t; i < M; i += nt)
                quantize_row(w + (size_t)i * K, sens ? sens + (size_t)i * K : nullptr, K, n_seed, n, iters,
                             idx_out + (size_t)i * K, luts_out, i);
        });
    for (auto &t : th) t.join();
    return AP_OK;
}
