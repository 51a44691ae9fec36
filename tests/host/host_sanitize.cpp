// Host-side driver for the sanitizer run: the packer, the quantiser, the argument checks of every
// C-ABI entry point and the C oracle, built with -fsanitize=address,undefined and run on the CPU.
// No GPU: the kernel launchers are stubs (never reached: every call below fails its checks first or
// is host-only).  Exit status 0 = every check held and the sanitizers stayed silent.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/apgemv.h"
#include "../../paper_2402_10517_amd/csrc/kernels.h"
#include "../../paper_2402_10517_amd/csrc/dense_gemm.h"

extern "C" {
int oracle_gemv(const uint8_t *idx, int M, int K, int n, const uint16_t *lut, int b, const uint16_t *x, int batch,
                double *y, double *mag);
int oracle_dequantize(const uint8_t *idx, int M, int K, int n, const uint16_t *lut, int b, double *w);
unsigned oracle_truncate_index(unsigned idx_n, int n, int b);
double oracle_fp16_to_double(uint16_t h);
}

// ---- stubs of what needs a GPU -------------------------------------------------------------------
namespace apgemv {
hipError_t launch_gemv(const GemvArgs &, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_gemv_multi(const MultiArgs &, int, int, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_matrix_tile_multi(const MultiArgs &, int, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_matrix_tile_list(ListArgs &, int, int, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_gemv_list(ListArgs &, int, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_dequantize(const GemvArgs &, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_probe_read(const void *, size_t, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_probe_issue(int, int, hipStream_t) { return hipErrorInvalidValue; }
bool static_scratch_setup() { return false; }
bool dense_gemm_f16(const void *, const void *, void *, int, int, int, hipStream_t) { return false; }
} // namespace apgemv

#define CHECK(c)                                                                  \
    do {                                                                          \
        if (!(c)) {                                                               \
            std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); \
            return 1;                                                             \
        }                                                                         \
    } while (0)

static uint32_t rng_state = 20240210u;
static uint32_t rnd() { return rng_state = rng_state * 1664525u + 1013904223u; }

int main()
{
    const unsigned full = 0x1f8; // tables for b = 3..8
    size_t sz = 0;
    CHECK(ap_packed_size(0, 64, 8, full, &sz) == AP_ERR_SHAPE);
    CHECK(ap_packed_size(8, 48, 8, full, &sz) == AP_ERR_SHAPE);
    CHECK(ap_packed_size(8, 64, 9, full, &sz) == AP_ERR_BITS);
    CHECK(ap_packed_size(8, 64, 8, 0, &sz) == AP_ERR_BITS);
    CHECK(ap_packed_size(8, 64, 8, full, nullptr) == AP_ERR_INVALID_ARG);

    const int shapes[][3] = {{8, 64, 8}, {37, 96, 8}, {5, 2048 + 160, 8}, {130, 4096 + 32, 8}, {9, 512, 6}, {3, 32, 3}};
    for (const auto &sh : shapes) {
        const int M = sh[0], K = sh[1], n = sh[2];
        for (int pattern = 0; pattern < 4; ++pattern) {
            std::vector<uint8_t> idx((size_t)M * K);
            for (auto &v : idx)
                v = pattern == 0 ? (uint8_t)(rnd() >> 24) & ((1u << n) - 1)
                    : pattern == 1 ? 0 : pattern == 2 ? (uint8_t)((1u << n) - 1) : (uint8_t)(1u << (rnd() % n));
            std::vector<std::vector<uint16_t>> luts(9);
            const uint16_t *ptr[9] = {};
            unsigned mask = 0;
            for (int b = 3; b <= n; ++b) {
                if (pattern == 3 && b == 4 && n > 4) continue; // a sparse supported set
                luts[b].resize((size_t)M << b);
                for (auto &v : luts[b]) v = (uint16_t)(rnd() >> 16);
                ptr[b] = luts[b].data();
                mask |= 1u << b;
            }
            CHECK(ap_packed_size(M, K, n, mask, &sz) == AP_OK);
            std::vector<uint8_t> blob(sz);
            CHECK(ap_pack_host(idx.data(), M, K, n, ptr, blob.data(), sz - 1) == AP_ERR_BUFFER_TOO_SMALL);
            CHECK(ap_pack_host(idx.data(), M, K, n, ptr, blob.data(), sz) == AP_OK);
            std::vector<uint8_t> back((size_t)M * K, 0xee);
            CHECK(ap_unpack_host(blob.data(), sz, back.data()) == AP_OK);
            CHECK(back == idx);
            for (int b = 3; b <= n; ++b) {
                if (!ptr[b]) continue;
                for (int t = 0; t < 16; ++t) {
                    const int row = rnd() % M, e = rnd() % (1 << b);
                    uint16_t got = 0;
                    CHECK(ap_blob_lut_entry(blob.data(), sz, b, row, e, &got) == AP_OK);
                    CHECK(got == luts[b][((size_t)row << b) + e]);
                }
                size_t s0, s1, l0, l1;
                CHECK(ap_read_extent(M, K, n, mask, b, &s0, &s1, &l0, &l1) == AP_OK);
                CHECK(s0 < s1 && s1 <= l0 && l0 < l1 && l1 <= sz);
            }
            CHECK(ap_unpack_host(blob.data(), 10, back.data()) == AP_ERR_INVALID_ARG);
            blob[0] ^= 1;
            CHECK(ap_unpack_host(blob.data(), sz, back.data()) == AP_ERR_INVALID_ARG);
            if (n < 8 && pattern == 0) {
                idx[idx.size() / 2] = (uint8_t)(1u << n);
                CHECK(ap_pack_host(idx.data(), M, K, n, ptr, blob.data(), sz) == AP_ERR_INDEX_RANGE);
            }
        }
    }

    // the quantiser: indices within range, prefix nesting of the tables' clusters, degenerate rows
    {
        const int M = 5, K = 256;
        std::vector<float> w((size_t)M * K), s((size_t)M * K);
        for (auto &v : w) v = ((int)(rnd() >> 20) - 2048) * 1e-5f;
        for (auto &v : s) v = 1e-3f + (rnd() >> 20) * 1e-3f;
        for (int j = 0; j < K; ++j) w[(size_t)4 * K + j] = 0.125f; // a constant row
        std::vector<uint8_t> idx((size_t)M * K);
        std::vector<std::vector<uint16_t>> luts(9);
        uint16_t *ptr[9] = {};
        for (int b = 3; b <= 8; ++b) {
            luts[b].resize((size_t)M << b);
            ptr[b] = luts[b].data();
        }
        CHECK(ap_quantize(w.data(), s.data(), M, K, 3, 8, 12, idx.data(), ptr) == AP_OK);
        CHECK(ap_quantize(w.data(), nullptr, M, K, 3, 6, 12, idx.data(), ptr) == AP_OK);
        for (auto v : idx) CHECK(v < 64);
        CHECK(ap_quantize(w.data(), s.data(), M, K, 4, 3, 12, idx.data(), ptr) == AP_ERR_BITS);
        CHECK(ap_quantize(nullptr, s.data(), M, K, 3, 8, 12, idx.data(), ptr) == AP_ERR_INVALID_ARG);
    }

    // device entry points: every argument check precedes the first HIP call
    {
        void *fake = reinterpret_cast<void *>(0x10000);
        ap_matrix *h = nullptr;
        std::vector<uint8_t> idx(8 * 64, 1);
        std::vector<uint16_t> lut(8 * 8, 0x3c00);
        const uint16_t *ptr[9] = {};
        ptr[3] = lut.data();
        CHECK(ap_pack(nullptr, 8, 64, 8, ptr, fake, 1 << 20, nullptr, &h) == AP_ERR_INVALID_ARG);
        CHECK(ap_pack(idx.data(), 8, 40, 8, ptr, fake, 1 << 20, nullptr, &h) == AP_ERR_SHAPE);
        CHECK(ap_pack(idx.data(), 8, 64, 8, ptr, fake, 16, nullptr, &h) == AP_ERR_BUFFER_TOO_SMALL);
        CHECK(ap_pack(idx.data(), 8, 64, 8, ptr, reinterpret_cast<void *>(0x10004), 1 << 20, nullptr, &h) == AP_ERR_INVALID_ARG);
        CHECK(ap_attach(nullptr, 1 << 20, nullptr, &h) == AP_ERR_INVALID_ARG);
        CHECK(ap_gemv(nullptr, 4, fake, fake, 1, nullptr) == AP_ERR_INVALID_ARG);
        CHECK(ap_gemv_multi(nullptr, 1, 4, 1, nullptr) == AP_ERR_INVALID_ARG);
        CHECK(ap_gemv_list(nullptr, 1, nullptr) == AP_ERR_INVALID_ARG);
        ap_gemv_list_item li = {nullptr, 4, fake, fake};
        CHECK(ap_gemv_list(&li, 1, nullptr) == AP_ERR_INVALID_ARG);
        CHECK(ap_gemv_list(&li, 0, nullptr) == AP_ERR_INVALID_ARG);
        CHECK(ap_dequantize(nullptr, 4, fake, nullptr) == AP_ERR_INVALID_ARG);
        CHECK(ap_gemm(nullptr, 4, fake, fake, 32, fake, 1 << 20, nullptr) == AP_ERR_INVALID_ARG);
        CHECK(ap_gemm_workspace_size(nullptr, &sz) == AP_ERR_INVALID_ARG);
        CHECK(ap_set_option(nullptr, 0, 0) == AP_ERR_INVALID_ARG);
        CHECK(ap_unpack(nullptr, idx.data(), nullptr) == AP_ERR_INVALID_ARG);
        CHECK(ap_matrix_info(nullptr, nullptr, nullptr, nullptr, nullptr) == AP_ERR_INVALID_ARG);
        CHECK(ap_probe_read(fake, 1000, nullptr) == AP_ERR_INVALID_ARG);
        ap_free(nullptr);
        for (int st = 0; st < 10; ++st) CHECK(std::strlen(ap_strerror((ap_status)st)) > 0);
    }

    // the oracle: a one-hot activation returns the looked-up table entry exactly, for every b
    {
        const int M = 7, K = 96, n = 8;
        std::vector<uint8_t> idx((size_t)M * K);
        for (auto &v : idx) v = (uint8_t)(rnd() >> 24);
        for (int b = 3; b <= 8; ++b) {
            std::vector<uint16_t> lut((size_t)M << b);
            for (size_t i = 0; i < lut.size(); ++i) lut[i] = (uint16_t)(0x3c00 + (i & 0x3ff)); // 1.0 .. 2.0
            std::vector<uint16_t> x(K, 0);
            const int j = (int)(rnd() % K);
            x[j] = 0x3c00;
            std::vector<double> y(M), mag(M), dense((size_t)M * K);
            CHECK(oracle_gemv(idx.data(), M, K, n, lut.data(), b, x.data(), 1, y.data(), mag.data()) == 0);
            CHECK(oracle_dequantize(idx.data(), M, K, n, lut.data(), b, dense.data()) == 0);
            for (int i = 0; i < M; ++i) {
                const unsigned e = oracle_truncate_index(idx[(size_t)i * K + j], n, b);
                CHECK(e == (unsigned)(idx[(size_t)i * K + j] >> (n - b)));
                CHECK(y[i] == oracle_fp16_to_double(lut[((size_t)i << b) + e]));
                CHECK(dense[(size_t)i * K + j] == y[i]);
            }
        }
    }
    std::puts("host sanitizer driver: all checks held");
    return 0;
}
