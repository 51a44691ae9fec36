// C-ABI entry points that touch the device: upload, download, attach, GEMV dispatch.
#include <hip/hip_runtime_api.h>

#include <cstring>
#include <mutex>
#include <new>

#include "dense_gemm.h"
#include "handle.h"
#include "kernels.h"
#include "pack.h"

using namespace apgemv;

// Pinned host staging for uploads and downloads of packed matrices: one buffer per process, grown to
// the largest size asked for and kept (pinned memory transfers at about twice the rate of pageable
// memory, and allocating it per call would cost more than the transfer).  Calls are serialised on it.
namespace {
struct Staging {
    std::mutex lock;
    void *ptr = nullptr;
    size_t capacity = 0;
    // with `lock` held
    uint8_t *reserve(size_t bytes)
    {
        if (bytes <= capacity) return static_cast<uint8_t *>(ptr);
        if (ptr) (void)hipHostFree(ptr);
        ptr = nullptr;
        capacity = 0;
        if (hipHostMalloc(&ptr, bytes, hipHostMallocDefault) != hipSuccess) {
            ptr = nullptr;
            (void)hipGetLastError();
            return nullptr;
        }
        capacity = bytes;
        return static_cast<uint8_t *>(ptr);
    }
};
Staging &staging_buffer()
{
    static Staging *s = new Staging; // never destroyed: no HIP call during process teardown
    return *s;
}
} // namespace

static void default_tuning(ap_matrix *h)
{
    h->waves_per_group = 0;
    h->row_groups_per_wg = -1;
    h->mfma_min_batch = 0;
    h->variant = 0;
}

extern "C" ap_status ap_pack(const uint8_t *idx_host, int M, int K, int n,
                             const uint16_t *const luts_host[9], void *dev_buf,
                             size_t dev_buf_bytes, void *stream, ap_matrix **out)
{
    if (!idx_host || !luts_host || !dev_buf || !out) return AP_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dev_buf) % AP_BLOB_ALIGN) return AP_ERR_INVALID_ARG;
    ap_status s = check_shape(M, K, n);
    if (s != AP_OK) return s;
    unsigned mask = 0;
    for (int b = AP_MIN_BITS; b <= n; ++b)
        if (luts_host[b]) mask |= 1u << b;
    BlobHeader hdr;
    s = make_header(M, K, n, mask, &hdr);
    if (s != AP_OK) return s;
    if (dev_buf_bytes < hdr.total_bytes) return AP_ERR_BUFFER_TOO_SMALL;
    s = check_index_range(idx_host, M, K, n); // the last check that needs no HIP call
    if (s != AP_OK) return s;

    ap_matrix *h = new (std::nothrow) ap_matrix;
    if (!h) return AP_ERR_NO_MEMORY;
    {
        Staging &sb = staging_buffer();
        std::lock_guard<std::mutex> guard(sb.lock);
        uint8_t *staging = sb.reserve(hdr.total_bytes);
        if (!staging) {
            delete h;
            return AP_ERR_NO_MEMORY;
        }
        s = ap_pack_host(idx_host, M, K, n, luts_host, staging, hdr.total_bytes);
        hipStream_t st = static_cast<hipStream_t>(stream);
        if (s == AP_OK && (hipMemcpyAsync(dev_buf, staging, hdr.total_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
                           hipStreamSynchronize(st) != hipSuccess))
            s = AP_ERR_HIP;
        if (s != AP_OK) {
            delete h;
            return s;
        }
    }
    h->tag = kHandleTag;
    h->hdr = hdr;
    h->dev = static_cast<uint8_t *>(dev_buf);
    default_tuning(h);
    static_scratch_setup(); // set-up time: ap_gemm_static then finds its array without a lookup
    *out = h;
    return AP_OK;
}

extern "C" ap_status ap_attach(void *dev_buf, size_t dev_buf_bytes, void *stream, ap_matrix **out)
{
    if (!dev_buf || !out || dev_buf_bytes < sizeof(BlobHeader)) return AP_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dev_buf) % AP_BLOB_ALIGN) return AP_ERR_INVALID_ARG;
    BlobHeader hdr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(&hdr, dev_buf, sizeof(hdr), hipMemcpyDeviceToHost, st) != hipSuccess)
        return AP_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return AP_ERR_HIP;
    ap_status s = validate_header(&hdr, dev_buf_bytes);
    if (s != AP_OK) return s;
    ap_matrix *h = new (std::nothrow) ap_matrix;
    if (!h) return AP_ERR_NO_MEMORY;
    h->tag = kHandleTag;
    h->hdr = hdr;
    h->dev = static_cast<uint8_t *>(dev_buf);
    default_tuning(h);
    static_scratch_setup(); // set-up time: ap_gemm_static then finds its array without a lookup
    *out = h;
    return AP_OK;
}

extern "C" ap_status ap_set_option(ap_matrix *h, int option, int value)
{
    if (!handle_ok(h)) return AP_ERR_INVALID_ARG;
    switch (option) {
    case AP_OPT_WAVES_PER_GROUP:
        if (value < 0 || value > 8) return AP_ERR_INVALID_ARG;
        h->waves_per_group = value;
        return AP_OK;
    case AP_OPT_ROW_GROUPS_PER_WG:
        if (value < -1 || value == 0 || value > 4) return AP_ERR_INVALID_ARG;
        h->row_groups_per_wg = value;
        return AP_OK;
    case AP_OPT_MFMA_MIN_BATCH:
        if (value < -9 || value > 9) return AP_ERR_INVALID_ARG;
        h->mfma_min_batch = value;
        return AP_OK;
    case AP_OPT_VARIANT:
        if (value != AP_VARIANT_AUTO && value != AP_VARIANT_NO_EXCHANGE && value != AP_VARIANT_EXCHANGE &&
            value != AP_VARIANT_BANK_PER_LANE && value != AP_VARIANT_PAIR && value != AP_VARIANT_NO_PAIR &&
            value != AP_VARIANT_TILE && value != AP_VARIANT_TILE2)
            return AP_ERR_INVALID_ARG;
        h->variant = value;
        return AP_OK;
    }
    return AP_ERR_INVALID_ARG;
}

extern "C" ap_status ap_unpack(const ap_matrix *h, uint8_t *idx_host_out, void *stream)
{
    if (!handle_ok(h) || !idx_host_out) return AP_ERR_INVALID_ARG;
    const size_t bytes = h->hdr.slice_off + (size_t)h->hdr.n * h->hdr.slice_bytes;
    Staging &sb = staging_buffer();
    std::lock_guard<std::mutex> guard(sb.lock);
    uint8_t *staging = sb.reserve(bytes);
    if (!staging) return AP_ERR_NO_MEMORY;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(staging, h->dev, bytes, hipMemcpyDeviceToHost, st) != hipSuccess) return AP_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return AP_ERR_HIP;
    BlobHeader hdr;
    std::memcpy(&hdr, staging, sizeof(hdr));
    if (std::memcmp(&hdr, &h->hdr, sizeof(hdr)) != 0) return AP_ERR_INVALID_ARG;
    unpack_slices(staging, hdr, idx_host_out);
    return AP_OK;
}

extern "C" ap_status ap_gemv(const ap_matrix *h, int b, const void *x_dev, void *y_dev, int batch,
                             void *stream)
{
    if (!handle_ok(h) || !x_dev || !y_dev) return AP_ERR_INVALID_ARG;
    if (b < AP_MIN_BITS || b > h->hdr.n || !(h->hdr.lut_mask & (1u << b))) return AP_ERR_BITS;
    if (batch < 1 || batch > AP_MAX_BATCH) return AP_ERR_BATCH;
    if (reinterpret_cast<uintptr_t>(x_dev) % 16 || reinterpret_cast<uintptr_t>(y_dev) % 2)
        return AP_ERR_INVALID_ARG;
    GemvArgs a;
    a.slices = h->dev + h->hdr.slice_off;
    a.slice_bytes = h->hdr.slice_bytes;
    a.lut = reinterpret_cast<const uint16_t *>(h->dev + h->hdr.lut_off[b]);
    a.x = static_cast<const uint16_t *>(x_dev);
    a.y = static_cast<uint16_t *>(y_dev);
    a.M = h->hdr.M;
    a.K = h->hdr.K;
    a.b = b;
    a.batch = batch;
    a.waves_per_group = h->waves_per_group;
    a.row_groups_per_wg = h->row_groups_per_wg;
    a.mfma_min_batch = h->mfma_min_batch;
    a.variant = h->variant;
    // the kernels take up to 8 activation rows: larger batches in passes of 8 rows
    for (int first = 0; first < batch; first += AP_MAX_MULTI_BATCH) {
        a.x = static_cast<const uint16_t *>(x_dev) + (size_t)first * a.K;
        a.y = static_cast<uint16_t *>(y_dev) + (size_t)first * a.M;
        a.batch = batch - first < AP_MAX_MULTI_BATCH ? batch - first : AP_MAX_MULTI_BATCH;
        if (launch_gemv(a, static_cast<hipStream_t>(stream)) != hipSuccess) return AP_ERR_HIP;
    }
    return AP_OK;
}

static ap_status fill_args(const ap_matrix *h, int b, GemvArgs *a)
{
    if (!handle_ok(h)) return AP_ERR_INVALID_ARG;
    if (b < AP_MIN_BITS || b > h->hdr.n || !(h->hdr.lut_mask & (1u << b))) return AP_ERR_BITS;
    a->slices = h->dev + h->hdr.slice_off;
    a->slice_bytes = h->hdr.slice_bytes;
    a->lut = reinterpret_cast<const uint16_t *>(h->dev + h->hdr.lut_off[b]);
    a->x = nullptr;
    a->y = nullptr;
    a->M = h->hdr.M;
    a->K = h->hdr.K;
    a->b = b;
    a->batch = 1;
    a->waves_per_group = h->waves_per_group;
    a->row_groups_per_wg = h->row_groups_per_wg;
    a->mfma_min_batch = h->mfma_min_batch;
    a->variant = h->variant;
    return AP_OK;
}

// Checks one item of a batch-1 list and fills its slot of the kernel argument.
static ap_status fill_list_item(const ap_matrix *h, int b, const void *x_dev, void *y_dev, ListItem *li)
{
    GemvArgs a;
    ap_status s = fill_args(h, b, &a);
    if (s != AP_OK) return s;
    if (!x_dev || !y_dev) return AP_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(x_dev) % 16 || reinterpret_cast<uintptr_t>(y_dev) % 2) return AP_ERR_INVALID_ARG;
    li->slices = a.slices;
    li->slice_bytes = a.slice_bytes;
    li->lut = a.lut;
    li->x = static_cast<const uint16_t *>(x_dev);
    li->y = static_cast<uint16_t *>(y_dev);
    li->M = a.M;
    li->K = a.K;
    li->b = b;
    li->pad = 0;
    return AP_OK;
}

extern "C" ap_status ap_gemv_list(const ap_gemv_list_item *items, int count, void *stream)
{
    if (!items || count < 1) return AP_ERR_INVALID_ARG;
    ListItem probe;
    for (int i = 0; i < count; ++i) { // every item is checked before anything is enqueued
        ap_status s = fill_list_item(items[i].h, items[i].b, items[i].x_dev, items[i].y_dev, &probe);
        if (s != AP_OK) return s;
    }
    for (int first = 0; first < count; first += kMaxListItems) {
        ListArgs la;
        std::memset(&la, 0, sizeof(la));
        la.count = count - first < kMaxListItems ? count - first : kMaxListItems;
        for (int i = 0; i < la.count; ++i)
            fill_list_item(items[first + i].h, items[first + i].b, items[first + i].x_dev, items[first + i].y_dev,
                           &la.item[i]);
        if (launch_gemv_list(la, 1, static_cast<hipStream_t>(stream)) != hipSuccess) return AP_ERR_HIP;
    }
    return AP_OK;
}

extern "C" ap_status ap_gemv_list_batch(const ap_gemv_list_item *items, int count, int batch, void *stream)
{
    if (batch == 1) return ap_gemv_list(items, count, stream);
    if (!items || count < 1) return AP_ERR_INVALID_ARG;
    if (batch < 1 || batch > AP_MAX_MULTI_BATCH) return AP_ERR_BATCH;
    ListItem probe;
    for (int i = 0; i < count; ++i) { // every item is checked before anything is enqueued
        ap_status s = fill_list_item(items[i].h, items[i].b, items[i].x_dev, items[i].y_dev, &probe);
        if (s != AP_OK) return s;
    }
    if (batch == 2) {
        // single calls at batch 2 run the batch-1/2 kernel: the items without a tuning override go into list
        // launches of that kernel (any shapes and bit-widths together), the others run on their own
        auto plain = [](const ap_matrix *h) {
            return h->variant == AP_VARIANT_AUTO && h->waves_per_group == 0 && h->row_groups_per_wg < 0 && h->mfma_min_batch == 0;
        };
        ListArgs la;
        std::memset(&la, 0, sizeof(la));
        for (int i = 0; i < count; ++i) {
            if (!plain(items[i].h)) continue;
            fill_list_item(items[i].h, items[i].b, items[i].x_dev, items[i].y_dev, &la.item[la.count++]);
            if (la.count == kMaxListItems) {
                if (launch_gemv_list(la, 2, static_cast<hipStream_t>(stream)) != hipSuccess) return AP_ERR_HIP;
                la.count = 0;
            }
        }
        if (la.count > 0 && launch_gemv_list(la, 2, static_cast<hipStream_t>(stream)) != hipSuccess) return AP_ERR_HIP;
        for (int i = 0; i < count; ++i) {
            if (plain(items[i].h)) continue;
            ap_status s = ap_gemv(items[i].h, items[i].b, items[i].x_dev, items[i].y_dev, batch, stream);
            if (s != AP_OK) return s;
        }
        return AP_OK;
    }
    // Groups of items the tile kernel takes together: same bit-width, same class of row length; an item
    // whose handle carries a tuning override runs on its own.  Three passes over the list, no allocation.
    auto group_of = [](const ap_gemv_list_item &it, int *b, int *cls) {
        const ap_matrix *h = it.h;
        const bool plain = h->variant == AP_VARIANT_AUTO && h->waves_per_group == 0 && h->row_groups_per_wg < 0 &&
                           h->mfma_min_batch == 0;
        if (h->hdr.K % 256 != 0 || !plain) return false;
        *b = it.b;
        *cls = h->hdr.K >= 12288 ? 1 : 0;
        return true;
    };
    int members[AP_MAX_BITS + 1][2] = {};
    long long row_groups[AP_MAX_BITS + 1][2] = {};
    for (int i = 0; i < count; ++i) {
        int gb, gc;
        if (!group_of(items[i], &gb, &gc)) continue;
        ++members[gb][gc];
        row_groups[gb][gc] += padded_rows(items[i].h->hdr.M) / kRowsPerGroup;
    }
    auto together = [&](int gb, int gc) { return members[gb][gc] >= 2 && row_groups[gb][gc] >= 1024; };
    for (int gb = AP_MIN_BITS; gb <= AP_MAX_BITS; ++gb)
        for (int gc = 0; gc < 2; ++gc) {
            if (!together(gb, gc)) continue;
            ListArgs la;
            std::memset(&la, 0, sizeof(la));
            for (int i = 0; i < count; ++i) {
                int ib, ic;
                if (!group_of(items[i], &ib, &ic) || ib != gb || ic != gc) continue;
                fill_list_item(items[i].h, gb, items[i].x_dev, items[i].y_dev, &la.item[la.count++]);
                if (la.count == kMaxListItems) {
                    if (launch_matrix_tile_list(la, gb, batch, static_cast<hipStream_t>(stream)) != hipSuccess) return AP_ERR_HIP;
                    la.count = 0;
                }
            }
            if (la.count > 0 && launch_matrix_tile_list(la, gb, batch, static_cast<hipStream_t>(stream)) != hipSuccess)
                return AP_ERR_HIP;
        }
    for (int i = 0; i < count; ++i) {
        int ib, ic;
        if (group_of(items[i], &ib, &ic) && together(ib, ic)) continue;
        ap_status s = ap_gemv(items[i].h, items[i].b, items[i].x_dev, items[i].y_dev, batch, stream);
        if (s != AP_OK) return s;
    }
    return AP_OK;
}

extern "C" ap_status ap_gemv_multi(const ap_gemv_item *items, int count, int b, int batch, void *stream)
{
    if (!items || count < 1 || count > kMaxMulti) return AP_ERR_INVALID_ARG;
    if (batch < 1 || batch > AP_MAX_MULTI_BATCH) return AP_ERR_BATCH;
    if (batch == 1) { // any shapes: the list kernel, every item at bit-width b
        ListArgs la;
        std::memset(&la, 0, sizeof(la));
        la.count = count;
        for (int i = 0; i < count; ++i) {
            ap_status s = fill_list_item(items[i].h, b, items[i].x_dev, items[i].y_dev, &la.item[i]);
            if (s != AP_OK) return s;
        }
        return launch_gemv_list(la, 1, static_cast<hipStream_t>(stream)) == hipSuccess ? AP_OK : AP_ERR_HIP;
    }
    MultiArgs m;
    std::memset(&m, 0, sizeof(m));
    int total = 0;
    for (int i = 0; i < count; ++i) {
        GemvArgs a;
        ap_status s = fill_args(items[i].h, b, &a);
        if (s != AP_OK) return s;
        if (!items[i].x_dev || !items[i].y_dev) return AP_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(items[i].x_dev) % 16 || reinterpret_cast<uintptr_t>(items[i].y_dev) % 2)
            return AP_ERR_INVALID_ARG;
        if (i > 0 && a.K != m.K) return AP_ERR_SHAPE;
        m.K = a.K;
        m.slices[i] = a.slices;
        m.slice_bytes[i] = a.slice_bytes;
        m.lut[i] = a.lut;
        m.x[i] = static_cast<const uint16_t *>(items[i].x_dev);
        m.y[i] = static_cast<uint16_t *>(items[i].y_dev);
        m.M[i] = a.M;
        m.group_begin[i] = total;
        total += padded_rows(a.M) / kRowsPerGroup;
    }
    m.count = count;
    m.batch = batch;
    // The matrix-core kernel on tiles of 16 rows when the launch as a whole is large enough for it (the
    // rule of ap_gemv, applied to the sum of the row groups) or when the first handle asks for it
    // (AP_VARIANT_TILE).  Measured on the 7B projections (q,k,v: 3 x 4096x4096; gate,up: 2 x 11008x4096)
    // against the ALU kernel of this launch: batch 5..8 9.8 / 11.5 / 16.7 us against 17.7 / 19.7 / 23.7
    // (q,k,v; b = 3, 4, 8) and 15.0 / 19.0 / 28.4 against 27.7 / 31.2 / 35.9 (gate,up); batch 3..4 level
    // to 10 % faster.
    const int first_variant = items[0].h->variant;
    const bool tile = m.K % 256 == 0 &&
                      (first_variant == AP_VARIANT_TILE ||
                       (first_variant == AP_VARIANT_AUTO && ((batch >= 5 && total >= 1024) || (batch >= 3 && total >= 2048))));
    const hipError_t e = tile ? launch_matrix_tile_multi(m, b, static_cast<hipStream_t>(stream))
                              : launch_gemv_multi(m, b, total, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

extern "C" ap_status ap_dequantize(const ap_matrix *h, int b, void *w_dev, void *stream)
{
    GemvArgs a;
    ap_status s = fill_args(h, b, &a);
    if (s != AP_OK) return s;
    if (!w_dev || reinterpret_cast<uintptr_t>(w_dev) % 16) return AP_ERR_INVALID_ARG;
    a.y = static_cast<uint16_t *>(w_dev);
    return launch_dequantize(a, static_cast<hipStream_t>(stream)) == hipSuccess ? AP_OK : AP_ERR_HIP;
}

extern "C" ap_status ap_gemm_workspace_size(const ap_matrix *h, size_t *bytes)
{
    if (!handle_ok(h) || !bytes) return AP_ERR_INVALID_ARG;
    *bytes = (size_t)h->hdr.M * (size_t)h->hdr.K * 2;
    return AP_OK;
}

extern "C" ap_status ap_gemm(const ap_matrix *h, int b, const void *x_dev, void *y_dev, int batch,
                             void *work_dev, size_t work_bytes, void *stream)
{
    GemvArgs a;
    ap_status s = fill_args(h, b, &a);
    if (s != AP_OK) return s;
    if (!x_dev || !y_dev || !work_dev) return AP_ERR_INVALID_ARG;
    if (batch < 1 || batch > (1 << 20)) return AP_ERR_BATCH;
    if (reinterpret_cast<uintptr_t>(work_dev) % 16 || reinterpret_cast<uintptr_t>(x_dev) % 2 ||
        reinterpret_cast<uintptr_t>(y_dev) % 2)
        return AP_ERR_INVALID_ARG;
    if (work_bytes < (size_t)a.M * (size_t)a.K * 2) return AP_ERR_BUFFER_TOO_SMALL;
    a.y = static_cast<uint16_t *>(work_dev);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (launch_dequantize(a, st) != hipSuccess) return AP_ERR_HIP;
    return dense_gemm_f16(work_dev, x_dev, y_dev, a.M, a.K, batch, st) ? AP_OK : AP_ERR_HIP;
}

extern "C" ap_status ap_probe_read(const void *dev_buf, size_t bytes, void *stream)
{
    if (!dev_buf || bytes == 0 || bytes % 16384 || reinterpret_cast<uintptr_t>(dev_buf) % 16)
        return AP_ERR_INVALID_ARG;
    if (bytes / 16384 > 0x7fffffffu) return AP_ERR_INVALID_ARG;
    return launch_probe_read(dev_buf, bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? AP_OK
                                                                                              : AP_ERR_HIP;
}

extern "C" ap_status ap_probe_issue(int kind, int passes, void *stream)
{
    if (kind < 0 || kind >= AP_PROBE_ISSUE_KINDS || passes < 1 || passes > (1 << 20)) return AP_ERR_INVALID_ARG;
    return launch_probe_issue(kind, passes, static_cast<hipStream_t>(stream)) == hipSuccess ? AP_OK : AP_ERR_HIP;
}

extern "C" ap_status ap_matrix_info(const ap_matrix *h, int *M, int *K, int *n, unsigned *lut_mask)
{
    if (!handle_ok(h)) return AP_ERR_INVALID_ARG;
    if (M) *M = h->hdr.M;
    if (K) *K = h->hdr.K;
    if (n) *n = h->hdr.n;
    if (lut_mask) *lut_mask = h->hdr.lut_mask;
    return AP_OK;
}

extern "C" void ap_free(ap_matrix *h)
{
    if (!h) return;
    h->tag = 0;
    delete h;
}
