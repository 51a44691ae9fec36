/*
 * apgemv - any-precision matrix-vector product for AMD MI355X (gfx950).
 *
 * One stored n-bit index per weight serves every b-bit model, 3 <= b <= n <= 8: a b-bit call
 * uses the b most significant bits of each index and looks them up in the output channel's own
 * table of 2^b binary16 centroids (Any-Precision LLM, Section 3.3 "Concept"; Section 4.1; the
 * engine overview of Section 5.2).  The device layout is bit-sliced, so a b-bit call reads b bits
 * per weight (Section 5.1, bitplane representation).
 *
 * Conventions: W is M x K, row = output channel; x is batch x K, y is batch x M, both row-major
 * binary16 (the paper writes the product as (1,K) x (M,K), Table 6).  All functions return an
 * ap_status; none throws, aborts or prints.  Every argument check happens before the first HIP
 * call of a function, so the error paths need no GPU.  "host" and "device" below say where a
 * pointer must point.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef APGEMV_H
#define APGEMV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ap_matrix ap_matrix; /* opaque host-side handle of one packed matrix */

typedef enum {
    AP_OK = 0,
    AP_ERR_INVALID_ARG = 1,      /* NULL pointer, misaligned buffer, bad handle */
    AP_ERR_SHAPE = 2,            /* M < 1, K < 32 or K not a multiple of 32, M or K beyond 2^24, more than
                                    2^32 weights (rows counted up to a multiple of 4) */
    AP_ERR_BITS = 3,             /* n outside 3..8, b outside 3..n, or no table given for b */
    AP_ERR_INDEX_RANGE = 4,      /* an index >= 2^n */
    AP_ERR_BUFFER_TOO_SMALL = 5, /* destination smaller than ap_packed_size */
    AP_ERR_BATCH = 6,            /* batch outside 1..16 (ap_gemv) or 1..8 (the multi and list calls) */
    AP_ERR_HIP = 7,              /* a HIP runtime call or kernel launch failed */
    AP_ERR_NO_MEMORY = 8         /* host memory (a handle, the pinned staging buffer) could not be allocated */
} ap_status;

#define AP_MIN_BITS 3
#define AP_MAX_BITS 8
#define AP_MAX_BATCH 16      /* ap_gemv */
#define AP_MAX_MULTI_BATCH 8 /* ap_gemv_multi */
#define AP_BLOB_ALIGN 256

/*
 * Bytes of the packed form of an M x K matrix with an n-bit parent and centroid tables for every
 * b whose bit is set in lut_mask (bit b <=> b-bit model supported, 3 <= b <= n; Section 3.3: only
 * the tables of the supported bit-widths are stored).  The packed form is position independent:
 * a 256-byte header, then n bit slices of ceil(M/4)*4*K/8 bytes each, most significant slice
 * first, then the tables, each region 256-byte aligned.
 */
ap_status ap_packed_size(int M, int K, int n, unsigned lut_mask, size_t *bytes);

/*
 * Host-only packing (no HIP call): split every n-bit index into bit slices in the device layout
 * and append the centroid tables (Section 5.1 bitplanes; Section 5.3 layout pre-processing).
 *   idx       host, M*K bytes row-major, every value < 2^n (else AP_ERR_INDEX_RANGE)
 *   luts[b]   host, for 3 <= b <= n: M * 2^b binary16 bit patterns, entry e of row i at
 *             [i*2^b + e]; NULL = b not supported.  luts[0..2] are ignored.  Tables need not be
 *             sorted.  At least one table must be given.
 *   blob      host, blob_bytes >= ap_packed_size(M, K, n, mask of non-NULL tables); written fully
 */
ap_status ap_pack_host(const uint8_t *idx, int M, int K, int n, const uint16_t *const luts[9],
                       void *blob, size_t blob_bytes);

/* Inverse of the index part of ap_pack_host: writes M*K index bytes (host) from a packed blob
 * (host).  Bit-exact round trip is part of the contract. */
ap_status ap_unpack_host(const void *blob, size_t blob_bytes, uint8_t *idx_out);

/* Reads table entry e (natural index) of row i for bit-width b back out of a packed blob (host):
 * binary16 bits.  Inside the blob the entries of a row are stored in the kernel's lookup order. */
ap_status ap_blob_lut_entry(const void *blob, size_t blob_bytes, int b, int row, int entry,
                            uint16_t *out);

/*
 * Byte range of the packed form that an ap_gemv call with bit-width b reads: the slice prefix
 * [slices_begin, slices_end) and the table [lut_begin, lut_end), as offsets into the blob.
 * The prefix of b is contained in the prefix of b+1 (a b-bit call loads only b bits per weight).
 */
ap_status ap_read_extent(int M, int K, int n, unsigned lut_mask, int b, size_t *slices_begin,
                         size_t *slices_end, size_t *lut_begin, size_t *lut_end);

/*
 * Pack on the host and upload into caller-owned device memory.
 *   dev_buf   device, dev_buf_bytes >= ap_packed_size(...), 256-byte aligned, must outlive the
 *             handle; the library never allocates device memory for model data
 *   stream    the upload is enqueued on it and has completed when the call returns
 *   out       receives the handle (host object; release with ap_free)
 * The host arrays may be released after return.  The packed form is staged in pinned host memory that
 * the library keeps and reuses for later ap_pack / ap_unpack calls (as large as the largest matrix
 * handled so far; calls are serialised on it); AP_ERR_NO_MEMORY if it cannot be had.
 */
ap_status ap_pack(const uint8_t *idx_host, int M, int K, int n, const uint16_t *const luts_host[9],
                  void *dev_buf, size_t dev_buf_bytes, void *stream, ap_matrix **out);

/* Adopt a blob that is already in device memory (e.g. a device-to-device copy of a packed
 * matrix).  Reads the 256-byte header back to the host to validate it. */
ap_status ap_attach(void *dev_buf, size_t dev_buf_bytes, void *stream, ap_matrix **out);

/* Download the slices and undo the packing: writes M*K index bytes to idx_host_out (host).
 * Synchronises `stream`. */
ap_status ap_unpack(const ap_matrix *h, uint8_t *idx_host_out, void *stream);

/*
 * y[t][i] = sum_j  C_b[i][ idx[i][j] >> (n-b) ] * x[t][j],   0 <= t < batch     (Section 5.2)
 *   h      packed matrix; b: 3 <= b <= n and a table for b was packed (else AP_ERR_BITS)
 *   x_dev  device, batch*K binary16 row-major, 16-byte aligned
 *   y_dev  device, batch*M binary16 row-major, 2-byte aligned; must not overlap x_dev or the blob
 *   batch  1..16 (the paper switches to a dequantise + dense GEMM path above about 16, Section 6.2).
 *          The kernels take up to 8 activation rows; batches 9..16 run as two passes on the stream, the
 *          first over rows 0..7, and cost what the two batches cost separately
 * Products are exact in binary32, accumulation is binary32, the result is rounded to binary16
 * (round to nearest even).  Asynchronous on `stream`; allocates nothing, synchronises nothing,
 * never repacks; the bit-width is chosen per call.  Results are deterministic (no atomics).
 */
ap_status ap_gemv(const ap_matrix *h, int b, const void *x_dev, void *y_dev, int batch,
                  void *stream);

/*
 * Kernel-selection overrides of one handle, for tests (to reach every kernel variant on small shapes)
 * and for A/B measurements; production callers set none.  ap_gemv chooses the kernel from (b, batch,
 * shape); an override replaces part of that choice.  Every variant meets the same tolerance, but the
 * bit-identity statements below (repeated calls, ap_gemv_multi) assume that the options of a handle
 * do not change between the calls compared.  Not thread-safe against concurrent calls on the handle.
 *   AP_OPT_WAVES_PER_GROUP    1..8 waves per group of 4 rows in the batch-1 kernels; 0 = from the shape
 *   AP_OPT_ROW_GROUPS_PER_WG  1..4 groups of 4 rows per workgroup (forces the row-group kernels);
 *                             -1 = from the shape
 *   AP_OPT_MFMA_MIN_BATCH     smallest batch sent to the one-row-per-lane matrix-core kernel (1..9,
 *                             9 = never); a negative value -m means m and also lifts its b >= 6 limit;
 *                             0 = default (3)
 *   AP_OPT_VARIANT            AP_VARIANT_AUTO; AP_VARIANT_NO_EXCHANGE = never the matrix-core kernel
 *                             with in-wave exchange; AP_VARIANT_EXCHANGE = that kernel whenever the
 *                             shape allows (batch >= 2, K % 128 == 0); AP_VARIANT_BANK_PER_LANE = at
 *                             batch 1, b >= 7: the kernel in which every lane looks up its own LDS
 *                             bank column (8 copies of each row's table) instead of the default;
 *                             AP_VARIANT_PAIR / AP_VARIANT_NO_PAIR = at batch 1: the kernel with two
 *                             groups of 4 rows per workgroup whenever every span has its own wave
 *                             (2048 < K <= 16384) / never (the default);
 *                             AP_VARIANT_TILE / AP_VARIANT_TILE2 = at batch >= 2, K % 256 == 0: the
 *                             matrix-core kernel that works on tiles of 16 rows, with one / two
 *                             tiles per workgroup
 * AP_ERR_INVALID_ARG for an unknown option or a value outside its range.
 */
typedef enum {
    AP_OPT_WAVES_PER_GROUP = 0,
    AP_OPT_ROW_GROUPS_PER_WG = 1,
    AP_OPT_MFMA_MIN_BATCH = 2,
    AP_OPT_VARIANT = 3
} ap_option;
#define AP_VARIANT_AUTO 0
#define AP_VARIANT_NO_EXCHANGE 1
#define AP_VARIANT_EXCHANGE 3
#define AP_VARIANT_BANK_PER_LANE 5
#define AP_VARIANT_PAIR 7
#define AP_VARIANT_NO_PAIR 8
#define AP_VARIANT_TILE 9
#define AP_VARIANT_TILE2 10
ap_status ap_set_option(ap_matrix *h, int option, int value);

/*
 * Several GEMVs of the same bit-width in ONE launch: y_i = W_i,b * x_i for i < count (1..8), e.g. the
 * q/k/v or the gate/up projections of a decoder layer (Section 6.3 measures whole-model decoding,
 * where the per-launch cost of 224 small GEMVs per token matters).  Every matrix needs a table for b;
 * M may differ; at batch >= 2 all matrices must have the same K (AP_ERR_SHAPE otherwise), at batch 1
 * any shapes go together; x_dev/y_dev may be shared or distinct per item (outputs must not overlap).
 * At batch 1 and 2 each output is bit-identical to the one ap_gemv produces with default options (same
 * kernel per row group); at larger batches ap_gemv may pick another variant with a different
 * summation order, and both meet the same tolerance.  The kernel is chosen from the launch as a whole
 * (b, batch, K, the sum of the rows); of the per-handle options only AP_OPT_VARIANT of the FIRST item's
 * handle is looked at (AP_VARIANT_TILE forces the matrix-core kernel on tiles when K % 256 == 0, any
 * other value than AP_VARIANT_AUTO keeps the launch on the ALU kernel).  batch 1..8 here.  Same argument
 * rules and error codes as ap_gemv.
 */
typedef struct {
    const ap_matrix *h;
    const void *x_dev; /* batch*K binary16 */
    void *y_dev;       /* batch*M_i binary16 */
} ap_gemv_item;
ap_status ap_gemv_multi(const ap_gemv_item *items, int count, int b, int batch, void *stream);

/*
 * A work list of batch-1 products, each with its OWN bit-width, in as few launches as possible (one per
 * 32 items): y_i = W_i,b_i * x_i.  This is the call for a decode step at per-layer mixed precision
 * (Section 3.3: the bit-width is chosen at run time, per query; Section 6.3: end-to-end decoding is
 * hundreds of small products per token): matrices of any shapes and bit-widths share a launch, so the
 * per-launch start-up is paid once per list instead of once per matrix.
 *   items[i].h      packed matrix;  items[i].b  its bit-width for this call (a table must be packed)
 *   items[i].x_dev  device, K_i binary16, 16-byte aligned;  items[i].y_dev  device, M_i binary16
 * count >= 1.  Outputs must not overlap each other, the inputs or the blobs; no item may depend on
 * another item's output (all run concurrently).  Every item is checked before anything is enqueued;
 * the status is that of the first bad item.  Each output is bit-identical to ap_gemv(h, b, x, y, 1)
 * with default options.  Asynchronous on `stream`, allocates nothing, capturable in a graph.
 */
typedef struct {
    const ap_matrix *h;
    int b;
    const void *x_dev;
    void *y_dev;
} ap_gemv_list_item;
ap_status ap_gemv_list(const ap_gemv_list_item *items, int count, void *stream);

/*
 * The same work list for `batch` activation rows per item (1 <= batch <= 8): y_i (batch x M_i) =
 * x_i (batch x K_i) * W_i,b_i^T, the decode step of `batch` queries that run at the same precision
 * (Section 6.2 measures the kernel up to batch 8).  batch 1 is ap_gemv_list.  At batch 2 the items go into
 * list launches of the kernel that single calls use at batch 1 and 2 (any shapes and bit-widths together, up
 * to 32 per launch; bit-identical to separate ap_gemv calls).  At batch >= 3 the items
 * that the matrix-core kernel on tiles of 16 rows can take (K_i % 256 == 0) are launched together per
 * bit-width and class of row length, up to 32 per launch, whenever such a group has at least 1024 row
 * groups in total (the size rule of ap_gemv applied to the launch); every other item runs as its own
 * ap_gemv call on the same stream.  Outputs meet the tolerance of ap_gemv; an item that runs on the tile
 * kernel is bit-identical to ap_gemv on that kernel (AP_VARIANT_TILE) when every row of its launch has
 * at least 2048 columns (shorter rows lower the number of waves per tile of the launch, which changes the
 * order of the final sums).  Same argument rules as
 * ap_gemv_list; x_dev of an item holds batch * K_i, y_dev batch * M_i values.
 */
ap_status ap_gemv_list_batch(const ap_gemv_list_item *items, int count, int batch, void *stream);

/*
 * Dense binary16 weights of the b-bit model: w_dev[i*K + j] = C_b[i][ idx[i][j] >> (n-b) ], bit for
 * bit the table entries (Section 6.2, "Matrix-Matrix Multiplication Performance": for large batches
 * the engine dequantises with a separate kernel and uses a dense FP16 GEMM).
 *   w_dev   device, M*K binary16 row-major, 16-byte aligned, caller-owned
 * Asynchronous on `stream`; allocates nothing.
 */
ap_status ap_dequantize(const ap_matrix *h, int b, void *w_dev, void *stream);

/*
 * y = x * W_b^T for any batch >= 1 through the dequantise + dense GEMM path (the paper's route for
 * batch above ~16): ap_dequantize into work_dev, then one FP16 GEMM with binary32 accumulation
 * from rocBLAS, which is loaded on first use (AP_ERR_HIP if it cannot be loaded or fails).
 *   x_dev     device, batch*K binary16 row-major;  y_dev  device, batch*M binary16 row-major
 *   work_dev  device, >= ap_gemm_workspace_size bytes (M*K*2), 16-byte aligned, caller-owned
 * The first call on a process creates the rocBLAS handle (that call allocates and is not
 * capturable in a graph); later calls only enqueue work on `stream`.
 */
ap_status ap_gemm_workspace_size(const ap_matrix *h, size_t *bytes);
ap_status ap_gemm(const ap_matrix *h, int b, const void *x_dev, void *y_dev, int batch,
                  void *work_dev, size_t work_bytes, void *stream);

/*
 * ap_gemm for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same result contract as ap_gemm (binary32 accumulation,
 * binary16 output, the tolerance of ap_gemv), but the call allocates nothing and calls no library that
 * might: the dequantised weights go to a device array built into this library, AP_GEMM_STATIC_MAX_BYTES
 * large (each GPU the library runs on holds its own copy until the process ends), and the product is
 * computed by a kernel of this library.  The array's device address is looked up once per device, by
 * ap_pack / ap_attach or else by the first call here.
 *   x_dev   device, batch*K binary16 row-major, 16-byte aligned;  y_dev  device, batch*M binary16
 *   AP_ERR_BUFFER_TOO_SMALL if M*K*2 > AP_GEMM_STATIC_MAX_BYTES (use ap_gemm with your own workspace)
 * All calls on one GPU share the one array: calls that may overlap in time on the same GPU (different
 * streams, or threads) race on it and must be serialised by the caller.  The array keeps the last
 * call's weights; every call rewrites all it reads, so nothing needs clearing.
 */
#define AP_GEMM_STATIC_MAX_BYTES (32u << 20)
ap_status ap_gemm_static(const ap_matrix *h, int b, const void *x_dev, void *y_dev, int batch,
                         void *stream);

/*
 * Host-only any-precision quantiser (no HIP call): incremental upscaling of Section 4.  Every output
 * channel (row of w) is clustered on its own: a seed model of n_seed bits from a weighted 1-D k-means
 * (weights = sens, the per-weight sensitivities; NULL = all ones), then for b = n_seed..n-1 every
 * cluster is divided in two by a weighted 2-means and the new bit is appended at the end of the index.
 *   w, sens    host, M*K binary32 row-major
 *   idx_out    host, M*K bytes: the n-bit parent indices (idx >> (n-b) is the b-bit model's index)
 *   luts_out[b] host, for n_seed <= b <= n: M * 2^b binary16 bit patterns (NULL = not wanted)
 *   iters      Lloyd rounds per clustering (>= 1; 20 is plenty for one-dimensional data)
 * The outputs are what ap_pack takes.  AP_ERR_BITS unless 1 <= n_seed <= n <= 8.
 */
ap_status ap_quantize(const float *w, const float *sens, int M, int K, int n_seed, int n, int iters,
                      uint8_t *idx_out, uint16_t *const luts_out[9]);

/*
 * Measurement aid, not part of the method: reads `bytes` (a multiple of 16384) of device memory
 * with the same instruction and access shape as the GEMV's slice loads (non-temporal 16-byte
 * loads, 1 KB contiguous per wave) and discards them.  Profiling counters of HBM traffic are
 * calibrated against this launch, whose byte count is known.  Asynchronous on `stream`.
 */
ap_status ap_probe_read(const void *dev_buf, size_t bytes, void *stream);

/*
 * Measurement aid, not part of the method: launches 2048 workgroups of 256 threads (8 resident waves
 * per SIMD) in which every wave runs `passes` (1 .. 2^20) passes of one fixed group of independent
 * instructions, so that the time of the launch divided by the instructions per compute unit is the
 * issue rate of that kind on this device.  The kinds are the instructions the dequantising kernels are
 * made of; the ceilings they set (an LDS read costs a SIMD about as much issue time as a vector
 * instruction, and the two overlap only partly) are what bounds those kernels before HBM does.
 *   kind 0  8 ds_read_b32, every lane its own bank     kind 1  8 ds_read_b32 with 2-way bank conflicts
 *   kind 2  8 ds_bpermute_b32                          kind 3  4 ds_read_b128
 *   kind 4  32 v_perm_b32                              kind 5  kind 0 and kind 4 together
 *   kind 6  kind 2 and kind 4 together
 * Uses no device memory beyond its own LDS; asynchronous on `stream`; AP_ERR_INVALID_ARG for another
 * kind or pass count.
 */
#define AP_PROBE_ISSUE_KINDS 7
ap_status ap_probe_issue(int kind, int passes, void *stream);

/* Shape and supported bit-widths of a handle; any output pointer may be NULL. */
ap_status ap_matrix_info(const ap_matrix *h, int *M, int *K, int *n, unsigned *lut_mask);

/* Releases the host handle only; the device buffer stays with the caller. NULL is allowed.  A handle
 * must not be passed to any call after ap_free (the checks of a handle cannot detect that). */
void ap_free(ap_matrix *h);

/* Static, never NULL. */
const char *ap_strerror(ap_status s);

#ifdef __cplusplus
}
#endif
#endif /* APGEMV_H */
