// Internal interface between the host packer and the C-ABI entry points.
#ifndef APGEMV_PACK_H
#define APGEMV_PACK_H

#include "../../include/apgemv.h"
#include "layout.h"

namespace apgemv {

ap_status check_shape(int M, int K, int n);
ap_status check_mask(int n, unsigned lut_mask);
ap_status check_index_range(const uint8_t *idx, int M, int K, int n); // every index < 2^n
ap_status make_header(int M, int K, int n, unsigned lut_mask, BlobHeader *h);
ap_status validate_header(const BlobHeader *h, size_t blob_bytes);
void pack_slices(const uint8_t *idx, const BlobHeader &h, uint8_t *blob);
void unpack_slices(const uint8_t *blob, const BlobHeader &h, uint8_t *idx);

} // namespace apgemv
#endif
