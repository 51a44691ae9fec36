// The host-side handle of a packed matrix (opaque to callers of the C-ABI).
#ifndef APGEMV_HANDLE_H
#define APGEMV_HANDLE_H

#include "layout.h"

struct ap_matrix {
    uint32_t tag;
    apgemv::BlobHeader hdr;
    uint8_t *dev;
    int waves_per_group;
    int row_groups_per_wg;
    int mfma_min_batch;
    int variant;
};

namespace apgemv {
constexpr uint32_t kHandleTag = 0x41504d58u;
inline bool handle_ok(const ap_matrix *h) { return h && h->tag == kHandleTag && h->dev; }
} // namespace apgemv

#endif
