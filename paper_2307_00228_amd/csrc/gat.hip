// Attention-weighted gather (GAT reduce).  Not built yet: the entry reports ITB_ERR_UNSUPPORTED.
#include "common.h"

namespace itb {
int32_t gat_gather_impl(const itb_gather_desc *, int64_t, const int64_t *, const int32_t *, const itb_split *, const void *,
                        const float *, const float *, void *, int64_t, int64_t, void *, size_t *workspace_bytes, hipStream_t) {
    if (workspace_bytes) *workspace_bytes = 0;
    return ITB_ERR_UNSUPPORTED;
}
}  // namespace itb
