// Dual (k x k) form of the row update for rows with few stored entries.  Not built yet: every row
// takes the primal path.
#include "als_internal.h"

namespace als {

int dual_supported_max_k(int) { return 0; }

als_status launch_dual(als_ctx *ctx, const als_csr *, const als_table *, const float *, const als_params *,
                       als_table *, int64_t, int64_t, int, hipStream_t) {
    return fail(ctx, ALS_EINVAL, "dual path not available");
}

}  // namespace als
