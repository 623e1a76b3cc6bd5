// k-means index construction and online update (host sequencing + kernels).
#include "mp_ctx.h"
#include "mp_device.h"
#include "mp_internal.h"

namespace mp {

mp_status cluster_kv_impl(mp_ctx* ctx, const void*, const void*, int32_t, int32_t, int32_t, int32_t, uint64_t,
                          const int32_t*, const int32_t*, hipStream_t)
{
    return fail(ctx, MP_ESTATE, "mp_cluster_kv: not implemented yet");
}

mp_status update_clusters_impl(mp_ctx* ctx, const void*, const void*, int32_t, int32_t, int32_t, int32_t, int32_t,
                               uint64_t, const int32_t*, hipStream_t)
{
    return fail(ctx, MP_ESTATE, "mp_update_clusters: not implemented yet");
}

}  // namespace mp
