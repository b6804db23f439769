// fp64 matrix-core path (placeholder until the kernels land).
#include "fs_internal.h"
namespace fs {
fs_status f64_lse(Ctx *c, const Prepared *, const Side *, const Side *, double, int *)
{
    return fail(c, FS_ERR_UNSUPPORTED, "d > 16 in fp32 mode is not built yet");
}
size_t f64_apply_ws(const Ctx *, int64_t, int64_t, int64_t, int64_t) { return 0; }
fs_status f64_apply(Ctx *c, const Prepared *, const Side *, const Side *, double, const float *, int64_t, int64_t,
                    float *, int64_t, float *)
{
    return fail(c, FS_ERR_UNSUPPORTED, "d > 16 in fp32 mode is not built yet");
}
}  // namespace fs
