// bf16 matrix-core path (placeholder until the kernels land).
#include "fs_internal.h"
namespace fs {
fs_status bf16_lse(Ctx *c, const Prepared *, const Side *, const Side *, double, int *)
{
    return fail(c, FS_ERR_UNSUPPORTED, "bf16 mode is not built yet");
}
}  // namespace fs
