// Streamed schedule (operands in pinned host memory): not built yet.
#include "gp_internal.h"

namespace gp {

gp_status propagate_streamed(const gp_plan*, const void*, int64_t, int32_t, gp_dtype, gp_agg, int32_t, void*, int64_t)
{
    return fail(GP_ERR_UNSUPPORTED, "pinned-host operands (streamed schedule) are not supported yet");
}

}  // namespace gp
