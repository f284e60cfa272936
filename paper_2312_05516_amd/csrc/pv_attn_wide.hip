// Matrix-core attention kernel for work items with many query rows (placeholder until the
// LDS-staged kernel lands: the plan sends every item to the narrow kernel).
#include "pv_device.h"

namespace pv {

hipError_t launch_attn_wide(const pv_plan *plan, const void *, const void *, const void *,
                            const int32_t *, float, void *, float *, float *, hipStream_t)
{
    return plan->wide.empty() ? hipSuccess : hipErrorNotSupported;
}

}  // namespace pv
