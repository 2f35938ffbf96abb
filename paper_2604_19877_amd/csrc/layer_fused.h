// The fused per-layer launch of a placement stack (see layer_fused.hip).
#pragma once
#include "attn_device.h"
#include "delta_step_device.h"

namespace sa {

// Enqueues one kernel that runs the prepared launches of a layer (any of them may have rows == 0) and, if an
// attention call has several page ranges, one merge kernel.  All four must be single-token decode calls
// (T == 1) at 128x128 states and at most 16 query rows per KV head.
sa_status layer_fused_launch(const AttnLaunch& fa, const AttnLaunch& swa, const DeltaLaunch& kda, const DeltaLaunch& gdn,
                             void* stream);

}  // namespace sa
