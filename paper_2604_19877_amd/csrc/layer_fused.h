// The fused per-layer launch of a placement stack (see layer_fused.hip).
#pragma once
#include "attn_device.h"
#include "delta_step_device.h"

namespace sa {

// Partial results of a layer's attention calls that still wait to be merged into the layer's output: n_fa and
// n_swa count the (request, KV head, query row) items of each call (0: nothing to merge).
struct PendingMerge {
  AttnParams fa, swa;
  int n_fa = 0, n_swa = 0;
};

// Enqueues one kernel that first merges what `pending` holds (the partial results of an earlier layer) and then
// runs the prepared launches of this layer (any of them may have rows == 0).  recurrent_order: device list of the
// kda.rows + gdn.rows requests of both recurrent launches in the order their tiles are to be visited, a GDN request r
// stored as ~r (used by the one-token launch, which runs one tile body for both mixers; may be null: KDA's list, then GDN's).  On return `pending` describes this
// layer's own partial results, to be merged by the next layer's launch or by layer_merge_flush: the buffers it
// points to must not be written before that.  All four launches must be calls of at most 4 tokens at 128x128 states
// and at most 16 query rows per KV head.
sa_status layer_fused_launch(const AttnLaunch& fa, const AttnLaunch& swa, const DeltaLaunch& kda, const DeltaLaunch& gdn,
                             const int32_t* recurrent_order, PendingMerge* pending, void* stream);

// Merges what `pending` holds in a launch of its own (no-op when empty) and empties it.
sa_status layer_merge_flush(PendingMerge* pending, void* stream);

}  // namespace sa
