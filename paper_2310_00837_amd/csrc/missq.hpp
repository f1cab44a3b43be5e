// The asynchronous miss queue: what the rest of the host runtime needs to know of it.
#pragma once
#include "context.hpp"

namespace helios {

// Called by a batch (directly launched or being recorded) right after its cache lookup, when a
// queue is attached to the context: enqueues the submission kernel for the batch's miss list.
// For a directly launched batch it also opens the queue's next round; a recorded batch reads the
// round on the device, and missq_open_round opens it at every launch of the recording.
int missq_submit_from_batch(helios_ctx* c, const int32_t* miss_pos, const int32_t* miss_slot, Count n_miss,
                            int64_t n_miss_max, int64_t out_rows);
// A recorded batch about to be launched: *round_out is the number of the queue's next round, which the
// batch's BatchVars carry; missq_commit_round opens that round once the launch has succeeded (a launch
// that failed leaves the queue as it was).
int missq_next_round(helios_ctx* c, helios_missq* q, uint32_t* round_out);
void missq_commit_round(helios_missq* q, uint32_t round);
// True if q is still usable with the context's current cache.
bool missq_matches_cache(const helios_ctx* c, const helios_missq* q);

}  // namespace helios
