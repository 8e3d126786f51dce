// Optional per-stage GPU timing with HIP events on the caller's stream.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace dynb {

// Stage ids reported for moe_forward; dynbatch_execute reports its launch-group index instead.
enum { ST_GATE = 0, ST_TOPK = 1, ST_SORT = 2, ST_PERMUTE = 3, ST_FFN1 = 4, ST_FFN2 = 5, ST_COMBINE = 6 };

bool timing_on();
// True when only whole kernel sequences are bracketed (mode 2) instead of every launch group.
bool timing_coarse();
// Tag of the mark that closes a call's set-up work (weight packing, leaf copies).
enum { ST_SETUP = -2 };
// Starts a new timed call: drops the marks of the previous one and records the opening event.
void timing_begin(hipStream_t st);
// Records an event that closes a stage: everything enqueued since the previous mark belongs to it.
void timing_mark(hipStream_t st, int32_t tag, int32_t units);

}  // namespace dynb
