// Optional per-launch timing with HIP events (diagnostic; off unless started).
#pragma once
#include <hip/hip_runtime.h>

namespace fhpc {

// True while fhpc_profile_start has armed the hook (launchers format their record's name only then).
bool prof_on();
// Records a start event on `s` if profiling is on; returns a slot (or -1).
int prof_begin(const char* name, double flops, double bytes, hipStream_t s);
// Records the matching stop event.
void prof_end(int slot, hipStream_t s);

}  // namespace fhpc
