// What the host-side translation units of the library share beyond the public header.
#pragma once
#include <hip/hip_runtime.h>

namespace imm {

// Text that imm_last_error() returns on the calling thread.
void set_last_error(const char* text);
// Records "<what>: <HIP error string>" and returns IMM_E_HIP.
int fail_hip(hipError_t e, const char* what);

// Looks up, once per device, where that device keeps the library's statically allocated working
// memory (static_eval.hip).  The device must be the calling thread's current one.  Called when a
// context is created, so that later calls that must not touch the runtime's symbol tables (under
// stream capture, for one) find the address ready.  Returns IMM_OK or IMM_E_HIP.
int static_scratch_prepare(int device);

}  // namespace imm
