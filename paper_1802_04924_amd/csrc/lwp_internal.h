// Access to the opaque context for the translation units that implement parts of the C ABI.
#pragma once
#include <hip/hip_runtime.h>

#include "lwp.h"

namespace lwp {
hipStream_t ctx_stream(lwp_ctx* ctx);
// Clears the last error and makes the context's device current.
lwp_status ctx_enter(lwp_ctx* ctx);
// Records `why` as the context's last error and returns `s`.
lwp_status ctx_fail(lwp_ctx* ctx, lwp_status s, const char* why);
}  // namespace lwp
