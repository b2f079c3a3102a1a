// Calls shared by the module and the pipeline that are not part of the C boundary.
#pragma once
#include "../../include/ddg.h"
#include <hip/hip_runtime_api.h>

extern "C" {
// While set, the module's calls advance their host-side state (iteration counter, ring
// position) and validate arguments but enqueue nothing: the pipeline replays a captured
// graph of the same call instead.
void ddg_internal_skip_launches(ddg_module* m, bool skip);
// The update reads its step size from this device float instead of the call argument.
void ddg_internal_lr_from(ddg_module* m, const float* lr_dev);
bool ddg_internal_profiling(const ddg_module* m);
// A pipeline orders the module's two streams itself (events around graph launches); the module
// then records and waits on nothing.
void ddg_internal_external_sync(ddg_module* m, bool on);
// The streams ddg_forward and ddg_backward_delayed/ddg_update enqueue on (equal unless the
// module runs its forward pass on a stream of its own).
void ddg_internal_streams(ddg_module* m, hipStream_t* fwd, hipStream_t* bwd);
// Sets the message ddg_last_error returns on this thread.
void ddg_internal_set_error(const char* msg);
}
