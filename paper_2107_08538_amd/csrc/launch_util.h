// Internal helpers shared by the kernel translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>

// Record `what: <hip error text>` as the calling thread's last error.
void mgb_internal_set_error(const char* what, hipError_t e);
void mgb_internal_set_error_text(const char* text);

// Turn the launch status of the kernels just enqueued into an ABI status code.
static inline int mgb_check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return 0;   // MGB_OK
  mgb_internal_set_error(what, e);
  return -6;                       // MGB_E_BACKEND
}

// Scheduler facts the other translation units need (the struct itself is private to sched.cpp).
struct mgb_sched;
unsigned mgb_internal_backend(const mgb_sched* s);   // MGB_BACKEND_*
int mgb_internal_device(const mgb_sched* s);         // HIP device ordinal
// Profiling aid: an empty kernel on `stream` whose grid size names the partition (see cu_trace.hip).
int mgb_internal_tag_partition(hipStream_t stream, uint32_t first_granule, uint32_t n_granules);
