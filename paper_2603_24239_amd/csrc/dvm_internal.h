// Declarations shared by the host encoder (dvm_encode.cpp) and the device file (dvm_vm.hip).
#ifndef DVM_INTERNAL_H
#define DVM_INTERNAL_H

#include "../../include/dvm.h"

#ifdef __cplusplus
extern "C" {
#endif

// Record an error detail for dvm_last_error_detail() on this thread and return `status`.
int dvm_set_error(int status, const char *detail);
// HIP device the context was created for, or -1.
int dvm_ctx_device(const dvm_ctx *ctx);
// Planner inputs of the context (either pointer may be null).
void dvm_ctx_planner_get(const dvm_ctx *ctx, int *n_cu, int *overhead);
// Bound on the polls of a grid-wide synchronisation point (dvm_ctx_set_sync_limit).
int64_t dvm_ctx_sync_limit(const dvm_ctx *ctx);
// Implemented in the device file so that the encoder object stays free of HIP calls.
int dvm_ctx_query_device(int hip_device, int *n_cu);

#ifdef __cplusplus
}
#endif
#endif
