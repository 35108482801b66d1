// Internal launch interface between the C-ABI layer and the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace knap {

hipError_t launch_fwd(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq,
                      int H, int d, float scale, bool causal, void* out, float* lse, unsigned* counters,
                      int grid, hipStream_t stream);

// Device address (on the current device) of the forward kernel's work-queue counters:
// fwd_queue_slots() sets of 8, one set per launch in flight; nullptr on failure.
unsigned* fwd_queue_base();
int fwd_queue_slots();

hipError_t launch_bwd(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq, int H, int d,
                      float scale, bool causal, const void* out, const float* lse, const void* dout,
                      void* dq, void* dk, void* dv, float* delta, unsigned* counters,
                      int grid_dkdv, int grid_dq, hipStream_t stream,
                      hipEvent_t ev_start, hipEvent_t ev_stop);

// resident workgroups per compute unit of the persistent kernels
int fwd_workgroups_per_cu(int d);
int bwd_dkdv_workgroups_per_cu(int d);
int bwd_dq_workgroups_per_cu(int d);

}  // namespace knap
