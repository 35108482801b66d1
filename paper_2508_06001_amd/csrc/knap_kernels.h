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
                      void* dq, void* dk, void* dv, float* delta, float* lse2, unsigned* counters,
                      int grid_dkdv, int grid_dq, hipStream_t stream,
                      hipEvent_t ev_start, hipEvent_t ev_stop);

// Ulysses layout switch, local data movement; rows of U 16-byte units.
hipError_t launch_ulysses_heads(const void* src, void* dst, uint32_t T, uint32_t U, uint32_t g, bool pack,
                                int cus, hipStream_t stream);
hipError_t launch_ulysses_rows(const void* src, void* dst, const int32_t* row_map, uint32_t T, uint32_t U,
                               bool gather, int cus, hipStream_t stream);
// table: (n_seq + 1) g ints of scratch
hipError_t launch_ulysses_plan(const int32_t* cu, int n_seq, int g, int T, int32_t* table, int32_t* row_map,
                               hipStream_t stream);

// resident workgroups per compute unit of the persistent kernels
int fwd_workgroups_per_cu(int d);
int bwd_dkdv_workgroups_per_cu(int d);
int bwd_dq_workgroups_per_cu(int d);

}  // namespace knap
