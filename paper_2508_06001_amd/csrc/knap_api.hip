// C-ABI entry points of libknapattn: argument checks, workspace carving and
// launches.  Nothing here allocates, frees or synchronises.
#include "knapattn.h"
#include "knapattn_bench.h"
#include "knap_kernels.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>

// Scratch of knap_varlen_attn_bwd_noalloc: the per-row dot products of dout and out and the base-2
// log-sum-exp (fp32, (H, T) each) and, in the last 256 bytes, the work-queue counters of the dQ kernel.  Part of the library's device image:
// every GPU the library runs on holds its own copy until the process ends.  Host code never uses this
// name as an address; it uses the pointer hipGetSymbolAddress returned on that device (DeviceInfo::scratch).
static __device__ __align__(256) unsigned char scratch[2 * KNAP_NOALLOC_MAX_ROWS * sizeof(float) + 256];

namespace {

thread_local int g_last_hip_error = 0;
thread_local hipEvent_t g_prof_start = nullptr;
thread_local hipEvent_t g_prof_stop = nullptr;

struct DeviceInfo {
  int cus = 0;
  int fwd_wg[2] = {0, 0};   // workgroups per CU, index 0: d = 64, 1: d = 128
  int dkdv_wg[2] = {0, 0};
  int dq_wg[2] = {0, 0};
  unsigned* fwd_queue = nullptr;   // this device's copy of the forward work-queue counters
  unsigned char* scratch = nullptr;   // this device's copy of `scratch`
};

// Counter sets of the forward's work queue: the lower half is handed out in rotation to eager launches,
// the upper half to launches recorded under stream capture.  A captured launch keeps its set for every
// replay of its graph, so it must never be one that eager launches rotate through.
std::atomic<unsigned> g_fwd_launches{0};
std::atomic<unsigned> g_fwd_captured{0};

constexpr int kMaxDevices = 64;

void fill_device_info(DeviceInfo& di, int dev) {
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    return;
  }
  di.fwd_wg[0] = knap::fwd_workgroups_per_cu(64);
  di.fwd_wg[1] = knap::fwd_workgroups_per_cu(128);
  di.dkdv_wg[0] = knap::bwd_dkdv_workgroups_per_cu(64);
  di.dkdv_wg[1] = knap::bwd_dkdv_workgroups_per_cu(128);
  di.dq_wg[0] = knap::bwd_dq_workgroups_per_cu(64);
  di.dq_wg[1] = knap::bwd_dq_workgroups_per_cu(128);
  di.fwd_queue = knap::fwd_queue_base();
  if (!di.fwd_queue) return;
  void* p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
    (void)hipGetLastError();
    return;
  }
  di.scratch = static_cast<unsigned char*>(p);
  di.cus = cus;     // last: marks the entry as complete
}

// per-device launch geometry and device-image addresses, looked up once per device with that
// device current (occupancy and symbol queries do not allocate); nullptr if the lookup failed
DeviceInfo* device_info() {
  static DeviceInfo info[kMaxDevices];
  static std::once_flag once[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
  std::call_once(once[dev], fill_device_info, std::ref(info[dev]), dev);
  return info[dev].cus > 0 ? &info[dev] : nullptr;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_common(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq, int H, int d,
                 float scale) {
  if (n_seq < 0 || H <= 0 || (d != 64 && d != 128)) return KNAP_ERR_INVALID_ARG;
  if (!(scale > 0.f) || !(scale < 3.0e38f)) return KNAP_ERR_INVALID_ARG;   // positive and finite
  if (n_seq > KNAP_MAX_SEQS) return KNAP_ERR_TOO_MANY_SEQS;
  if (n_seq == 0) return KNAP_OK;
  if (!q || !k || !v || !cu) return KNAP_ERR_INVALID_ARG;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(cu, 4)) return KNAP_ERR_INVALID_ARG;
  return KNAP_OK;
}

int fwd_impl(const void* q, const void* k, const void* v, const int32_t* cu_seqlens, int n_seq,
             int H, int d, float scale, bool causal, void* out, float* lse, void* stream) {
  const int rc = check_common(q, k, v, cu_seqlens, n_seq, H, d, scale);
  if (rc != KNAP_OK) return rc;
  if (n_seq == 0) return KNAP_OK;
  if (!out || !lse || !aligned(out, 16) || !aligned(lse, 4)) return KNAP_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return KNAP_ERR_INVALID_ARG;
  DeviceInfo* di = device_info();
  if (!di) return KNAP_ERR_LAUNCH_FAILED;
  const int grid = di->cus * di->fwd_wg[d == 128];
  const unsigned half = (unsigned)knap::fwd_queue_slots() / 2u;
  hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(static_cast<hipStream_t>(stream), &capture) != hipSuccess) {
    (void)hipGetLastError();
    capture = hipStreamCaptureStatusNone;
  }
  const unsigned slot = capture == hipStreamCaptureStatusNone ? g_fwd_launches.fetch_add(1u) % half
                                                              : half + g_fwd_captured.fetch_add(1u) % half;
  unsigned* counters = di->fwd_queue + 8u * slot;
  const hipError_t e = knap::launch_fwd(q, k, v, cu_seqlens, n_seq, H, d, scale, causal, out, lse, counters,
                                        grid, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) { g_last_hip_error = static_cast<int>(e); return KNAP_ERR_LAUNCH_FAILED; }
  return KNAP_OK;
}

int bwd_impl(const void* q, const void* k, const void* v, const int32_t* cu_seqlens, int n_seq,
             int H, int d, float scale, bool causal,
             const void* out, const float* lse, const void* dout, void* dq, void* dk, void* dv,
             int64_t total_tokens, void* workspace, size_t workspace_bytes, bool own_scratch, void* stream);

}  // namespace

extern "C" {

int knap_varlen_attn_fwd(const void* q, const void* k, const void* v,
                         const int32_t* cu_seqlens, int n_seq,
                         int H, int d, float scale,
                         void* out, float* lse, void* stream) {
  return fwd_impl(q, k, v, cu_seqlens, n_seq, H, d, scale, false, out, lse, stream);
}

int knap_varlen_attn_causal_fwd(const void* q, const void* k, const void* v,
                                const int32_t* cu_seqlens, int n_seq,
                                int H, int d, float scale,
                                void* out, float* lse, void* stream) {
  return fwd_impl(q, k, v, cu_seqlens, n_seq, H, d, scale, true, out, lse, stream);
}

size_t knap_varlen_attn_bwd_workspace_bytes(int64_t total_tokens, int n_seq, int H, int d) {
  (void)n_seq;
  if (total_tokens <= 0 || H <= 0 || d <= 0) return 0;
  // delta and the base-2 log-sum-exp, fp32 (H, T) each, then 256 bytes of work-queue counters
  return 2 * round_up(static_cast<size_t>(total_tokens) * H * sizeof(float), 256) + 256;
}

int knap_varlen_attn_bwd(const void* q, const void* k, const void* v,
                         const int32_t* cu_seqlens, int n_seq,
                         int H, int d, float scale,
                         const void* out, const float* lse, const void* dout,
                         void* dq, void* dk, void* dv,
                         int64_t total_tokens,
                         void* workspace, size_t workspace_bytes, void* stream) {
  return bwd_impl(q, k, v, cu_seqlens, n_seq, H, d, scale, false, out, lse, dout, dq, dk, dv, total_tokens,
                  workspace, workspace_bytes, false, stream);
}

int knap_varlen_attn_bwd_noalloc(const void* q, const void* k, const void* v,
                                 const int32_t* cu_seqlens, int n_seq,
                                 int H, int d, float scale,
                                 const void* out, const float* lse, const void* dout,
                                 void* dq, void* dk, void* dv,
                                 int64_t total_tokens, void* stream) {
  return bwd_impl(q, k, v, cu_seqlens, n_seq, H, d, scale, false, out, lse, dout, dq, dk, dv, total_tokens,
                  nullptr, 0, true, stream);
}

int knap_varlen_attn_causal_bwd(const void* q, const void* k, const void* v,
                                const int32_t* cu_seqlens, int n_seq,
                                int H, int d, float scale,
                                const void* out, const float* lse, const void* dout,
                                void* dq, void* dk, void* dv,
                                int64_t total_tokens,
                                void* workspace, size_t workspace_bytes, void* stream) {
  return bwd_impl(q, k, v, cu_seqlens, n_seq, H, d, scale, true, out, lse, dout, dq, dk, dv, total_tokens,
                  workspace, workspace_bytes, false, stream);
}

}  // extern "C"

namespace {

int bwd_impl(const void* q, const void* k, const void* v, const int32_t* cu_seqlens, int n_seq,
             int H, int d, float scale, bool causal,
             const void* out, const float* lse, const void* dout, void* dq, void* dk, void* dv,
             int64_t total_tokens, void* workspace, size_t workspace_bytes, bool own_scratch, void* stream) {
  const int rc = check_common(q, k, v, cu_seqlens, n_seq, H, d, scale);
  if (rc != KNAP_OK) return rc;
  if (total_tokens < 0 || total_tokens > INT32_MAX) return KNAP_ERR_INVALID_ARG;
  // the library's own scratch holds one float per (row, head): larger bags are refused, whatever else is wrong
  if (own_scratch && total_tokens * (int64_t)H > (int64_t)KNAP_NOALLOC_MAX_ROWS) return KNAP_ERR_SCRATCH_TOO_SMALL;
  if (n_seq == 0 || total_tokens == 0) return KNAP_OK;
  if (!out || !lse || !dout || !dq || !dk || !dv) return KNAP_ERR_INVALID_ARG;
  if (!aligned(out, 16) || !aligned(dout, 16) || !aligned(dq, 16) || !aligned(dk, 16) || !aligned(dv, 16) ||
      !aligned(lse, 4))
    return KNAP_ERR_INVALID_ARG;
  if (dq == dk || dq == dv || dk == dv || dq == q || dk == k || dv == v) return KNAP_ERR_INVALID_ARG;
  const size_t need = knap_varlen_attn_bwd_workspace_bytes(total_tokens, n_seq, H, d);
  if (!own_scratch) {
    if (!workspace || !aligned(workspace, 256)) return KNAP_ERR_INVALID_ARG;
    if (workspace_bytes < need) return KNAP_ERR_WORKSPACE_TOO_SMALL;
  }
  DeviceInfo* di = device_info();
  if (!di) return KNAP_ERR_LAUNCH_FAILED;
  if (own_scratch) workspace = di->scratch;     // carved exactly as a caller's workspace; need <= sizeof(scratch)

  float* delta = static_cast<float*>(workspace);
  float* lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + (need - 256) / 2);
  unsigned* counters = reinterpret_cast<unsigned*>(static_cast<char*>(workspace) + need - 256);
  const int grid_dkdv = di->cus * di->dkdv_wg[d == 128];
  const int grid_dq = di->cus * di->dq_wg[d == 128];
  const hipError_t e = knap::launch_bwd(q, k, v, cu_seqlens, n_seq, H, d, scale, causal, out, lse, dout,
                                        dq, dk, dv, delta, lse2, counters, grid_dkdv, grid_dq,
                                        static_cast<hipStream_t>(stream), g_prof_start, g_prof_stop);
  if (e != hipSuccess) { g_last_hip_error = static_cast<int>(e); return KNAP_ERR_LAUNCH_FAILED; }
  return KNAP_OK;
}

}  // namespace

extern "C" {

// ---------------------------------------------------------------------------
// Ulysses layout switch: local data movement
// ---------------------------------------------------------------------------

namespace {

// 16-byte units per row of `heads` heads of d two-byte elements; 0 if the row is not a whole number of units
uint64_t row_units(int heads, int d) {
  const uint64_t bytes = (uint64_t)heads * (uint64_t)d * 2u;
  return bytes % 16u ? 0u : bytes / 16u;
}

int ulysses_heads(const void* src, void* dst, int64_t local_tokens, int H, int d, int g, bool pack, void* stream) {
  if (local_tokens < 0 || H <= 0 || d <= 0 || g <= 0 || H % g != 0) return KNAP_ERR_INVALID_ARG;
  const uint64_t U = row_units(H / g, d);
  if (U == 0) return KNAP_ERR_INVALID_ARG;
  if (local_tokens == 0) return KNAP_OK;
  if ((uint64_t)local_tokens * g * U > (1ull << 31)) return KNAP_ERR_INVALID_ARG;
  if (!src || !dst || src == dst || !aligned(src, 16) || !aligned(dst, 16)) return KNAP_ERR_INVALID_ARG;
  DeviceInfo* di = device_info();
  if (!di) return KNAP_ERR_LAUNCH_FAILED;
  const hipError_t e = knap::launch_ulysses_heads(src, dst, (uint32_t)local_tokens, (uint32_t)U, (uint32_t)g, pack,
                                                  di->cus, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) { g_last_hip_error = static_cast<int>(e); return KNAP_ERR_LAUNCH_FAILED; }
  return KNAP_OK;
}

int ulysses_rows(const void* src, void* dst, const int32_t* row_map, int64_t total_tokens, int heads_local, int d,
                 bool gather, void* stream) {
  if (total_tokens < 0 || heads_local <= 0 || d <= 0) return KNAP_ERR_INVALID_ARG;
  const uint64_t U = row_units(heads_local, d);
  if (U == 0) return KNAP_ERR_INVALID_ARG;
  if (total_tokens == 0) return KNAP_OK;
  if ((uint64_t)total_tokens * U > (1ull << 31)) return KNAP_ERR_INVALID_ARG;
  if (!src || !dst || !row_map || src == dst || !aligned(src, 16) || !aligned(dst, 16) || !aligned(row_map, 4))
    return KNAP_ERR_INVALID_ARG;
  DeviceInfo* di = device_info();
  if (!di) return KNAP_ERR_LAUNCH_FAILED;
  const hipError_t e = knap::launch_ulysses_rows(src, dst, row_map, (uint32_t)total_tokens, (uint32_t)U, gather,
                                                 di->cus, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) { g_last_hip_error = static_cast<int>(e); return KNAP_ERR_LAUNCH_FAILED; }
  return KNAP_OK;
}

}  // namespace

int knap_ulysses_pack_heads(const void* x, int64_t local_tokens, int H, int d, int g, void* y, void* stream) {
  return ulysses_heads(x, y, local_tokens, H, d, g, true, stream);
}

int knap_ulysses_unpack_heads(const void* y, int64_t local_tokens, int H, int d, int g, void* x, void* stream) {
  return ulysses_heads(y, x, local_tokens, H, d, g, false, stream);
}

size_t knap_ulysses_plan_workspace_bytes(int n_seq, int g) {
  if (n_seq < 0 || g <= 0) return 0;
  return round_up((static_cast<size_t>(n_seq) + 1) * static_cast<size_t>(g) * sizeof(int32_t), 256);
}

int knap_ulysses_plan(const int32_t* cu_seqlens, int n_seq, int64_t total_tokens, int g,
                      int32_t* row_map, void* workspace, size_t workspace_bytes, void* stream) {
  if (n_seq < 0 || g <= 0 || g > KNAP_ULYSSES_MAX_GPUS || total_tokens < 0 || total_tokens > INT32_MAX)
    return KNAP_ERR_INVALID_ARG;
  if (n_seq > KNAP_MAX_SEQS) return KNAP_ERR_TOO_MANY_SEQS;
  if (n_seq == 0 || total_tokens == 0) return KNAP_OK;
  if (!cu_seqlens || !row_map || !workspace || !aligned(cu_seqlens, 4) || !aligned(row_map, 4) ||
      !aligned(workspace, 4))
    return KNAP_ERR_INVALID_ARG;
  if (workspace_bytes < knap_ulysses_plan_workspace_bytes(n_seq, g)) return KNAP_ERR_WORKSPACE_TOO_SMALL;
  const hipError_t e = knap::launch_ulysses_plan(cu_seqlens, n_seq, g, (int)total_tokens,
                                                 static_cast<int32_t*>(workspace), row_map,
                                                 static_cast<hipStream_t>(stream));
  if (e != hipSuccess) { g_last_hip_error = static_cast<int>(e); return KNAP_ERR_LAUNCH_FAILED; }
  return KNAP_OK;
}

int knap_ulysses_gather_chunks(const void* recv, const int32_t* row_map, int64_t total_tokens,
                               int heads_local, int d, void* z, void* stream) {
  return ulysses_rows(recv, z, row_map, total_tokens, heads_local, d, true, stream);
}

int knap_ulysses_scatter_chunks(const void* z, const int32_t* row_map, int64_t total_tokens,
                                int heads_local, int d, void* send, void* stream) {
  return ulysses_rows(z, send, row_map, total_tokens, heads_local, d, false, stream);
}

const char* knap_strerror(int code) {
  switch (code) {
    case KNAP_OK: return "success";
    case KNAP_ERR_INVALID_ARG: return "invalid argument";
    case KNAP_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case KNAP_ERR_LAUNCH_FAILED: return "kernel launch failed";
    case KNAP_ERR_TOO_MANY_SEQS: return "too many sequences in one bag";
    case KNAP_ERR_CAPACITY: return "output array too small";
    case KNAP_ERR_PARSE: return "malformed topology string";
    case KNAP_ERR_SCRATCH_TOO_SMALL: return "bag exceeds the library's own scratch (KNAP_NOALLOC_MAX_ROWS)";
    default: return "unknown error";
  }
}

int knap_last_hip_error(void) { return g_last_hip_error; }

void knap_bwd_profile_events(void* start, void* stop) {
  g_prof_start = static_cast<hipEvent_t>(start);
  g_prof_stop = static_cast<hipEvent_t>(stop);
}

int knap_launch_workgroups(int which) {
  DeviceInfo* di = device_info();
  if (!di) return -1;
  return di->cus * (which == 0 ? di->fwd_wg[1] : which == 1 ? di->dkdv_wg[1] : di->dq_wg[1]);
}

}  // extern "C"
