// Local (one-GPU) data movement of the Ulysses layout switch (Sec. 3.4): a multi-GPU bag goes from
// (partial sequences, full heads) to (full sequences, partial heads) with one all-to-all before
// attention and back with one after it.  The all-to-all moves contiguous buffers, so each GPU
//   before sending   splits its (T_r, H, d) tensor into g slabs (T_r, H/g, d), one per destination,
//   after receiving  puts the chunks of the g received slabs (chunk r of every sequence, from GPU r;
//                    chunks as cut by the second pass of Sec. 3.3) together into whole sequences,
// and runs the inverse of each on the way back.  Both are permutations of (token, head-group) rows of
// (H/g) d elements; the kernels move them in 16-byte units, every unit read once and written once, and
// are bound by HBM bandwidth.  The row permutation of the second step depends only on the bag's sequence
// lengths and is built once per bag (ulysses plan) for q, k, v, the output and every layer.
#include "knap_kernels.h"

#include <stdint.h>

namespace knap {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 256;
// Tuned on an MI355X (one (24576, 24, 128) bf16 tensor, buffers rotated out of the Infinity Cache):
// non-temporal loads and stores +12 % over plain ones, 32 workgroups per CU +4 % over 16, two units per
// thread and trip as good as four or eight; 5.7 TB/s against 5.3 TB/s of the runtime's device copy.
constexpr int kUnroll = 2;           // 16-byte units per thread and loop trip
constexpr int kWorkgroupsPerCu = 32; // grid cap; beyond it the kernels loop with a grid stride

__device__ __forceinline__ u32x4_t ld_unit(const u32x4_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st_unit(u32x4_t* p, u32x4_t v) { __builtin_nontemporal_store(v, p); }

// y[(r T + t) U + c] = x[(t g + r) U + c]: U units per (token, head-group) row.  Iterates over x's
// linear index, so x is touched in address order and y in runs of U units.
template <bool PACK>
__global__ __launch_bounds__(kCopyThreads) void ulysses_heads_kernel(
    const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, uint32_t T, uint32_t U, uint32_t g) {
  const uint32_t GU = g * U;
  const uint32_t N = T * GU;
  const uint32_t stride = gridDim.x * kCopyThreads;
  for (uint32_t e0 = blockIdx.x * kCopyThreads + threadIdx.x; e0 < N; e0 += kUnroll * stride) {
    uint32_t xi[kUnroll], yi[kUnroll];
    u32x4_t val[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const uint32_t e = e0 + k * stride;
      const uint32_t t = e / GU;
      const uint32_t w = e - t * GU;
      const uint32_t r = w / U;
      xi[k] = e;
      yi[k] = (r * T + t) * U + (w - r * U);
    }
#pragma unroll
    for (int k = 0; k < kUnroll; ++k)
      if (xi[k] < N) val[k] = ld_unit(&src[PACK ? xi[k] : yi[k]]);
#pragma unroll
    for (int k = 0; k < kUnroll; ++k)
      if (xi[k] < N) st_unit(&dst[PACK ? yi[k] : xi[k]], val[k]);
  }
}

// gather: z[t] = recv[row_map[t]]; scatter: send[row_map[t]] = z[t]; rows of U units.
template <bool GATHER>
__global__ __launch_bounds__(kCopyThreads) void ulysses_rows_kernel(
    const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, const int32_t* __restrict__ row_map,
    uint32_t T, uint32_t U) {
  const uint32_t N = T * U;
  const uint32_t stride = gridDim.x * kCopyThreads;
  for (uint32_t e0 = blockIdx.x * kCopyThreads + threadIdx.x; e0 < N; e0 += kUnroll * stride) {
    uint32_t zi[kUnroll], mi[kUnroll];
    u32x4_t val[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const uint32_t e = e0 + k * stride;
      const uint32_t t = e / U;
      zi[k] = e;
      mi[k] = e < N ? (uint32_t)row_map[t] * U + (e - t * U) : 0u;
    }
#pragma unroll
    for (int k = 0; k < kUnroll; ++k)
      if (zi[k] < N) val[k] = ld_unit(&src[GATHER ? mi[k] : zi[k]]);
#pragma unroll
    for (int k = 0; k < kUnroll; ++k)
      if (zi[k] < N) st_unit(&dst[GATHER ? zi[k] : mi[k]], val[k]);
  }
}

// chunk r of a sequence of L tokens cut into g chunks, the first L mod g one token longer
__device__ __forceinline__ int chunk_len(int L, int g, int r) { return L / g + (r < L % g ? 1 : 0); }

// table[s g + r]       rows of slab r that belong to sequences before s      (s = 0 .. n_seq - 1)
// table[n_seq g + r]   first row of slab r in the receive buffer (slabs in GPU order)
// One workgroup; thread r walks the sequences for GPU r.  cu_seqlens is staged in LDS first.
__global__ __launch_bounds__(kCopyThreads) void ulysses_offsets_kernel(
    const int32_t* __restrict__ cu, int n_seq, int g, int32_t* __restrict__ table) {
  extern __shared__ int32_t s_cu[];          // n_seq + 1 lengths boundaries, then g slab sizes
  int32_t* s_rows = s_cu + n_seq + 1;
  for (int i = threadIdx.x; i <= n_seq; i += kCopyThreads) s_cu[i] = cu[i];
  __syncthreads();
  const int r = threadIdx.x;
  if (r < g) {
    int run = 0;
    for (int s = 0; s < n_seq; ++s) {
      table[s * g + r] = run;
      run += chunk_len(s_cu[s + 1] - s_cu[s], g, r);
    }
    s_rows[r] = run;
  }
  __syncthreads();
  if (r < g) {
    int start = 0;
    for (int q = 0; q < r; ++q) start += s_rows[q];
    table[n_seq * g + r] = start;
  }
}

// row_map[t] for every row t of the (full sequences) layout
__global__ __launch_bounds__(kCopyThreads) void ulysses_row_map_kernel(
    const int32_t* __restrict__ cu, int n_seq, int g, const int32_t* __restrict__ table, int T,
    int32_t* __restrict__ row_map) {
  const int t = blockIdx.x * kCopyThreads + threadIdx.x;
  if (t >= T) return;
  // the sequence of row t: largest s with cu[s] <= t among the sequences that have rows
  int lo = 0, hi = n_seq - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid - 1;
  }
  const int s = lo;
  const int L = cu[s + 1] - cu[s];
  const int i = t - cu[s];
  const int base = L / g, rem = L % g;
  // chunks 0 .. rem - 1 hold base + 1 tokens, the others base
  int r, j;
  if (i < rem * (base + 1)) {
    r = i / (base + 1);
    j = i - r * (base + 1);
  } else {
    const int k = i - rem * (base + 1);
    r = rem + k / base;               // base > 0 here: i < L and the longer chunks are used up
    j = k - (r - rem) * base;
  }
  // rows past cu[n_seq] (a total_tokens larger than the lengths add up to) must not index outside the table
  r = min(max(r, 0), g - 1);
  row_map[t] = table[n_seq * g + r] + table[s * g + r] + j;
}

int copy_grid(uint64_t units, int cus) {
  const uint64_t per_wg = (uint64_t)kCopyThreads * kUnroll;
  const uint64_t want = (units + per_wg - 1) / per_wg;
  const uint64_t cap = (uint64_t)cus * kWorkgroupsPerCu;
  return (int)(want < cap ? (want ? want : 1) : cap);
}

}  // namespace

hipError_t launch_ulysses_heads(const void* src, void* dst, uint32_t T, uint32_t U, uint32_t g, bool pack,
                                int cus, hipStream_t stream) {
  const int grid = copy_grid((uint64_t)T * g * U, cus);
  if (pack)
    hipLaunchKernelGGL(ulysses_heads_kernel<true>, dim3(grid), dim3(kCopyThreads), 0, stream,
                       (const u32x4_t*)src, (u32x4_t*)dst, T, U, g);
  else
    hipLaunchKernelGGL(ulysses_heads_kernel<false>, dim3(grid), dim3(kCopyThreads), 0, stream,
                       (const u32x4_t*)src, (u32x4_t*)dst, T, U, g);
  return hipGetLastError();
}

hipError_t launch_ulysses_rows(const void* src, void* dst, const int32_t* row_map, uint32_t T, uint32_t U,
                               bool gather, int cus, hipStream_t stream) {
  const int grid = copy_grid((uint64_t)T * U, cus);
  if (gather)
    hipLaunchKernelGGL(ulysses_rows_kernel<true>, dim3(grid), dim3(kCopyThreads), 0, stream,
                       (const u32x4_t*)src, (u32x4_t*)dst, row_map, T, U);
  else
    hipLaunchKernelGGL(ulysses_rows_kernel<false>, dim3(grid), dim3(kCopyThreads), 0, stream,
                       (const u32x4_t*)src, (u32x4_t*)dst, row_map, T, U);
  return hipGetLastError();
}

hipError_t launch_ulysses_plan(const int32_t* cu, int n_seq, int g, int T, int32_t* table, int32_t* row_map,
                               hipStream_t stream) {
  const size_t dyn = (size_t)(n_seq + 1 + g) * sizeof(int32_t);
  hipLaunchKernelGGL(ulysses_offsets_kernel, dim3(1), dim3(kCopyThreads), dyn, stream, cu, n_seq, g, table);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int grid = (T + kCopyThreads - 1) / kCopyThreads;
  hipLaunchKernelGGL(ulysses_row_map_kernel, dim3(grid), dim3(kCopyThreads), 0, stream,
                     cu, n_seq, g, (const int32_t*)table, T, row_map);
  return hipGetLastError();
}

}  // namespace knap
