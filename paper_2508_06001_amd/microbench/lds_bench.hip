// LDS read throughput for the access patterns of the attention kernels (in-bounds, gfx950).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

// mode 0: b128 contiguous (lane i -> 16 B at 16 i)
// mode 1: b128 row reads: lane l -> row (l%32) * stride + 16*(l/32) bytes  (+ chunk offset)
// mode 2: tr b64: 16-lane block: lane i -> row (k0 + i/4)*stride + (n0 + 4*(i%4))*2, n0 = 16*((l/16)&1), k0 = 4*(l/32)
template <int MODE>
__global__ __launch_bounds__(256) void lds_kernel(unsigned* out, int iters, int stride_bytes) {
  extern __shared__ char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < 40960 / 4; i += 256) ((unsigned*)lds)[i] = i;
  __syncthreads();
  unsigned acc = 0;
  int base;
  if (MODE == 0) base = lane * 16;
  else if (MODE == 1) base = (lane & 31) * stride_bytes + 16 * (lane >> 5);
  else { const int i = lane & 15; base = (4 * (lane >> 5) + (i >> 2)) * stride_bytes + (16 * ((lane >> 4) & 1) + 4 * (i & 3)) * 2; }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (MODE == 2) {
        bf16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(lds + base + u * 64));
        acc += __builtin_bit_cast(unsigned long long, v) & 0xffff;
      } else {
        u32x4 v = *(u32x4*)(lds + base + u * 32);
        acc += v[0] ^ v[1] ^ v[2] ^ v[3];
      }
    }
    asm volatile("" ::: "memory");
  }
  if (acc == 0x12345678) out[0] = acc;
}

template <int MODE>
void run(const char* name, int stride, int bytes_per_lane) {
  unsigned* d; CK(hipMalloc(&d, 4));
  const int iters = 20000; const int wgs = getenv("WGS") ? atoi(getenv("WGS")) : 1; const int grid = 256 * wgs;
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  lds_kernel<MODE><<<grid, 256, 40960>>>(d, 100, stride); CK(hipDeviceSynchronize());
  CK(hipEventRecord(a)); lds_kernel<MODE><<<grid, 256, 40960>>>(d, iters, stride); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b));
  double bytes_per_cu = (double)iters * 8 * 256 * bytes_per_lane * wgs;
  double clk = ms * 1e-3 * 2.4e9;
  printf("%-34s stride %4d B: %.1f B/clk/CU  (%.2f ms)\n", name, stride, bytes_per_cu / clk, ms);
  CK(hipFree(d));
}

int main() {
  run<0>("b128 contiguous", 0, 16);
  for (int s : {272, 288, 304, 320, 336, 352, 368, 400, 144, 208}) run<1>("b128 row reads (32 rows x 2 chunks)", s, 16);
  for (int s : {272, 288, 304, 320, 336, 352, 368, 400, 144, 208}) run<2>("tr b64 (8 rows x 64 B)", s, 8);
  return 0;
}
