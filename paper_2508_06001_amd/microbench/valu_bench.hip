// VALU issue cost per wave64 instruction on gfx950 (1 or 2 waves per SIMD).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
template <int OP>
__global__ __launch_bounds__(256) void k(float* out, int iters, float seed) {
  float a[16];
  for (int i = 0; i < 16; ++i) a[i] = seed + threadIdx.x * 1e-3f + i;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (OP == 0) a[i] = __builtin_amdgcn_exp2f(a[i]);
      if (OP == 1) a[i] = __builtin_fmaf(a[i], 1.0001f, 0.5f);
      if (OP == 2) a[i] = fmaxf(fmaxf(a[i], a[(i + 1) & 15]), a[(i + 2) & 15]);
      if (OP == 3) { bf16x2 p; p[0] = (__bf16)a[i]; p[1] = (__bf16)a[(i + 1) & 15]; a[i] += __builtin_bit_cast(float, p); }
      if (OP == 4) a[i] = a[i] * 1.0001f;
    }
  }
  float s = 0; for (int i = 0; i < 16; ++i) s += a[i];
  if (s == 123.f) out[0] = s;
}
template <int OP> void run(const char* name, int wgs, int instr_per_elem) {
  float* d; CK(hipMalloc(&d, 4));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  const int iters = 20000;
  k<OP><<<256 * wgs, 256>>>(d, 10, 0.001f); CK(hipDeviceSynchronize());
  CK(hipEventRecord(a)); k<OP><<<256 * wgs, 256>>>(d, iters, 0.001f); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b));
  double clk = ms * 1e-3 * 2.4e9;
  double instrs_per_simd = (double)iters * 16 * instr_per_elem * wgs;   // one wave per SIMD per WG
  printf("%-28s waves/SIMD %d: %.2f cycles per wave-instruction (%.2f ms)\n", name, wgs, clk / instrs_per_simd, ms);
}
int main() {
  for (int w : {1, 2}) {
    run<0>("v_exp_f32", w, 1);
    run<1>("v_fma_f32", w, 1);
    run<4>("v_mul_f32", w, 1);
    run<2>("v_max3_f32 (or 2 max)", w, 1);
    run<3>("cvt_pk_bf16 + add", w, 2);
  }
  return 0;
}
