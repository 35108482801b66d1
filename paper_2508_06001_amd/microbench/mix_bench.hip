// MFMA occupancy a SIMD reaches on an attention kernel's instruction mix, and which ingredient costs it:
// per 8 MFMAs (32x32x16 bf16) a wave issues NL LDS operand reads (ds_read_b128, 1 KB each), NF plain VALU
// instructions and NE exponentials, interleaved under scheduling hints; 1 to 4 waves per SIMD.  Times are
// shader clocks (s_memtime), so the clock the chip settles at does not matter.
// build: hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops mix_bench.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
// per iteration: 8 MFMAs, NL LDS b128 reads (operands when NL == 8 or 4), NF fmas, NE exps; PRIO: s_setprio 1 around nothing/ whole loop
template <int NF, int NE, int NL, int PRIO, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void k(float* out, long long* clk, int iters, float seed) {
  __shared__ bf16x8 lds[64 * 16];
  for (int i = threadIdx.x; i < 64 * 16; i += 64 * WAVES) for (int e = 0; e < 8; ++e) lds[i][e] = (__bf16)(seed * i + e);
  __syncthreads();
  f32x16 acc0 = {}, acc1 = {};
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(seed + e); b[e] = (__bf16)(seed - e); }
  float v[16];
  for (int i = 0; i < 16; ++i) v[i] = seed + threadIdx.x * 1e-3f + i;
  bf16x8 r[8];
  for (int i = 0; i < 8; ++i) r[i] = a;
  if (PRIO == 1) { if ((threadIdx.x >> 6) & 4) __builtin_amdgcn_s_setprio(1); }   // waves 4..7 higher
  const long long t0 = __builtin_amdgcn_s_memtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (PRIO == 2) __builtin_amdgcn_s_setprio(1);
      // NL == 4: every operand read feeds two MFMAs (a 64 x 64 register block per wave)
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(NL == 8 ? r[2 * i] : NL == 4 ? r[i] : a, b, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(NL == 8 ? r[2 * i + 1] : NL == 4 ? r[i] : a, b, acc1, 0, 0, 0);
      if (PRIO == 2) __builtin_amdgcn_s_setprio(0);
    }
#pragma unroll
    for (int i = 0; i < NL; ++i) r[i] = lds[(threadIdx.x & 63) + 64 * ((i + it) & 15)];
#pragma unroll
    for (int i = 0; i < NE; ++i) v[i & 7] = __builtin_amdgcn_exp2f(v[i & 7]);
#pragma unroll
    for (int j = 0; j < NF; ++j) v[8 + (j & 7)] = __builtin_fmaf(v[8 + (j & 7)], 1.0001f, 0.5f);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x8, 1, 0);
      if (NL >= 8 || (NL == 4 && (i & 1))) __builtin_amdgcn_sched_group_barrier(0x100, NL >= 8 ? NL / 8 : 1, 0);
      if (NF + NE) __builtin_amdgcn_sched_group_barrier(0x2, (NF + NE + 7) / 8, 0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  const long long t1 = __builtin_amdgcn_s_memtime();
  float s = acc0[0] + acc1[3];
  for (int i = 0; i < 16; ++i) s += v[i];
  for (int i = 0; i < 8; ++i) s += (float)r[i][1];
  if (s == 123.456f) out[0] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) clk[0] = t1 - t0;
  if (threadIdx.x == 64 * (WAVES - 1) && blockIdx.x == 0) clk[1] = t1 - t0;
}
template <int NF, int NE, int NL, int PRIO, int WAVES> void run(const char* name) {
  float* d; long long* c; CK(hipMalloc(&d, 4)); CK(hipMalloc(&c, 16));
  const int iters = 20000;
  k<NF, NE, NL, PRIO, WAVES><<<256, 64 * WAVES>>>(d, c, 100, 0.001f); CK(hipDeviceSynchronize());
  k<NF, NE, NL, PRIO, WAVES><<<256, 64 * WAVES>>>(d, c, iters, 0.001f); CK(hipDeviceSynchronize());
  long long h[2]; CK(hipMemcpy(h, c, 16, hipMemcpyDeviceToHost));
  const double per_simd_mfma = 8.0 * 32 * (WAVES / 4);   // MFMA pipe clocks needed per iteration of all waves on a SIMD
  printf("%-44s waves/SIMD %d: first wave %7.1f last wave %7.1f clk/iter -> MFMA busy %.0f %%\n", name, WAVES / 4,
         (double)h[0] / iters, (double)h[1] / iters, 100.0 * per_simd_mfma / ((double)h[1] / iters));
  CK(hipFree(d)); CK(hipFree(c));
}
int main() {
  run<36, 8, 8, 0, 8>("36 FMA + 8 EXP + 8 LDS");
  run<36, 8, 0, 0, 8>("36 FMA + 8 EXP, no LDS");
  run<36, 0, 8, 0, 8>("36 FMA + 8 LDS, no EXP");
  run<0, 8, 8, 0, 8>("8 EXP + 8 LDS, no FMA");
  run<16, 8, 8, 0, 8>("16 FMA + 8 EXP + 8 LDS");
  run<24, 8, 8, 0, 8>("24 FMA + 8 EXP + 8 LDS");
  run<36, 8, 8, 1, 8>("36+8+8, waves 4..7 at priority 1");
  run<36, 8, 8, 2, 8>("36+8+8, priority 1 around MFMAs");
  run<36, 8, 8, 0, 4>("36 FMA + 8 EXP + 8 LDS");
  run<36, 8, 8, 0, 12>("36 FMA + 8 EXP + 8 LDS");
  run<36, 8, 8, 0, 16>("36 FMA + 8 EXP + 8 LDS");
  run<16, 8, 8, 0, 16>("16 FMA + 8 EXP + 8 LDS");
  run<36, 8, 4, 0, 4>("36 FMA + 8 EXP + 4 LDS (each read feeds 2)");
  run<36, 8, 4, 0, 8>("36 FMA + 8 EXP + 4 LDS (each read feeds 2)");
  run<28, 8, 4, 0, 4>("28 FMA + 8 EXP + 4 LDS (each read feeds 2)");
  run<28, 8, 4, 0, 8>("28 FMA + 8 EXP + 4 LDS (each read feeds 2)");
  run<36, 8, 0, 0, 4>("36 FMA + 8 EXP, no LDS");
  // head dimension 64: the softmax arithmetic per MFMA doubles
  run<72, 16, 8, 0, 8>("72 FMA + 16 EXP + 8 LDS (d = 64 mix)");
  run<72, 16, 4, 0, 8>("72 FMA + 16 EXP + 4 LDS (d = 64, each read feeds 2)");
  run<72, 16, 0, 0, 8>("72 FMA + 16 EXP, no LDS");
  return 0;
}
