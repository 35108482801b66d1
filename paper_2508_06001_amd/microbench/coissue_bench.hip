// Do MFMA and VALU / LDS instructions of DIFFERENT waves on one SIMD overlap on gfx950, and do they
// overlap inside ONE wave?  A workgroup of 8 waves puts waves w and w + 4 on the same SIMD; waves
// 0..3 run workload A and waves 4..7 workload B (or exit at once).  Times are in shader clocks read
// with s_memtime on both sides of the loop, so they do not depend on the clock the chip settles at;
// the clock itself is reported from the ratio to the constant 100 MHz counter.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <algorithm>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

enum Work { NONE = 0, MFMA = 1, FMA = 2, EXP = 3, LDS = 4, MFMA_FMA = 5, MFMA_EXP = 6, MFMA_LDS = 7, MIX = 8, MIX_TR = 9 };

// per loop iteration: MFMA: 8 MFMAs (2 accumulators alternating); FMA / EXP: 48 VALU instructions on 16
// independent chains; LDS: 8 ds_read_b128; the MFMA_x kinds issue both, interleaved by the compiler's
// scheduler under group hints (1 MFMA then 6 VALU, or 1 MFMA then 1 read).
template <int W>
__device__ __forceinline__ void body(int iters, float seed, const bf16x8* lds, float& sink) {
  f32x16 acc0 = {}, acc1 = {};
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(seed + e); b[e] = (__bf16)(seed - e); }
  float v[16];
  for (int i = 0; i < 16; ++i) v[i] = seed + threadIdx.x * 1e-3f + i;
  bf16x8 r[8];
  for (int i = 0; i < 8; ++i) r[i] = a;
  for (int it = 0; it < iters; ++it) {
    if (W == MIX || W == MIX_TR) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(r[2 * i], b, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(r[2 * i + 1], b, acc1, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (W == MIX) {
          r[i] = lds[(threadIdx.x & 63) + 64 * ((i + it) & 15)];
        } else {   // two 64-bit transposing reads per operand
          typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
          const __bf16* p = reinterpret_cast<const __bf16*>(&lds[64 * ((i + it) & 15)]) + 4 * (threadIdx.x & 63);
          bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(p));
          bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(p + 256));
          r[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = __builtin_amdgcn_exp2f(v[i]);
#pragma unroll
      for (int j = 0; j < 36; ++j) v[8 + (j & 7)] = __builtin_fmaf(v[8 + (j & 7)], 1.0001f, 0.5f);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x8, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, W == MIX ? 1 : 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x2, 6, 0);
      }
    }
    if (W == MFMA || W == MFMA_FMA || W == MFMA_EXP || W == MFMA_LDS) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(W == MFMA_LDS ? r[2 * i] : a, b, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(W == MFMA_LDS ? r[2 * i + 1] : a, b, acc1, 0, 0, 0);
      }
    }
    if (W == FMA || W == MFMA_FMA) {
#pragma unroll
      for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = __builtin_fmaf(v[i], 1.0001f, 0.5f);
    }
    if (W == EXP || W == MFMA_EXP) {
#pragma unroll
      for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = __builtin_amdgcn_exp2f(v[i]);
    }
    if (W == LDS || W == MFMA_LDS) {
#pragma unroll
      for (int i = 0; i < 8; ++i) r[i] = lds[(threadIdx.x & 63) + 64 * ((i + it) & 15)];
    }
    if (W == MFMA_FMA || W == MFMA_EXP) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x8, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x2, 6, 0);
      }
    }
    if (W == MFMA_LDS) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x8, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
    if (W == LDS) {   // consume the reads without an MFMA
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] += __builtin_bit_cast(float, (uint32_t)__builtin_bit_cast(uint16_t, r[i][0]) << 16);
    }
  }
  float s = acc0[0] + acc1[3];
  for (int i = 0; i < 16; ++i) s += v[i];
  for (int i = 0; i < 8; ++i) s += (float)r[i][1];
  sink = s;
}

template <int WA, int WB>
__global__ __launch_bounds__(512) void k(float* out, long long* clk, int iters, float seed) {
  __shared__ bf16x8 lds[64 * 16];
  for (int i = threadIdx.x; i < 64 * 16; i += 512) for (int e = 0; e < 8; ++e) lds[i][e] = (__bf16)(seed * i + e);
  __syncthreads();
  const int role = threadIdx.x >> 8;     // waves 0..3 / 4..7
  float sink = 0.f;
  const long long t0 = __builtin_amdgcn_s_memtime();
  const long long w0 = wall_clock64();
  if (role == 0) body<WA>(iters, seed, lds, sink);
  else if (WB != NONE) body<WB>(iters, seed, lds, sink);
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  const long long t1 = __builtin_amdgcn_s_memtime();
  const long long w1 = wall_clock64();
  if (sink == 123.456f) out[0] = sink;
  if ((threadIdx.x & 63) == 0 && blockIdx.x == 0) {
    clk[2 * (threadIdx.x >> 6)] = t1 - t0;
    clk[2 * (threadIdx.x >> 6) + 1] = w1 - w0;
  }
}

template <int WA, int WB>
void run(const char* name) {
  float* d; long long* c; CK(hipMalloc(&d, 4)); CK(hipMalloc(&c, 16 * sizeof(long long)));
  const int iters = 20000;
  k<WA, WB><<<256, 512>>>(d, c, 100, 0.001f); CK(hipDeviceSynchronize());
  k<WA, WB><<<256, 512>>>(d, c, iters, 0.001f); CK(hipDeviceSynchronize());
  long long h[16]; CK(hipMemcpy(h, c, sizeof(h), hipMemcpyDeviceToHost));
  // wave 0 runs A, wave 4 runs B
  printf("%-34s A: %7.1f clk/iter   B: %7.1f clk/iter   shader clock %.2f GHz\n", name,
         (double)h[0] / iters, (double)h[8] / iters, (double)h[0] / ((double)h[1] * 10e-9) / 1e9);
  CK(hipFree(d)); CK(hipFree(c));
}

int main() {
  printf("per iteration: MFMA = 8 x mfma_f32_32x32x16_bf16 (2 chains), FMA/EXP = 48 VALU, LDS = 8 ds_read_b128\n");
  run<MFMA, NONE>("A=MFMA alone");
  run<FMA, NONE>("A=FMA alone");
  run<EXP, NONE>("A=EXP alone");
  run<LDS, NONE>("A=LDS alone");
  run<MFMA, MFMA>("A=MFMA  B=MFMA");
  run<MFMA, FMA>("A=MFMA  B=FMA (other wave)");
  run<MFMA, EXP>("A=MFMA  B=EXP (other wave)");
  run<MFMA, LDS>("A=MFMA  B=LDS (other wave)");
  run<FMA, FMA>("A=FMA   B=FMA");
  run<EXP, EXP>("A=EXP   B=EXP");
  run<MFMA_FMA, NONE>("A=MFMA+FMA in one wave");
  run<MFMA_EXP, NONE>("A=MFMA+EXP in one wave");
  run<MFMA_LDS, NONE>("A=MFMA<-LDS in one wave");
  run<MFMA_FMA, MFMA_FMA>("A=B=MFMA+FMA");
  run<MFMA_EXP, MFMA_EXP>("A=B=MFMA+EXP");
  run<MFMA_LDS, MFMA_LDS>("A=B=MFMA<-LDS");
  printf("MIX = 8 MFMA fed from 8 LDS reads + 36 FMA + 8 EXP per iteration (an attention kernel's mix per MFMA); _TR: transposing reads\n");
  run<MIX, NONE>("A=MIX alone");
  run<MIX, MIX>("A=B=MIX");
  run<MIX_TR, MIX_TR>("A=B=MIX_TR");
  return 0;
}
