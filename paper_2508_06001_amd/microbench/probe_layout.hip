// In-bounds probe of MFMA operand/result lane layouts and ds_read_tr16_b64 on gfx950.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

// A: 32x16 row-major (M x K), B: 16x32 (K x N) row-major, floats holding small ints.
// Hypothesis: lane l holds A[l%32][8*(l/32)+e], B[8*(l/32)+e][l%32]; D reg r: row 8*(r/4)+4*(l/32)+r%4, col l%32
__global__ void probe_mfma32(const float* A, const float* B, float* D) {
  int l = threadIdx.x;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)A[(l % 32) * 16 + 8 * (l / 32) + e];
    b[e] = (__bf16)B[(8 * (l / 32) + e) * 32 + (l % 32)];
  }
  f32x16 c = {0};
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  for (int r = 0; r < 16; ++r) {
    int row = 8 * (r / 4) + 4 * (l / 32) + (r % 4);
    D[row * 32 + (l % 32)] = c[r];
  }
}

// 16x16x32: A 16x32, B 32x16. lane l: A[l%16][8*(l/16)+e], B[8*(l/16)+e][l%16]; D reg r: row 4*(l/16)+r, col l%16
__global__ void probe_mfma16(const float* A, const float* B, float* D) {
  int l = threadIdx.x;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)A[(l % 16) * 32 + 8 * (l / 16) + e];
    b[e] = (__bf16)B[(8 * (l / 16) + e) * 16 + (l % 16)];
  }
  f32x4 c = {0};
  c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  for (int r = 0; r < 4; ++r) {
    int row = 4 * (l / 16) + r;
    D[row * 16 + (l % 16)] = c[r];
  }
}

// ds_read_tr16_b64: LDS holds u16 value = index. lane l reads from byte address 8*l (4 u16 each).
__global__ void probe_tr(uint16_t* out, int stride_elems) {
  __shared__ uint16_t lds[4096];
  int l = threadIdx.x;
  for (int i = l; i < 4096; i += 64) lds[i] = (uint16_t)i;
  __syncthreads();
  short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(lds + l * stride_elems));
  for (int e = 0; e < 4; ++e) out[l * 4 + e] = (uint16_t)v[e];
}

int main() {
  hipDeviceProp_t p; CK(hipGetDeviceProperties(&p, 0));
  printf("device %s arch %s CUs %d clock %d kHz mem %.1f GiB L2 %d sharedPerBlock %zu sharedPerCU %zu regsPerBlock %d warp %d memclock %d kHz buswidth %d\n",
         p.name, p.gcnArchName, p.multiProcessorCount, p.clockRate, p.totalGlobalMem / 1073741824.0, p.l2CacheSize,
         p.sharedMemPerBlock, p.maxSharedMemoryPerMultiProcessor, p.regsPerBlock, p.warpSize, p.memoryClockRate, p.memoryBusWidth);
  // mfma32
  {
    std::vector<float> A(32 * 16), B(16 * 32), D(32 * 32), R(32 * 32, 0.f);
    for (auto& x : A) x = (float)(rand() % 7 - 3);
    for (auto& x : B) x = (float)(rand() % 7 - 3);
    for (int i = 0; i < 32; ++i) for (int j = 0; j < 32; ++j) { float s = 0; for (int k = 0; k < 16; ++k) s += A[i * 16 + k] * B[k * 32 + j]; R[i * 32 + j] = s; }
    float *dA, *dB, *dD; CK(hipMalloc(&dA, A.size() * 4)); CK(hipMalloc(&dB, B.size() * 4)); CK(hipMalloc(&dD, D.size() * 4));
    CK(hipMemcpy(dA, A.data(), A.size() * 4, hipMemcpyHostToDevice)); CK(hipMemcpy(dB, B.data(), B.size() * 4, hipMemcpyHostToDevice));
    probe_mfma32<<<1, 64>>>(dA, dB, dD); CK(hipDeviceSynchronize());
    CK(hipMemcpy(D.data(), dD, D.size() * 4, hipMemcpyDeviceToHost));
    int bad = 0; for (int i = 0; i < 1024; ++i) bad += (D[i] != R[i]);
    printf("mfma_f32_32x32x16_bf16 layout hypothesis: %s (%d mismatches)\n", bad ? "WRONG" : "OK", bad);
  }
  {
    std::vector<float> A(16 * 32), B(32 * 16), D(16 * 16), R(16 * 16, 0.f);
    for (auto& x : A) x = (float)(rand() % 7 - 3);
    for (auto& x : B) x = (float)(rand() % 7 - 3);
    for (int i = 0; i < 16; ++i) for (int j = 0; j < 16; ++j) { float s = 0; for (int k = 0; k < 32; ++k) s += A[i * 32 + k] * B[k * 16 + j]; R[i * 16 + j] = s; }
    float *dA, *dB, *dD; CK(hipMalloc(&dA, A.size() * 4)); CK(hipMalloc(&dB, B.size() * 4)); CK(hipMalloc(&dD, D.size() * 4));
    CK(hipMemcpy(dA, A.data(), A.size() * 4, hipMemcpyHostToDevice)); CK(hipMemcpy(dB, B.data(), B.size() * 4, hipMemcpyHostToDevice));
    probe_mfma16<<<1, 64>>>(dA, dB, dD); CK(hipDeviceSynchronize());
    CK(hipMemcpy(D.data(), dD, D.size() * 4, hipMemcpyDeviceToHost));
    int bad = 0; for (int i = 0; i < 256; ++i) bad += (D[i] != R[i]);
    printf("mfma_f32_16x16x32_bf16 layout hypothesis: %s (%d mismatches)\n", bad ? "WRONG" : "OK", bad);
  }
  for (int stride : {4, 16, 32}) {
    uint16_t* dO; CK(hipMalloc(&dO, 256 * 2));
    probe_tr<<<1, 64>>>(dO, stride); CK(hipDeviceSynchronize());
    std::vector<uint16_t> O(256); CK(hipMemcpy(O.data(), dO, 512, hipMemcpyDeviceToHost));
    printf("ds_read_tr16_b64, lane l reads 4 u16 at element offset %d*l; result per lane (element indices):\n", stride);
    for (int l = 0; l < 64; ++l) printf("  lane %2d: %4d %4d %4d %4d\n", l, O[l * 4], O[l * 4 + 1], O[l * 4 + 2], O[l * 4 + 3]);
  }
  return 0;
}
