// In-bounds probe of buffer_load_dwordx4 ... lds on gfx950: which LDS bytes does each lane's data land in,
// what happens for lanes whose offset is beyond num_records, and does vmcnt(0) + barrier make it visible.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

__global__ void probe(const unsigned* src, unsigned* out, int num_bytes, int mode) {
  __shared__ __attribute__((aligned(16))) unsigned lds[2048];
  const int l = threadIdx.x;
  for (int i = l; i < 2048; i += 64) lds[i] = 0xdeadbeef;
  __syncthreads();
  __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)src, 0, num_bytes, 0x00020000);
  // lane l loads the 16 B chunk number perm(l) of the source
  int chunk = (mode == 0) ? l : (l ^ 5);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(lds + 256), 16, chunk * 16, 0, 0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  for (int i = l; i < 2048; i += 64) out[i] = lds[i];
}

int main() {
  std::vector<unsigned> h(4096);
  for (int i = 0; i < 4096; ++i) h[i] = i;          // dword i holds i; chunk c holds 4c..4c+3
  unsigned *dsrc, *dout; CK(hipMalloc(&dsrc, 4096 * 4)); CK(hipMalloc(&dout, 2048 * 4));
  CK(hipMemcpy(dsrc, h.data(), 4096 * 4, hipMemcpyHostToDevice));
  for (int mode = 0; mode < 3; ++mode) {
    int num_bytes = (mode == 2) ? 40 * 16 : 4096 * 4;   // mode 2: chunks >= 40 are out of range
    probe<<<1, 64>>>(dsrc, dout, num_bytes, mode == 1 ? 1 : 0); CK(hipDeviceSynchronize());
    std::vector<unsigned> o(2048); CK(hipMemcpy(o.data(), dout, 2048 * 4, hipMemcpyDeviceToHost));
    printf("mode %d: LDS dwords written (index: value), base offset 256 dwords:\n", mode);
    int first = -1, last = -1, n = 0;
    for (int i = 0; i < 2048; ++i) if (o[i] != 0xdeadbeef) { if (first < 0) first = i; last = i; ++n; }
    printf("  written range [%d, %d], count %d\n", first, last, n);
    for (int c = 0; c < 64; c += (mode == 0 ? 9 : 1)) {
      int i = 256 + 4 * c;
      printf("  lds chunk %2d: %08x %08x %08x %08x\n", c, o[i], o[i + 1], o[i + 2], o[i + 3]);
    }
  }
  return 0;
}
