// Device-side building blocks shared by the forward and backward attention
// kernels: MFMA wrappers, LDS transpose reads, bf16 packing and the tile
// schedule every persistent workgroup rebuilds from cu_seqlens.
//
// gfx950 only.  Lane layouts used throughout (wave64, lane l, hh = l / 32):
//   v_mfma_f32_32x32x16_bf16   A (32 x 16): lane holds A[l % 32][8 hh + e], e = 0..7
//                              B (16 x 32): lane holds B[8 hh + e][l % 32]
//                              D (32 x 32): reg r is D[8 (r / 4) + 4 hh + r % 4][l % 32]
//   ds_read_b64_tr_b16         per 16-lane block, lane i supplies the address of 4
//                              consecutive b16 of "row" i; lane i receives element
//                              (i % 4) of rows 4 e + i / 4, e = 0..3.  Pointing lane i
//                              at X[k0 + i / 4][n0 + 4 (i % 4)] of a row-major X[k][n]
//                              therefore returns X[k0 + e][n0 + i]: a 4 x 16 transpose.
// The contraction index of an MFMA may be permuted freely as long as A and B
// use the same permutation; the kernels exploit that to feed a D-layout result
// straight back in as an operand.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace knap {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;   // 4 waves per workgroup
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

__device__ __forceinline__ bf16x8 zero_bf16x8() {
  u32x4 z = {0u, 0u, 0u, 0u};
  return __builtin_bit_cast(bf16x8, z);
}

// 4 x 16 transposing LDS read (see the header comment).
__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
      (__attribute__((address_space(3))) bf16x4*)(p));
}

__device__ __forceinline__ bf16x8 join(bf16x4 lo, bf16x4 hi) {
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// LDS tile layout for tiles of bf16 rows of D elements, addressed in 16-byte chunks.
//  D = 128: rows are 256 B (all 64 banks), unpadded; chunk c of row r sits at position
//           c ^ (4 (r % 4) + (r / 4) % 4).  Sixteen consecutive rows put one chunk index in
//           sixteen different positions (128-bit row reads: no bank conflict), and four
//           consecutive rows starting at a multiple of four put a 64-byte column strip in
//           sixteen different positions (transposing 64-bit reads: no bank conflict).
//  D = 64:  rows are 128 B; chunk c of row r sits at position c ^ ((r / 2) % 8) (row reads
//           conflict-free, transposing reads partly two-way).
template <int D>
struct Tile {
  static constexpr int LD = D;                                  // row pitch in elements (no padding)
  static constexpr int CPR = D / 8;                             // 16-byte chunks per row
  __device__ static __forceinline__ int chunk_pos(int row, int chunk) {
    if constexpr (D == 128) return chunk ^ (4 * (row & 3) + ((row >> 2) & 3));
    else return chunk ^ ((row >> 1) & 7);                       // D = 64: two rows per 256 B of banks
  }
  // element offset of column `col` (a multiple of 4) of row `row`
  __device__ static __forceinline__ int off(int row, int col) {
    return row * LD + (chunk_pos(row, col >> 3) << 3) + (col & 7);
  }
};

// Asynchronous global -> LDS copy of `rows` x D bf16 rows into a Tile<D> (rows a multiple of
// 4 waves x 1 KB), straight into the swizzled layout: a wave instruction fills 1 KB of LDS,
// lane l supplying the 16 bytes that belong at offset 16 l, whatever global chunk that is.
// `r` covers the valid bytes of the source rows (pitch row_bytes); rows past it arrive as
// zeros.  Completion: s_waitcnt vmcnt(0) by every wave, then a workgroup barrier.
template <int D>
__device__ __forceinline__ void tile_load_async(__bf16* tile, __amdgpu_buffer_rsrc_t r, uint32_t row_bytes,
                                                int rows, int wave, int lane) {
  constexpr int CPR = Tile<D>::CPR;
  constexpr int ROWS_PER_INSTR = 64 / CPR;                       // 4 (D = 128) or 8 (D = 64)
  const int n_instr = rows / (4 * ROWS_PER_INSTR);               // per wave
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (i < n_instr) {
      const int row_base = (wave * n_instr + i) * ROWS_PER_INSTR;
      const int row = row_base + lane / CPR;
      const int chunk = Tile<D>::chunk_pos(row, lane % CPR);     // the swizzle is its own inverse
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          r, (__attribute__((address_space(3))) void*)(tile + row_base * Tile<D>::LD), 16,
          (int)((uint32_t)row * row_bytes + (uint32_t)chunk * 16u), 0, 0, 0);
    }
  }
}

__device__ __forceinline__ void wait_async_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// The swizzle only looks at the low four bits of the row, so a read at (row_base + r, col)
// with row_base a multiple of 16 is the read at (r, col) moved by row_base whole rows.  The
// two readers below keep the few lane-dependent offsets of a wave's access patterns in
// registers once and for all; everything else becomes an immediate offset of the LDS read.

// 128-bit row reads: the lane with l32 = lane % 32 reads elements 16 cc + 8 hh .. + 7 of row
// row_base + l32 (row_base a multiple of 32): an MFMA A or B operand whose contraction index
// runs along the row.
template <int D>
struct RowReader {
  int off[D / 16];
  __device__ __forceinline__ void init(int lane) {
    const int l32 = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int cc = 0; cc < D / 16; ++cc) off[cc] = Tile<D>::off(l32, 16 * cc + 8 * hh);
  }
  __device__ __forceinline__ bf16x8 get(const __bf16* tile, int row_base, int cc) const {
    return *reinterpret_cast<const bf16x8*>(tile + row_base * Tile<D>::LD + off[cc]);
  }
};

// Transposing reads: an MFMA operand whose contraction index runs down the rows.  Element e
// of the lane with column 32 db + lane % 32 is X[k_base + 8 (e / 4) + 4 hh + e % 4][column]
// (k_base a multiple of 16): the index permutation under which an MFMA result in registers
// is, unchanged, the other operand.
template <int D>
struct ColReader {
  int off[D / 32][2];
  __device__ __forceinline__ void init(int lane) {
    const int i = lane & 15, kr = i >> 2, hh = lane >> 5;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int hi = 0; hi < 2; ++hi)
        off[db][hi] = Tile<D>::off(4 * hh + kr + 8 * hi, 32 * db + ((lane >> 4) & 1) * 16 + 4 * (i & 3));
  }
  __device__ __forceinline__ bf16x8 get(const __bf16* tile, int k_base, int db) const {
    const __bf16* p = tile + k_base * Tile<D>::LD;
    return join(lds_read_tr(p + off[db][0]), lds_read_tr(p + off[db][1]));
  }
};

// Bounds-checked global loads.  A raw buffer descriptor covers `bytes` bytes from
// `base`; a 16-byte load at an offset at or past `bytes` returns zeros instead of
// touching memory, which replaces per-row predication (and its branches) when a
// tile hangs over the end of a sequence.  base and bytes must be wave-uniform.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  // readfirstlane pins the descriptor to scalar registers (no per-lane descriptor loop)
  const uint64_t b = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
  void* p = reinterpret_cast<void*>(((uint64_t)hi << 32) | lo);
  return __builtin_amdgcn_make_buffer_rsrc(p, 0, (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}

__device__ __forceinline__ u32x4 buffer_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_offset, 0, 0);
}

// Scheduling helpers.  A fence keeps the scheduler from moving anything across it; the
// group hints inside one fenced region ask for instruction classes in the given order,
// which is how MFMAs get interleaved with the LDS reads and arithmetic of another stage.
#define KNAP_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
#define KNAP_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
// Interleave n_mfma MFMAs with the LDS reads that feed them (reads_per_mfma each), keeping the
// reads `ahead` MFMAs in front of their use so that no MFMA waits out a full LDS latency.
#define KNAP_STREAM_READS(n_mfma, reads_per_mfma, ahead)                          \
  do {                                                                            \
    KNAP_SGB(KNAP_SG_DS_READ, (reads_per_mfma) * (ahead));                        \
    _Pragma("unroll") for (int i_ = 0; i_ < (n_mfma); ++i_) {                     \
      KNAP_SGB(KNAP_SG_MFMA, 1);                                                  \
      KNAP_SGB(KNAP_SG_DS_READ, (reads_per_mfma));                                \
    }                                                                             \
  } while (0)
#define KNAP_SG_VALU 0x002
#define KNAP_SG_MFMA 0x008
#define KNAP_SG_DS_READ 0x100
#define KNAP_SG_DS_WRITE 0x200

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float xor32(float x) {
  return __shfl_xor(x, 32, 64);
}

// round-to-nearest-even fp32 -> bf16 (the compiler selects v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3,
                                        float a4, float a5, float a6, float a7) {
  bf16x8 r;
  r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
  r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
  return r;
}

// Packs eight fp32 values into an MFMA operand and adds the eight ROUNDED values to `acc`
// (v_dot2c_f32_bf16 against ones).  Taking the row sum over the rounded probabilities, the
// ones the MFMA multiplies, makes the effective attention weights of a row sum to one exactly.
// The dot products are fed from the individually packed pairs: extracting dwords from the
// assembled 128-bit operand is miscompiled by this compiler (every extract reads dword 0).
__device__ __forceinline__ bf16x8 pack8_sum(float a0, float a1, float a2, float a3,
                                            float a4, float a5, float a6, float a7, float& acc) {
  bf16x2 ones;
  ones[0] = (__bf16)1.0f;
  ones[1] = (__bf16)1.0f;
  bf16x2 p0, p1, p2, p3;
  p0[0] = (__bf16)a0; p0[1] = (__bf16)a1;
  p1[0] = (__bf16)a2; p1[1] = (__bf16)a3;
  p2[0] = (__bf16)a4; p2[1] = (__bf16)a5;
  p3[0] = (__bf16)a6; p3[1] = (__bf16)a7;
  acc = __builtin_amdgcn_fdot2_f32_bf16(p0, ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(p1, ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(p2, ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(p3, ones, acc, false);
  u32x4 w;
  w[0] = __builtin_bit_cast(uint32_t, p0);
  w[1] = __builtin_bit_cast(uint32_t, p1);
  w[2] = __builtin_bit_cast(uint32_t, p2);
  w[3] = __builtin_bit_cast(uint32_t, p3);
  return __builtin_bit_cast(bf16x8, w);
}

__device__ __forceinline__ bf16x4 pack4(float a0, float a1, float a2, float a3) {
  bf16x4 r;
  r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
  return r;
}

// ---------------------------------------------------------------------------
// Tile schedule.  A work item is (sequence, head, tile of TILE rows).  Items
// are ordered by sequence length, longest first (an item's cost grows with the
// length of its sequence), then head, then tile, so that neighbouring items
// share one (sequence, head)'s K and V.  Every workgroup rebuilds the same
// schedule in LDS from cu_seqlens; the host never reads cu_seqlens.
//
// PAIRED (causal attention): the cost of a tile grows linearly with its index
// (query tiles) or falls linearly with it (key tiles), so tile p and tile
// tiles - 1 - p together cost the same for every p.  An item is then such a pair
// (the middle tile of an odd count stands alone), WorkItem::tile is p, and the
// items of one sequence are of equal cost again.
//
//   s_order[r]  original index of the r-th longest sequence
//   s_start[r]  first item of that sequence; s_start[n_seq] = number of items
// s_start doubles as the key array of the rank sort before it is filled.
// ---------------------------------------------------------------------------
struct WorkItem {
  int row0;   // first packed row of the sequence
  int len;    // its length
  int head;
  int tile;
};

template <bool PAIRED>
__device__ __forceinline__ int items_per_head(int tiles) { return PAIRED ? (tiles + 1) >> 1 : tiles; }

template <int TILE, int NT = kThreads, bool PAIRED = false>
__device__ __forceinline__ int build_schedule(const int32_t* __restrict__ cu, int n_seq, int H,
                                              int* s_order, int* s_start, int* s_part /* NT ints */) {
  constexpr int kThreads = NT;   // threads of the calling workgroup
  const int tid = threadIdx.x;
  for (int i = tid; i < n_seq; i += kThreads) s_start[i] = cu[i + 1] - cu[i];
  __syncthreads();
  // rank sort, descending length, ties by original index
  for (int i = tid; i < n_seq; i += kThreads) {
    const int li = s_start[i];
    int rank = 0;
    for (int j = 0; j < n_seq; ++j) {
      const int lj = s_start[j];
      rank += (lj > li) || (lj == li && j < i);
    }
    s_order[rank] = i;
  }
  __syncthreads();
  // exclusive prefix sum of items per sequence, in sorted order
  const int chunk = (n_seq + kThreads - 1) / kThreads;
  const int lo = min(tid * chunk, n_seq), hi = min(lo + chunk, n_seq);
  int local = 0;
  for (int r = lo; r < hi; ++r) {
    const int s = s_order[r];
    local += items_per_head<PAIRED>((cu[s + 1] - cu[s] + TILE - 1) / TILE) * H;
  }
  s_part[tid] = local;
  __syncthreads();
  for (int off = 1; off < kThreads; off <<= 1) {
    const int add = tid >= off ? s_part[tid - off] : 0;
    __syncthreads();
    s_part[tid] += add;
    __syncthreads();
  }
  int run = s_part[tid] - local;   // exclusive
  for (int r = lo; r < hi; ++r) {
    const int s = s_order[r];
    s_start[r] = run;
    run += items_per_head<PAIRED>((cu[s + 1] - cu[s] + TILE - 1) / TILE) * H;
  }
  if (tid == kThreads - 1) s_start[n_seq] = s_part[kThreads - 1];
  __syncthreads();
  return s_start[n_seq];
}

template <int TILE, bool PAIRED = false>
__device__ __forceinline__ WorkItem decode_item(int w, const int32_t* __restrict__ cu, int n_seq,
                                                const int* s_order, const int* s_start) {
  // largest r with s_start[r] <= w (sequences without items share their successor's start)
  int lo = 0, hi = n_seq - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (s_start[mid] <= w) lo = mid; else hi = mid - 1;
  }
  // every lane computed the same values; say so, so that addresses and buffer
  // descriptors derived from the item live in scalar registers
  const int s = __builtin_amdgcn_readfirstlane(s_order[lo]);
  const int first = __builtin_amdgcn_readfirstlane(s_start[lo]);
  WorkItem it;
  it.row0 = __builtin_amdgcn_readfirstlane(cu[s]);
  it.len = __builtin_amdgcn_readfirstlane(cu[s + 1]) - it.row0;
  const int per_head = items_per_head<PAIRED>((it.len + TILE - 1) / TILE);
  const int rem = w - first;
  it.head = rem / per_head;
  it.tile = rem - it.head * per_head;
  return it;
}

// Workgroups are handed to the 8 XCDs round-robin by blockIdx.  Renumber them
// so that the workgroups of one XCD take neighbouring work items and meet in
// that XCD's L2 on the same K and V.
__device__ __forceinline__ int xcd_major_block_id() {
  const int g = gridDim.x;
  const int b = blockIdx.x;
  return (g % 8 == 0) ? (b % 8) * (g / 8) + b / 8 : b;
}

// Static assignment of the descending-cost item list to G persistent workgroups: in round r
// workgroup wg takes item r G + wg, in odd rounds r G + (G - 1 - wg).  Dealing the rounds in
// serpentine order halves the imbalance of plain round-robin (whoever drew the dearest item of
// one round draws the cheapest of the next) and keeps neighbouring workgroups on neighbouring
// items.  Items at or past n_items (last round only) do not exist.
__device__ __forceinline__ int serpentine_item(int r, int wg, int G) {
  return r * G + ((r & 1) ? G - 1 - wg : wg);
}

// Dynamic assignment for kernels that are handed zeroed counters (one unsigned per XCD, 8 in
// all): the descending-cost item list is cut into chunks of G / 8 consecutive items, chunk j
// belongs to XCD j % 8 (so that the workgroups of an XCD keep meeting on the same K and V in its
// L2, and every XCD gets every eighth chunk of every cost band), and the workgroups of an XCD
// draw that XCD's items in order from its counter: list scheduling, longest first, within the
// XCD.  A ticket is the value the counter returned; the item of a ticket grows with the ticket,
// so the first ticket whose item is at or past n_items ends the workgroup.
struct ItemQueue {
  unsigned* ctr;
  int q, n_q, chunk;
  __device__ __forceinline__ void init(unsigned* counters) {
    n_q = (gridDim.x % 8 == 0) ? 8 : 1;
    q = (int)(blockIdx.x % n_q);                  // workgroups go to the XCDs round-robin
    chunk = max(1, (int)gridDim.x / n_q);
    ctr = counters + q;
  }
  __device__ __forceinline__ int item(int ticket) const {
    return ((ticket / chunk) * n_q + q) * chunk + ticket % chunk;
  }
};

}  // namespace knap
