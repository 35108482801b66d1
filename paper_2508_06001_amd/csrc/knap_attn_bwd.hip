// Backward kernels: gradients of sum(dout * out) with respect to q, k, v for
// packed block-diagonal attention, recomputing the probabilities from q, k and
// the forward's log-sum-exp (the training loop of Sec. 4 backpropagates through
// the attention of Sec. 3.4; Sec. 4.2 counts the backward as twice the forward).
//
//   delta_i = sum_c dO_ic O_ic                        (dQ kernel, which holds the dO rows of its queries anyway)
//   S = Q K^T, P = exp(scale S - LSE), dP = dO V^T, dS = P (dP - delta)
//   dQ = scale dS K                                    (dQ kernel, query-tile major; runs first)
//   dV = P^T dO, dK = scale dS^T Q                     (dK/dV kernel, key-tile major)
//
// dQ sums over keys and dK, dV sum over queries.  Doing all three in one pass
// needs a cross-workgroup reduction of one of them; on MI355X fp32 atomics into
// HBM-resident accumulators cap that design far below the MFMA rate (every
// atomic is a read-modify-write that leaves the XCD).  The backward is therefore
// two kernels that each keep their accumulators in registers and recompute S and
// dP: seven contractions are issued for the five the mathematics needs, nothing
// is reduced across workgroups, and the result is bitwise reproducible.
//
// dK/dV kernel: a persistent workgroup of 8 waves owns a 256-row key/value tile of one (sequence,
// head) and walks over that sequence's queries 32 rows at a time; wave pairs split the work by
// output (one wave S, P, dV; its partner dP, dS, dK, one tile behind) so that each wave holds a
// single accumulator and two waves fit on a SIMD.  Details at the kernel.
//
// dQ kernel: the forward kernel's structure.  S^T = K Q^T and dP^T = V dO^T put
// one query in each lane, LSE and delta are per-lane scalars, and dS^T is,
// unchanged, the B operand of dQ^T += K^T dS^T with K^T read transposed from LDS.
#include "knap_device.h"
#include "knap_kernels.h"

#include <type_traits>

namespace knap {

constexpr int kQueueCounters = 8;    // one work-queue counter per XCD for the dQ kernel

// the work queue of the dQ kernel, which follows on the stream, starts at zero
__global__ void bwd_queue_reset_kernel(unsigned* __restrict__ counters) {
  if (threadIdx.x < kQueueCounters) counters[threadIdx.x] = 0u;
}

// ---------------------------------------------------------------------------
// dK/dV kernel.  A persistent workgroup of 8 waves owns a 256-row key/value tile of one (sequence,
// head) and walks over that sequence's queries 32 rows at a time.  The waves form 4 pairs, pair i
// owning key rows [64 i, 64 i + 64) as two 32-row blocks; the two waves of a pair (placed on the same
// SIMD) split the work by output:
//   dV wave: keeps its K rows in registers, S = Q K^T, P = exp2(c S - LSE2), dV += P^T dO, and hands
//            the packed bf16 P to its partner through LDS (one way, double buffered);
//   dK wave: keeps its V rows in registers and runs ONE TILE BEHIND: dP = dO V^T, dS = P (dP - delta)
//            with the partner's P, dK += dS^T Q.
// Each wave holds one accumulator, so two waves fit on a SIMD and each one's MFMAs run against the
// other's exponentials, LDS reads and waits.  With S = Q K^T in the MFMA result layout a lane holds one
// key and its registers run over queries, so P and dS are, unchanged, the A operands of the second
// products; dO and Q enter those through transposing LDS reads.
//
// Every fragment of Q or dO that a wave reads from LDS, row-wise for S / dP and transposed for dV /
// dK, feeds TWO MFMAs, one per key block: 512 bytes of LDS operand per MFMA.  The registers just allow
// it because the accumulators sit on the key side: per wave 128 (dV or dK, 64 x d fp32) + 64 (its K or
// V rows) + 32 (scores of a step) + operands in flight, within the 256 of two waves per SIMD (every
// base address in scalar registers, every LDS address formed next to its read).
//
// Query-side tiles (32 rows of Q and dO, their LSE in base 2 and delta) go global -> LDS
// asynchronously, DEPTH tiles ahead, into a ring of DEPTH + 2 buffers (being filled / dV role / dK
// role).  The buffers are separate arrays and the loop is unrolled once around the ring, so that every
// LDS read names its buffer at compile time and is known not to depend on the copies in flight into
// the others; the waits are exact (vector-memory operations complete in issue order, every wave
// issues the same number per tile).  Rows past the end of the sequence arrive as zeros in all four
// (empty buffer descriptor): P = exp2(0 - 0) = 1 there, but dO = 0 and dP - delta = 0, so they add
// nothing to dV or dK.
//
// CAUSAL (query i sees keys 0..i): a key tile starting at row kv0 only meets the queries from row kv0
// on.  The walk over them runs BACKWARDS, from the sequence's last query tile down to the eight tiles
// that cross the diagonal (which get the mask): workgroups on different key tiles of one (sequence,
// head) then read the same query tiles at the same time, as they do without the mask, instead of each
// starting at its own diagonal.  Work items are pairs of key tiles of equal total cost (see
// build_schedule).
// ---------------------------------------------------------------------------
template <int D>
struct Bwd2Cfg {
  static constexpr int THREADS = 512;
  static constexpr int BM = 32;
  static constexpr int BN = 256;
  static constexpr int KB = 2;
  static constexpr int NB = D / 32;
  static constexpr int KC = D / 16;
  static constexpr int DEPTH = 3;
  static constexpr int NBUF = DEPTH + 2;
  static constexpr int TILE_ELEMS = BM * Tile<D>::LD;
  static constexpr int LOADS_PER_TILE = (D == 128 ? 2 : 1) + 1;
};

template <int N>
__device__ __forceinline__ void wait_vm_loads() {
  static_assert(N >= 0 && N < 64, "vmcnt is six bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Readers with ONE base register each: the swizzle is an XOR on the chunk index, so the offset of
// chunk pair cc of a row read is base ^ (32 cc) bytes-in-elements, and of (db, hi) of a transposing read
// (base ^ (32 db + 16 hi)) + 8 hi rows.
template <int D>
struct RowReaderX {
  int base;
  __device__ __forceinline__ void init(int lane) { base = 2 * Tile<D>::off(lane & 31, 8 * (lane >> 5)); }   // bytes
  // a copy of the base the optimizer cannot see through: what is derived from it stays in the step that
  // uses it (an address hoisted out of the loop would need a register of its own per buffer and chunk,
  // whereas formed next to its read the buffer's address becomes the read's immediate offset)
  __device__ __forceinline__ int fresh() const { int b = base; asm volatile("" : "+v"(b)); return b; }
  __device__ static __forceinline__ bf16x8 get(const __bf16* tile, int b, int cc) {
    return *reinterpret_cast<const bf16x8*>(reinterpret_cast<const char*>(tile) + (b ^ (32 * cc)));
  }
};
template <int D>
struct ColReaderX {
  int base;
  __device__ __forceinline__ void init(int lane) {
    const int i = lane & 15, kr = i >> 2, hh = lane >> 5;
    base = 2 * Tile<D>::off(4 * hh + kr, ((lane >> 4) & 1) * 16 + 4 * (i & 3));   // bytes
  }
  __device__ __forceinline__ int fresh() const { int b = base; asm volatile("" : "+v"(b)); return b; }
  __device__ static __forceinline__ bf16x8 get(const __bf16* tile, int b, int k_base, int db) {
    const char* p = reinterpret_cast<const char*>(tile + k_base * Tile<D>::LD);
    // rows 8 further down: at D = 128 the swizzle flips bit 1 of the chunk position there, at D = 64 bit 2
    // (the bit that db flips as well)
    return join(lds_read_tr(reinterpret_cast<const __bf16*>(p + (b ^ (64 * db)))),
                lds_read_tr(reinterpret_cast<const __bf16*>(p + ((b ^ (D == 128 ? 64 * db + 32 : 64 * (db ^ 1))) + 16 * Tile<D>::LD))));
  }
};

template <int D, bool CAUSAL>
__global__ __launch_bounds__(Bwd2Cfg<D>::THREADS, 2) void attn_bwd_dkdv64_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
    const __bf16* __restrict__ dout, const float* __restrict__ lse2, const float* __restrict__ delta,
    const int32_t* __restrict__ cu, int n_seq, int H, float scale,
    __bf16* __restrict__ dk, __bf16* __restrict__ dv) {
  using C = Bwd2Cfg<D>;
  extern __shared__ int s_dyn[];
  int* s_order = s_dyn;
  int* s_start = s_dyn + n_seq;
#define KNAP_RING(i)                                                                    \
  __shared__ __attribute__((aligned(1024))) __bf16 sQ##i[C::TILE_ELEMS];                \
  __shared__ __attribute__((aligned(1024))) __bf16 sdO##i[C::TILE_ELEMS];               \
  __shared__ __attribute__((aligned(256))) float sLse##i[64];                           \
  __shared__ __attribute__((aligned(256))) float sDelta##i[64];
  KNAP_RING(0) KNAP_RING(1) KNAP_RING(2) KNAP_RING(3) KNAP_RING(4)
#undef KNAP_RING
  __shared__ __attribute__((aligned(256))) float sSink[64];
  __shared__ __attribute__((aligned(16))) u32x4 sP[4][2][2 * C::KB][64];

  const int n_items = build_schedule<C::BN, C::THREADS, CAUSAL>(cu, n_seq, H, s_order, s_start, reinterpret_cast<int*>(&sP[0][0][0][0]));
  const int T = cu[n_seq];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int pair = wave & 3;
  const int role = wave >> 2;
  const int l32 = lane & 31;
  const int hh = lane >> 5;
  const float c = scale * kLog2e;
  const size_t row_stride = (size_t)H * D;
  const uint32_t row_bytes = (uint32_t)(row_stride * sizeof(__bf16));
  RowReaderX<D> rows;
  ColReaderX<D> cols;
  rows.init(lane);
  cols.init(lane);

  constexpr int ROWS_PER_INSTR = 512 / D;
  const int cp_row0 = (D == 128 ? wave : (wave & 3)) * ROWS_PER_INSTR;
  const int cp_row = cp_row0 + lane / Tile<D>::CPR;
  const uint32_t cp_off = (uint32_t)cp_row * row_bytes + (uint32_t)Tile<D>::chunk_pos(cp_row, lane % Tile<D>::CPR) * 16u;

  const int wg = xcd_major_block_id();
  for (int round = 0; round * (int)gridDim.x < n_items; ++round) {
    const int w = serpentine_item(round, wg, (int)gridDim.x);
    if (w >= n_items) continue;
    WorkItem it = decode_item<C::BN, CAUSAL>(w, cu, n_seq, s_order, s_start);
    // head and tile come out of a division, i.e. of vector instructions: say that they are wave-uniform, so
    // that every base address below lives in scalar registers
    it.head = __builtin_amdgcn_readfirstlane(it.head);
    it.tile = __builtin_amdgcn_readfirstlane(it.tile);
    const int L = it.len;
    const size_t head_off = (size_t)it.head * D;
    // CAUSAL: the item is the pair of key tiles {p, kv_tiles - 1 - p} (equal cost together, see build_schedule),
    // the one that meets more queries first; the middle tile of an odd count stands alone
    const int kv_tiles = (L + C::BN - 1) / C::BN;
    int sub = 0;
  second_tile_of_pair:;     // CAUSAL only: jumped back to once, from the end of the first tile
    const int kv_tile = (!CAUSAL || sub == 0) ? it.tile : kv_tiles - 1 - it.tile;
    const int kv0 = kv_tile * C::BN;
    // queries this key tile meets: rows q_first .. L - 1 of the sequence; tiles and rows below count from q_first
    const int q_first = CAUSAL ? kv0 : 0;
    const int Lq = L - q_first;
    const __bf16* q_base = q + (size_t)(it.row0 + q_first) * row_stride + head_off;
    const __bf16* do_base = dout + (size_t)(it.row0 + q_first) * row_stride + head_off;
    const float* lse_base = lse2 + (size_t)it.head * T + it.row0 + q_first;
    const float* delta_base = delta + (size_t)it.head * T + it.row0 + q_first;
    const int n_tiles = (Lq + C::BM - 1) / C::BM;
    // CAUSAL: step t works on query tile n_tiles - 1 - t: the walk runs BACKWARDS, from the sequence's last
    // query tile down to the eight tiles that cross the diagonal of this key tile (which get the mask), so
    // that workgroups on different key tiles of one (sequence, head) read the same query tiles at the same
    // time, as they do without the mask

    __syncthreads();

    bf16x8 kvf[C::KB][C::KC];
    {
      const uint32_t kv_bytes = (uint32_t)min(L - kv0, C::BN) * row_bytes;
      const __bf16* src = (role == 0 ? k : v) + (size_t)(it.row0 + kv0) * row_stride + head_off;
      const auto r = make_rsrc(src, kv_bytes);
#pragma unroll
      for (int kb = 0; kb < C::KB; ++kb) {
        const uint32_t off = (uint32_t)(64 * pair + 32 * kb + l32) * row_bytes + (uint32_t)(8 * hh) * 2u;
#pragma unroll
        for (int cc = 0; cc < C::KC; ++cc) kvf[kb][cc] = __builtin_bit_cast(bf16x8, buffer_load16(r, off + 32u * cc));
      }
    }

    f32x16 acc[C::KB][C::NB];
#pragma unroll
    for (int kb = 0; kb < C::KB; ++kb)
#pragma unroll
      for (int nb = 0; nb < C::NB; ++nb) acc[kb][nb] = zero16();

    auto issue_tile = [&](int t, __bf16* tQ, __bf16* tdO, float* tLse, float* tDelta) {
      int q0, n_rows;
      if constexpr (CAUSAL) {
        q0 = max(0, n_tiles - 1 - t) * C::BM;
        n_rows = t < n_tiles ? min(Lq - q0, C::BM) : 0;
      } else {
        q0 = t * C::BM;
        n_rows = max(0, min(L - q0, C::BM));
      }
      const auto rq = make_rsrc(q_base + (size_t)q0 * row_stride, (uint32_t)n_rows * row_bytes);
      const auto rd = make_rsrc(do_base + (size_t)q0 * row_stride, (uint32_t)n_rows * row_bytes);
      if constexpr (D == 128) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rq, (__attribute__((address_space(3))) void*)(tQ + cp_row0 * Tile<D>::LD), 16, (int)cp_off, 0, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rd, (__attribute__((address_space(3))) void*)(tdO + cp_row0 * Tile<D>::LD), 16, (int)cp_off, 0, 0, 0);
      } else {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(wave < 4 ? rq : rd,
            (__attribute__((address_space(3))) void*)((wave < 4 ? tQ : tdO) + cp_row0 * Tile<D>::LD), 16, (int)cp_off, 0, 0, 0);
      }
      const float* src = wave == 0 ? lse_base + q0 : delta_base + q0;
      float* dst = wave == 0 ? tLse : wave == 1 ? tDelta : sSink;
      const auto rs = make_rsrc(src, wave < 2 ? (uint32_t)n_rows * 4u : 0u);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)dst, 4, lane * 4, 0, 0, 0);
    };

    // End of a step: this wave's copies of the next tile have landed (all but the (DEPTH - 1) tiles requested
    // after it), its LDS writes (P) are done, then the workgroup barrier.  A bare s_barrier: __syncthreads()
    // would wait for EVERY copy in flight (its release fence covers the asynchronous LDS writes) and cut the
    // prefetch distance to one tile.  The empty asm statements keep the compiler from moving LDS accesses
    // across the barrier.
    auto step_sync = [&]() {
      wait_vm_loads<(C::DEPTH - 1) * C::LOADS_PER_TILE>();
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    };

    // Both roles share one shape of step, written as an explicit software pipeline (scheduling fences
    // between the groups, so that the order below is the order issued): LDS fragments are requested
    // AHEAD groups before the MFMAs that use them, and the arithmetic of the second half of the tile
    // (16 queries) is cut into slices that sit between the MFMAs of the first half.
    constexpr int AHEAD = 2;
    // first product: x[kb] = sum over d of tile rows (A, from LDS) x this wave's K or V rows (B, registers / LDS)
    auto first_product = [&](const __bf16* tA, int rb, f32x16 (&x)[C::KB]) {
      bf16x8 af[C::KC];
#pragma unroll
      for (int cc = 0; cc < AHEAD; ++cc) af[cc] = rows.get(tA, rb, cc);
      KNAP_SCHED_FENCE();
#pragma unroll
      for (int cc = 0; cc < C::KC; ++cc) {
#pragma unroll
        for (int kb = 0; kb < C::KB; ++kb) x[kb] = mfma32(af[cc], kvf[kb][cc], x[kb]);
        if (cc + AHEAD < C::KC) af[cc + AHEAD] = rows.get(tA, rb, cc + AHEAD);
        KNAP_SCHED_FENCE();
      }
    };
    // second product over the 16 queries of chunk cq: acc[kb][nb] += op[kb] (A, registers) x tile columns (B, LDS),
    // with `between(nb)` issued after the MFMAs of column block nb
    auto second_product = [&](const __bf16* tB, int cb, int cq, const bf16x8 (&op)[C::KB], auto between) {
      bf16x8 bf[C::NB];
      constexpr int AH2 = 2;
#pragma unroll
      for (int nb = 0; nb < AH2; ++nb) bf[nb] = cols.get(tB, cb, 16 * cq, nb);
      KNAP_SCHED_FENCE();
#pragma unroll
      for (int nb = 0; nb < C::NB; ++nb) {
#pragma unroll
        for (int kb = 0; kb < C::KB; ++kb) acc[kb][nb] = mfma32(op[kb], bf[nb], acc[kb][nb]);
        if (nb + AH2 < C::NB) bf[nb + AH2] = cols.get(tB, cb, 16 * cq, nb + AH2);
        between(nb);
        KNAP_SCHED_FENCE();
      }
    };

    // dV wave, tile t: S, P, hand P over, dV += P^T dO
    auto dv_step = [&](int t, const __bf16* tQ, const __bf16* tdO, const float* tLse) {
      const int rb = rows.fresh(), cb = cols.fresh();
      f32x16 s[C::KB];
#pragma unroll
      for (int kb = 0; kb < C::KB; ++kb) s[kb] = zero16();
      first_product(tQ, rb, s);
      // P = exp2(c S - LSE2); register r of a key block is query 8 (r / 4) + 4 hh + r % 4, chunk cq holds
      // registers 8 cq .. 8 cq + 7, slice (kb, half) four of them
      bf16x8 pa[2][C::KB];
      bf16x4 ph[2][C::KB][2];
      f32x4 lq[2][2];
      auto lse_of = [&](int cq) {
        lq[cq][0] = *reinterpret_cast<const f32x4*>(&tLse[16 * cq + 4 * hh]);
        lq[cq][1] = *reinterpret_cast<const f32x4*>(&tLse[16 * cq + 8 + 4 * hh]);
      };
      // CAUSAL, tiles that cross the diagonal (the first eight from q_first): a query before this lane's key
      // gets P = 0.  Counted from the tile's first query, the lane's key of block kb is the first one that
      // query `first_seen[kb]` sees.
      bool diag = false;
      int first_seen[C::KB];
      if constexpr (CAUSAL) {
        diag = n_tiles - 1 - t < C::BN / C::BM;
#pragma unroll
        for (int kb = 0; kb < C::KB; ++kb) first_seen[kb] = 64 * pair + 32 * kb + l32 - (n_tiles - 1 - t) * C::BM - 4 * hh;
      }
      auto exp_slice = [&](int cq, int kb, int half) {
        float p[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) p[e] = fast_exp2(__builtin_fmaf(s[kb][8 * cq + 4 * half + e], c, -lq[cq][half][e]));
        if constexpr (CAUSAL) {
          if (diag) {
#pragma unroll
            for (int e = 0; e < 4; ++e) p[e] = 8 * (2 * cq + half) + e < first_seen[kb] ? 0.f : p[e];
          }
        }
        ph[cq][kb][half] = pack4(p[0], p[1], p[2], p[3]);
        if (half == 1) {
          pa[cq][kb] = join(ph[cq][kb][0], ph[cq][kb][1]);
          sP[pair][t & 1][2 * kb + cq][lane] = __builtin_bit_cast(u32x4, pa[cq][kb]);
        }
      };
      lse_of(0);
#pragma unroll
      for (int j = 0; j < 2 * C::KB; ++j) exp_slice(0, j >> 1, j & 1);
      lse_of(1);
      KNAP_SCHED_FENCE();
      second_product(tdO, cb, 0, pa[0], [&](int nb) {
        // 2 KB slices of the second chunk spread over NB groups
        if constexpr (C::NB == 4) exp_slice(1, nb >> 1, nb & 1);
        else { exp_slice(1, nb, 0); exp_slice(1, nb, 1); }
      });
      second_product(tdO, cb, 1, pa[1], [&](int) {});
    };
    // dK wave, tile u: dP, dS = P (dP - delta) with the partner's P, dK += dS^T Q
    auto dk_step = [&](int u, const __bf16* tQ, const __bf16* tdO, const float* tDelta) {
      const int rb = rows.fresh();
      f32x16 dp[C::KB];
#pragma unroll
      for (int kb = 0; kb < C::KB; ++kb) dp[kb] = zero16();
      first_product(tdO, rb, dp);
      const int cb = cols.fresh();
      bf16x8 da[2][C::KB];
      bf16x4 dh[2][C::KB][2];
      f32x4 dq4[2][2];
      u32x4 pw[2][C::KB];
      auto fetch_of = [&](int cq) {
        dq4[cq][0] = *reinterpret_cast<const f32x4*>(&tDelta[16 * cq + 4 * hh]);
        dq4[cq][1] = *reinterpret_cast<const f32x4*>(&tDelta[16 * cq + 8 + 4 * hh]);
#pragma unroll
        for (int kb = 0; kb < C::KB; ++kb) pw[cq][kb] = sP[pair][u & 1][2 * kb + cq][lane];
      };
      auto ds_slice = [&](int cq, int kb, int half) {
        float ds[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t word = pw[cq][kb][2 * half + (e >> 1)];
          const float p = __builtin_bit_cast(float, (e & 1) ? (word & 0xffff0000u) : (word << 16));
          ds[e] = p * (dp[kb][8 * cq + 4 * half + e] - dq4[cq][half][e]);
        }
        dh[cq][kb][half] = pack4(ds[0], ds[1], ds[2], ds[3]);
        if (half == 1) da[cq][kb] = join(dh[cq][kb][0], dh[cq][kb][1]);
      };
      fetch_of(0);
#pragma unroll
      for (int j = 0; j < 2 * C::KB; ++j) ds_slice(0, j >> 1, j & 1);
      fetch_of(1);
      KNAP_SCHED_FENCE();
      second_product(tQ, cb, 0, da[0], [&](int nb) {
        if constexpr (C::NB == 4) ds_slice(1, nb >> 1, nb & 1);
        else { ds_slice(1, nb, 0); ds_slice(1, nb, 1); }
      });
      second_product(tQ, cb, 1, da[1], [&](int) {});
    };

    // Each role runs its own copy of the loop over the steps: with the roles as branches inside one
    // loop the accumulators would be merged at every step's join, and the register allocator then keeps
    // two sets.  Every wave still executes the same sequence of copies, waits and barriers.
#define KNAP_STEP(ROLE, t, cur, prev, nxt)                                                    \
    do {                                                                                      \
      issue_tile((t) + C::DEPTH, sQ##nxt, sdO##nxt, sLse##nxt, sDelta##nxt);                  \
      if constexpr (ROLE == 0) {                                                              \
        if ((t) < n_tiles) dv_step((t), sQ##cur, sdO##cur, sLse##cur);                        \
      } else {                                                                                \
        if ((t) >= 1) dk_step((t) - 1, sQ##prev, sdO##prev, sDelta##prev);                    \
      }                                                                                       \
      step_sync();                                                                            \
    } while (0)
#define KNAP_ROLE_LOOP(ROLE)                                                                  \
    do {                                                                                      \
      int t = 0;                                                                              \
      for (; t + 4 <= n_tiles; t += 5) {                                                      \
        KNAP_STEP(ROLE, t, 0, 4, 3);                                                          \
        KNAP_STEP(ROLE, t + 1, 1, 0, 4);                                                      \
        KNAP_STEP(ROLE, t + 2, 2, 1, 0);                                                      \
        KNAP_STEP(ROLE, t + 3, 3, 2, 1);                                                      \
        KNAP_STEP(ROLE, t + 4, 4, 3, 2);                                                      \
      }                                                                                       \
      if (t <= n_tiles) {                                                                     \
        KNAP_STEP(ROLE, t, 0, 4, 3);                                                          \
        if (t + 1 <= n_tiles) {                                                               \
          KNAP_STEP(ROLE, t + 1, 1, 0, 4);                                                    \
          if (t + 2 <= n_tiles) {                                                             \
            KNAP_STEP(ROLE, t + 2, 2, 1, 0);                                                  \
            if (t + 3 <= n_tiles) KNAP_STEP(ROLE, t + 3, 3, 2, 1);                            \
          }                                                                                   \
        }                                                                                     \
      }                                                                                       \
    } while (0)

    issue_tile(0, sQ0, sdO0, sLse0, sDelta0);
    issue_tile(1, sQ1, sdO1, sLse1, sDelta1);
    issue_tile(2, sQ2, sdO2, sLse2, sDelta2);
    step_sync();      // tile 0 has landed (and the K / V rows requested before it)

    if (role == 0) KNAP_ROLE_LOOP(0);
    else KNAP_ROLE_LOOP(1);
#undef KNAP_ROLE_LOOP
#undef KNAP_STEP
    wait_vm_loads<0>();

    __bf16* dst = role == 0 ? dv : dk;
    const float out_scale = role == 0 ? 1.0f : scale;
#pragma unroll
    for (int kb = 0; kb < C::KB; ++kb)
#pragma unroll
      for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kv0 + 64 * pair + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
          if (kv < L)
            dst[(size_t)(it.row0 + kv) * row_stride + head_off + 32 * nb + l32] = (__bf16)(acc[kb][nb][r] * out_scale);
        }
    if constexpr (CAUSAL) {
      if (sub == 0 && it.tile != kv_tiles - 1 - it.tile) {   // not the middle tile of an odd count
        sub = 1;
        goto second_tile_of_pair;
      }
    }
  }
}

template <int D>
struct DqCfg {
  static constexpr int BM = 128;         // query rows per work item
  static constexpr int BN = 64;          // key/value rows per LDS tile
  static constexpr int KC = D / 16;
  static constexpr int DB = D / 32;
  static constexpr int TILE_ELEMS = BN * Tile<D>::LD;
};

template <int D, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
    const __bf16* __restrict__ out, const __bf16* __restrict__ dout, const float* __restrict__ lse,
    float* __restrict__ delta, float* __restrict__ lse2_out, const int32_t* __restrict__ cu, int n_seq, int H, float scale,
    __bf16* __restrict__ dq, unsigned* __restrict__ counters) {
  using C = DqCfg<D>;
  extern __shared__ int s_dyn[];
  int* s_order = s_dyn;
  int* s_start = s_dyn + n_seq;
  // K is read row-wise (S^T) and transposed (dQ^T), V row-wise (dP^T); two buffers each, as
  // separate arrays so that reads of one are known not to depend on the copy into the other
  __shared__ __attribute__((aligned(1024))) __bf16 sK0[C::TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) __bf16 sK1[C::TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) __bf16 sV0[C::TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) __bf16 sV1[C::TILE_ELEMS];
  static_assert(sizeof(__bf16) * C::TILE_ELEMS >= sizeof(int) * kThreads, "scan scratch must fit in a tile");

  const int n_items = build_schedule<C::BM, kThreads, CAUSAL>(cu, n_seq, H, s_order, s_start, reinterpret_cast<int*>(&sK0[0]));
  const int T = cu[n_seq];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_u = CAUSAL ? __builtin_amdgcn_readfirstlane(wave) : 0;   // the same number, known to be wave-uniform
  const int l32 = lane & 31;
  const int hh = lane >> 5;
  const float c = scale * kLog2e;
  const size_t row_stride = (size_t)H * D;
  const uint32_t row_bytes = (uint32_t)(row_stride * sizeof(__bf16));
  RowReader<D> rows;     // K and V tile rows -> A operands of S^T and dP^T
  ColReader<D> cols;     // K tile columns -> A operands of dQ^T += K^T dS^T
  rows.init(lane);
  cols.init(lane);

  // Work items come from this XCD's queue.  The ticket for the NEXT item is requested right
  // after the item's first loads (vector-memory operations complete in issue order: requested
  // before them, the slow counter update would hold up the whole prologue) and only looked at
  // when the item is done, so the counter's latency is never waited for.
  __shared__ int s_ticket;
  ItemQueue queue;
  queue.init(counters);
  if (tid == 0) s_ticket = (int)atomicAdd(queue.ctr, 1u);
  __syncthreads();
  for (;;) {
    const int w = queue.item(__builtin_amdgcn_readfirstlane(s_ticket));
    if (w >= n_items) break;
    const WorkItem it = decode_item<C::BM, CAUSAL>(w, cu, n_seq, s_order, s_start);
    const int L = it.len;
    const size_t head_off = (size_t)it.head * D;
    unsigned next_ticket;      // thread 0 only; no initial value, which would be merged in (and waited for) at once
    // CAUSAL: the item is the pair of query tiles {q_tiles - 1 - p, p}, the long one first
    const int q_tiles = (L + C::BM - 1) / C::BM;
    int sub = 0;
  second_tile_of_pair:;     // CAUSAL only: jumped back to once, from the end of the first tile
    const int q_tile = !CAUSAL ? it.tile : sub == 0 ? q_tiles - 1 - it.tile : it.tile;
    const int q0 = q_tile * C::BM;
    const int q_row = q0 + wave * 32 + l32;
    const bool q_valid = q_row < L;
    // keys this query tile sees at all
    const int kv_end = CAUSAL ? min(L, q0 + C::BM) : L;

    // this lane's q and dO rows as B operands (rows past the end read as zero), and
    // delta = sum_c dO_c O_c of its query: the lane holds half of the row's elements (8 of every 16),
    // its partner at lane ^ 32 the other half.  The dK/dV kernel reads delta from memory afterwards.
    bf16x8 qf[C::KC], dof[C::KC];
    float dl = 0.f;
    {
      const uint32_t bytes = (uint32_t)min(L - q0, C::BM) * row_bytes;
      const auto rq = make_rsrc(q + (size_t)(it.row0 + q0) * row_stride + head_off, bytes);
      const auto rd = make_rsrc(dout + (size_t)(it.row0 + q0) * row_stride + head_off, bytes);
      const auto ro = make_rsrc(out + (size_t)(it.row0 + q0) * row_stride + head_off, bytes);
      const uint32_t off = (uint32_t)(wave * 32 + l32) * row_bytes + (uint32_t)(8 * hh) * 2u;
      bf16x8 of[C::KC];
#pragma unroll
      for (int cc = 0; cc < C::KC; ++cc) {
        qf[cc] = __builtin_bit_cast(bf16x8, buffer_load16(rq, off + 32u * cc));
        dof[cc] = __builtin_bit_cast(bf16x8, buffer_load16(rd, off + 32u * cc));
        of[cc] = __builtin_bit_cast(bf16x8, buffer_load16(ro, off + 32u * cc));
      }
#pragma unroll
      for (int cc = 0; cc < C::KC; ++cc)
#pragma unroll
        for (int e = 0; e < 8; ++e) dl = __builtin_fmaf((float)dof[cc][e], (float)of[cc][e], dl);
      dl += xor32(dl);
    }
    // per-lane scalars of this lane's query; +inf LSE turns rows past the end into P = 0
    const int q_idx = q_valid ? q_row : 0;
    const float lse_raw = lse[(size_t)it.head * T + it.row0 + q_idx];
    const float lse2 = q_valid ? lse_raw * kLog2e : INFINITY;
    if (q_valid && hh == 0) {     // for the dK/dV kernel: delta, and the LSE in base 2 (it copies both straight into LDS)
      delta[(size_t)it.head * T + it.row0 + q_row] = dl;
      lse2_out[(size_t)it.head * T + it.row0 + q_row] = lse_raw * kLog2e;
    }

    f32x16 acc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db) acc[db] = zero16();

    const __bf16* k_base = k + (size_t)it.row0 * row_stride + head_off;
    const __bf16* v_base = v + (size_t)it.row0 * row_stride + head_off;
    const int n_tiles = (kv_end + C::BN - 1) / C::BN;

    // asynchronous; rows past the end arrive as zeros and add nothing to dQ
    auto load_tile = [&](int t, __bf16* dK, __bf16* dV) {
      const int kv0 = t * C::BN;
      const uint32_t bytes = (uint32_t)max(0, min(kv_end - kv0, C::BN)) * row_bytes;
      tile_load_async<D>(dK, make_rsrc(k_base + (size_t)kv0 * row_stride, bytes), row_bytes, C::BN, wave, lane);
      tile_load_async<D>(dV, make_rsrc(v_base + (size_t)kv0 * row_stride, bytes), row_bytes, C::BN, wave, lane);
    };

    // One tile: 64 keys as two halves of 32, one after the other (the register file is full with
    // the q and dO fragments and the dQ accumulator; the second wave of the SIMD fills the gaps).
    // Within a half the LDS reads are streamed a few MFMAs ahead of their use.
    // MODE 2: the tile crosses the causal diagonal; keys after this lane's query get dS = 0, and a wave
    // whose 32 queries all precede the tile's first key has nothing to do in it.
    // MODE 1: the ragged last tile; the scores of keys past the end of the sequence start (and stay) at
    // -inf, so P = 0 and dS = 0 there.  Their K and V rows arrive as zeros: left at score 0, P would be
    // exp2(-LSE2), which overflows for a query whose scores are all far below zero, and the product of
    // that dS with the zero K row would be NaN.
    auto process_tile = [&](auto mode_tag, int t, const __bf16* tK, const __bf16* tV, __bf16* nK, __bf16* nV) {
      constexpr int MODE = decltype(mode_tag)::value;
      constexpr bool DIAG = MODE == 2;
      load_tile(t + 1, nK, nV);
      if (!(DIAG && t * C::BN > q0 + 32 * wave_u + 31)) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        f32x16 s = zero16(), dp = zero16();
        if constexpr (MODE == 1) {
          const int first_past = L - t * C::BN - 32 * half - 4 * hh;   // counted from this half's first key
#pragma unroll
          for (int r = 0; r < 16; ++r) s[r] = 8 * (r >> 2) + (r & 3) >= first_past ? -INFINITY : 0.f;
        }
#pragma unroll
        for (int cc = 0; cc < C::KC; ++cc) {
          s = mfma32(rows.get(tK, 32 * half, cc), qf[cc], s);
          dp = mfma32(rows.get(tV, 32 * half, cc), dof[cc], dp);
        }
        // K^T fragments of the first 16 keys are requested before the arithmetic
        bf16x8 kt0[C::DB];
#pragma unroll
        for (int db = 0; db < C::DB; ++db) kt0[db] = cols.get(tK, 32 * half, db);
        KNAP_STREAM_READS(2 * C::KC, 1, 4);
        KNAP_SCHED_FENCE();
        // dS^T = P^T (dP^T - delta), P^T = exp2(c S^T - LSE2); element e of chunk ck is key
        // 32 half + 16 ck + 8 (e / 4) + 4 hh + e % 4
        float ds[16];
        const int last_seen = q_row - t * C::BN - 32 * half - 4 * hh;   // counted from this half's first key
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float x = fast_exp2(__builtin_fmaf(s[r], c, -lse2)) * (dp[r] - dl);
          ds[r] = (DIAG && 8 * (r >> 2) + (r & 3) > last_seen) ? 0.f : x;
        }
        const bf16x8 d0 = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
        const bf16x8 d1 = pack8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
        KNAP_SCHED_FENCE();
#pragma unroll
        for (int db = 0; db < C::DB; ++db) acc[db] = mfma32(kt0[db], d0, acc[db]);
#pragma unroll
        for (int db = 0; db < C::DB; ++db) acc[db] = mfma32(cols.get(tK, 32 * half + 16, db), d1, acc[db]);
        KNAP_SGB(KNAP_SG_DS_READ, 2 * C::DB);          // the second chunk's K^T fragments go out first
        KNAP_SGB(KNAP_SG_MFMA, 2 * C::DB);
        KNAP_SCHED_FENCE();
      }
      }
      wait_async_loads();
      __syncthreads();     // next tile visible; this tile no longer read
    };

    __syncthreads();       // the previous item (or the schedule build) is done with both buffers
    load_tile(0, sK0, sV0);
    wait_async_loads();
    if (tid == 0 && sub == 0) next_ticket = atomicAdd(queue.ctr, 1u);
    __syncthreads();
    constexpr std::integral_constant<int, 0> plain{};
    constexpr std::integral_constant<int, 1> ragged_end{};
    constexpr std::integral_constant<int, 2> diagonal{};
    if constexpr (!CAUSAL) {
      const bool ragged = (L % C::BN) != 0;
      const int n_full = ragged ? n_tiles - 1 : n_tiles;
      for (int t = 0; t < n_full; t += 2) {
        process_tile(plain, t, sK0, sV0, sK1, sV1);
        if (t + 1 < n_full) process_tile(plain, t + 1, sK1, sV1, sK0, sV0);
      }
      if (ragged) {     // one instantiation for either buffer: the tile after the last is never loaded (empty descriptor)
        const bool odd = (n_tiles - 1) & 1;
        process_tile(ragged_end, n_tiles - 1, odd ? sK1 : sK0, odd ? sV1 : sV0, odd ? sK0 : sK1, odd ? sV0 : sV1);
      }
    } else {
      // tiles 0 .. 2 q_tile - 1 lie below the diagonal (an even count: the pair loop ends on buffer 0);
      // tiles 2 q_tile and, if the sequence reaches it, 2 q_tile + 1 cross it
      const int n_below = 2 * q_tile;
      for (int t = 0; t < n_below; t += 2) {
        process_tile(plain, t, sK0, sV0, sK1, sV1);
        process_tile(plain, t + 1, sK1, sV1, sK0, sV0);
      }
      process_tile(diagonal, n_below, sK0, sV0, sK1, sV1);
      if (n_below + 1 < n_tiles) process_tile(diagonal, n_below + 1, sK1, sV1, sK0, sV0);
    }

    if (q_valid) {
      __bf16* o_ptr = dq + (size_t)(it.row0 + q_row) * row_stride + head_off;
#pragma unroll
      for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 pk = pack4(acc[db][4 * g] * scale, acc[db][4 * g + 1] * scale,
                                  acc[db][4 * g + 2] * scale, acc[db][4 * g + 3] * scale);
          *reinterpret_cast<bf16x4*>(o_ptr + 32 * db + 8 * g + 4 * hh) = pk;
        }
    }
    if constexpr (CAUSAL) {
      if (sub == 0 && it.tile != q_tiles - 1 - it.tile) {   // not the middle tile of an odd count
        sub = 1;
        goto second_tile_of_pair;
      }
    }
    if (tid == 0) s_ticket = (int)next_ticket;   // every wave took its copy of the old ticket many barriers ago
    __syncthreads();
  }
}

template <int D, bool CAUSAL>
static hipError_t launch_bwd_t(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq, int H,
                               float scale, const void* out, const float* lse, const void* dout,
                               void* dq, void* dk, void* dv, float* delta, float* lse2, unsigned* counters,
                               int grid_dkdv, int grid_dq, hipStream_t stream,
                               hipEvent_t ev_start, hipEvent_t ev_stop) {
  hipLaunchKernelGGL(bwd_queue_reset_kernel, dim3(1), dim3(64), 0, stream, counters);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t dyn = (size_t)(2 * n_seq + 1) * sizeof(int);
  // the dQ kernel also produces delta, which the dK/dV kernel needs: it goes first
  hipLaunchKernelGGL((attn_bwd_dq_kernel<D, CAUSAL>), dim3(grid_dq), dim3(kThreads), dyn, stream,
                     (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)out,
                     (const __bf16*)dout, lse, delta, lse2, cu, n_seq, H, scale, (__bf16*)dq, counters);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev_start && ev_stop && (e = hipEventRecord(ev_start, stream)) != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_dkdv64_kernel<D, CAUSAL>), dim3(grid_dkdv), dim3(Bwd2Cfg<D>::THREADS), dyn, stream,
                     (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)dout,
                     (const float*)lse2, (const float*)delta, cu, n_seq, H, scale, (__bf16*)dk, (__bf16*)dv);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev_start && ev_stop && (e = hipEventRecord(ev_stop, stream)) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t launch_bwd(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq, int H, int d,
                      float scale, bool causal, const void* out, const float* lse, const void* dout,
                      void* dq, void* dk, void* dv, float* delta, float* lse2, unsigned* counters,
                      int grid_dkdv, int grid_dq, hipStream_t stream,
                      hipEvent_t ev_start, hipEvent_t ev_stop) {
#define KNAP_BWD_ARGS q, k, v, cu, n_seq, H, scale, out, lse, dout, dq, dk, dv, delta, lse2, counters, \
                      grid_dkdv, grid_dq, stream, ev_start, ev_stop
  if (causal) return d == 64 ? launch_bwd_t<64, true>(KNAP_BWD_ARGS) : launch_bwd_t<128, true>(KNAP_BWD_ARGS);
  return d == 64 ? launch_bwd_t<64, false>(KNAP_BWD_ARGS) : launch_bwd_t<128, false>(KNAP_BWD_ARGS);
#undef KNAP_BWD_ARGS
}

static int occupancy_of(const void* fn, int threads = kThreads) {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, fn, threads, 0) != hipSuccess || n < 1) {
    (void)hipGetLastError();
    n = 1;
  }
  return n;
}

int bwd_dkdv_workgroups_per_cu(int d) {
  return occupancy_of(d == 64 ? (const void*)attn_bwd_dkdv64_kernel<64, false> : (const void*)attn_bwd_dkdv64_kernel<128, false>,
                      Bwd2Cfg<128>::THREADS);
}

int bwd_dq_workgroups_per_cu(int d) {
  return occupancy_of(d == 64 ? (const void*)attn_bwd_dq_kernel<64, false> : (const void*)attn_bwd_dq_kernel<128, false>);
}

}  // namespace knap
