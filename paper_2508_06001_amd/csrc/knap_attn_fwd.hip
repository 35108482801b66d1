// Forward kernel: out = softmax(scale q k^T) v per (sequence, head) of a packed
// bag, with the row log-sum-exp (Sec. 3.4 / the attention listing of Sec. 3.5:
// full bidirectional attention inside each sequence, none across sequences).
// CAUSAL is the other mask the paper admits inside a datum (Limitations
// paragraph): query i sees keys 0..i of its own sequence.
//
// One persistent workgroup (4 waves) takes work items (sequence, head, 128-row
// query tile) from the longest-first schedule.  Wave w owns 32 query rows and
// streams the sequence's keys and values through LDS in tiles of 64 rows; the
// next tile is copied global -> LDS asynchronously (no staging registers) into
// the other buffer while the current one is used, behind one barrier per tile.
//
// Orientation: the scores are computed transposed, S^T = K Q^T, so that in the
// MFMA result layout a lane holds ONE query (column l % 32) and its registers
// run over keys.  Row max and row sum are then in-register reductions plus one
// exchange between lanes l and l ^ 32, the rescale factor is a per-lane scalar,
// and P^T in that layout is, unchanged, the B operand of O^T += V^T P^T.  V^T
// fragments come from the row-major V tile through transposing LDS reads.
//
// Softmax bookkeeping: the exponent reference m_ref of a query only moves when
// a tile's maximum exceeds it by more than 2^8 in base-2 units (the first tile
// always does).  Otherwise P is formed against the old reference, so P <= 256
// and the accumulated output needs no rescaling; the final division by the row
// sum removes the reference exactly as in the textbook recurrence.  The row sum
// is taken over the bf16-rounded P that the MFMA multiplies, so the effective
// weights of a row sum to one exactly (a one-hot row returns its v bit for bit);
// the stored log-sum-exp inherits at most a 2^-9 relative change of that sum.
#include "knap_device.h"
#include "knap_kernels.h"

#include <type_traits>

namespace knap {

template <int D>
struct FwdCfg {
  static constexpr int BM = 128;         // query rows per work item
  static constexpr int BN = 64;          // key/value rows per LDS tile
  static constexpr int KC = D / 16;      // contraction chunks over d
  static constexpr int DB = D / 32;      // 32-wide blocks of d
  static constexpr int TILE_ELEMS = BN * Tile<D>::LD;
};

constexpr float kRescaleThreshold = 8.0f;   // base-2 units
constexpr int kFwdQueueSlots = 256;

template <int D, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
    const int32_t* __restrict__ cu, int n_seq, int H, float scale,
    __bf16* __restrict__ out, float* __restrict__ lse, unsigned* __restrict__ counters) {
  using C = FwdCfg<D>;
  using TL = Tile<D>;
  extern __shared__ int s_dyn[];
  int* s_order = s_dyn;
  int* s_start = s_dyn + n_seq;
  // separate arrays (not one indexed array) so that reads of one buffer are known not to
  // depend on the asynchronous copy into the other
  __shared__ __attribute__((aligned(1024))) __bf16 sK0[C::TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) __bf16 sK1[C::TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) __bf16 sV0[C::TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) __bf16 sV1[C::TILE_ELEMS];
  static_assert(sizeof(__bf16) * C::TILE_ELEMS >= sizeof(int) * kThreads, "scan scratch must fit in a tile");

  // the scan scratch of the schedule lives in the first K buffer, which is not in use yet
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
  RowReader<D> k_rows;   // K tile rows -> A operands of S^T
  ColReader<D> v_cols;   // V tile columns -> A operands of O^T += V^T P^T
  k_rows.init(lane);
  v_cols.init(lane);

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
    const int q_row = q0 + wave * 32 + l32;      // row inside the sequence
    const bool q_valid = q_row < L;
    // keys this query tile sees at all
    const int kv_end = CAUSAL ? min(L, q0 + C::BM) : L;

    // this lane's query row as the B operand of S^T = K Q^T (rows past the end read as zero)
    bf16x8 qf[C::KC];
    {
      const auto rq = make_rsrc(q + (size_t)(it.row0 + q0) * row_stride + head_off,
                                (uint32_t)min(L - q0, C::BM) * row_bytes);
      const uint32_t off = (uint32_t)(wave * 32 + l32) * row_bytes + (uint32_t)(8 * hh) * 2u;
#pragma unroll
      for (int cc = 0; cc < C::KC; ++cc) qf[cc] = __builtin_bit_cast(bf16x8, buffer_load16(rq, off + 32u * cc));
    }

    f32x16 o[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db) o[db] = zero16();
    float m_ref = -INFINITY;   // exponent reference (raw score units)
    float l_run = 0.f;         // this lane's share of the row sum (its 32 of the 64 keys per tile)

    const __bf16* k_base = k + (size_t)it.row0 * row_stride + head_off;
    const __bf16* v_base = v + (size_t)it.row0 * row_stride + head_off;
    const int n_tiles = (kv_end + C::BN - 1) / C::BN;

    auto load_tile = [&](int t, __bf16* dK, __bf16* dV) {   // asynchronous; a tile past the end arrives as zeros
      const int kv0 = t * C::BN;
      const uint32_t bytes = (uint32_t)max(0, min(kv_end - kv0, C::BN)) * row_bytes;
      tile_load_async<D>(dK, make_rsrc(k_base + (size_t)kv0 * row_stride, bytes), row_bytes, C::BN, wave, lane);
      tile_load_async<D>(dV, make_rsrc(v_base + (size_t)kv0 * row_stride, bytes), row_bytes, C::BN, wave, lane);
    };

    // One tile: 64 keys as two halves of 32.  MODE 1 is the ragged last tile, MODE 2 a tile that
    // crosses the causal diagonal (for rows of the sequence that mask covers the ragged end too).
    // A wave whose 32 queries all precede the tile's first key has nothing to do in it.
    auto process_tile = [&](int t, auto mode_tag, const __bf16* tK, const __bf16* tV, __bf16* nK, __bf16* nV) {
      constexpr int MODE = decltype(mode_tag)::value;
      load_tile(t + 1, nK, nV);
      if (!(MODE == 2 && t * C::BN > q0 + 32 * wave_u + 31)) {

      bf16x8 ak0[C::KC], ak1[C::KC];
#pragma unroll
      for (int cc = 0; cc < C::KC; ++cc) ak0[cc] = k_rows.get(tK, 0, cc);
      KNAP_SCHED_FENCE();

      f32x16 s0, s1;
      if constexpr (MODE != 0) {   // keys past the end of the sequence, or after the query, start (and stay) at -inf
        const int kv0 = t * C::BN;
        const int kv_lim = MODE == 2 ? q_row + 1 : L;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kv0 + 8 * (r >> 2) + 4 * hh + (r & 3);
          s0[r] = kv < kv_lim ? 0.f : -INFINITY;
          s1[r] = kv + 32 < kv_lim ? 0.f : -INFINITY;
        }
      } else {
        s0 = zero16();
        s1 = zero16();
      }
      // slot 1: S^T of keys 0..31 | K fragments of keys 32..63
#pragma unroll
      for (int cc = 0; cc < C::KC; ++cc) s0 = mfma32(ak0[cc], qf[cc], s0);
#pragma unroll
      for (int cc = 0; cc < C::KC; ++cc) ak1[cc] = k_rows.get(tK, 32, cc);
#pragma unroll
      for (int i = 0; i < C::KC; ++i) { KNAP_SGB(KNAP_SG_MFMA, 1); KNAP_SGB(KNAP_SG_DS_READ, 1); }
      KNAP_SCHED_FENCE();

      // slot 2: S^T of keys 32..63 | max over keys 0..31, V^T fragments of keys 0..31
      bf16x8 vt0[2][C::DB], vt1[2][C::DB];
#pragma unroll
      for (int cc = 0; cc < C::KC; ++cc) s1 = mfma32(ak1[cc], qf[cc], s1);
      float m_loc = s0[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) m_loc = fmaxf(m_loc, s0[r]);
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
          vt0[0][db] = v_cols.get(tV, 0, db);
#pragma unroll
      for (int i = 0; i < C::KC; ++i) { KNAP_SGB(KNAP_SG_MFMA, 1); KNAP_SGB(KNAP_SG_DS_READ, 1); KNAP_SGB(KNAP_SG_VALU, 2); }
      KNAP_SCHED_FENCE();

#pragma unroll
      for (int r = 0; r < 16; ++r) m_loc = fmaxf(m_loc, s1[r]);
      m_loc = fmaxf(m_loc, xor32(m_loc));
      // move the reference only when the tile maximum is far above it (always on the first tile)
      if (__builtin_amdgcn_ballot_w64((m_loc - m_ref) * c > kRescaleThreshold) != 0) {
        const float m_new = fmaxf(m_ref, m_loc);
        const float alpha = fast_exp2((m_ref - m_new) * c);
        m_ref = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      }
      const float mc = m_ref * c;

      // P^T of a half, packed: element e of chunk ck is key 16 ck + 8 (e / 4) + 4 hh + e % 4
      auto exps = [&](const f32x16& s, bf16x8 (&pb)[2]) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) p[r] = fast_exp2(__builtin_fmaf(s[r], c, -mc));
#pragma unroll
        for (int ck = 0; ck < 2; ++ck) {
          const int r0 = 8 * ck;
          pb[ck] = pack8_sum(p[r0], p[r0 + 1], p[r0 + 2], p[r0 + 3], p[r0 + 4], p[r0 + 5], p[r0 + 6], p[r0 + 7], l_run);
        }
      };
      bf16x8 pb0[2], pb1[2];
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
          vt0[1][db] = v_cols.get(tV, 16, db);
      exps(s0, pb0);
      KNAP_SCHED_FENCE();

      // slot 3: O^T += V^T P^T over keys 0..31 | P^T of keys 32..63, V^T fragments of keys 32..47
#pragma unroll
      for (int ck = 0; ck < 2; ++ck)
#pragma unroll
        for (int db = 0; db < C::DB; ++db) o[db] = mfma32(vt0[ck][db], pb0[ck], o[db]);
      exps(s1, pb1);
#pragma unroll
      for (int db = 0; db < C::DB; ++db) vt1[0][db] = v_cols.get(tV, 32, db);
#pragma unroll
      for (int i = 0; i < 2 * C::DB; ++i) { KNAP_SGB(KNAP_SG_MFMA, 1); KNAP_SGB(KNAP_SG_DS_READ, 1); KNAP_SGB(KNAP_SG_VALU, 8); }
      KNAP_SCHED_FENCE();

      // slot 4: O^T += V^T P^T over keys 32..63 | V^T fragments of keys 48..63
#pragma unroll
      for (int db = 0; db < C::DB; ++db) vt1[1][db] = v_cols.get(tV, 48, db);
#pragma unroll
      for (int ck = 0; ck < 2; ++ck)
#pragma unroll
        for (int db = 0; db < C::DB; ++db) o[db] = mfma32(vt1[ck][db], pb1[ck], o[db]);
#pragma unroll
      for (int i = 0; i < C::DB; ++i) { KNAP_SGB(KNAP_SG_DS_READ, 2); KNAP_SGB(KNAP_SG_MFMA, 1); }
      KNAP_SCHED_FENCE();
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
        process_tile(t, plain, sK0, sV0, sK1, sV1);
        if (t + 1 < n_full) process_tile(t + 1, plain, sK1, sV1, sK0, sV0);
      }
      if (ragged) {
        if ((n_tiles - 1) & 1) process_tile(n_tiles - 1, ragged_end, sK1, sV1, sK0, sV0);
        else process_tile(n_tiles - 1, ragged_end, sK0, sV0, sK1, sV1);
      }
    } else {
      // tiles 0 .. 2 q_tile - 1 lie below the diagonal (an even count: the pair loop ends on buffer 0);
      // tiles 2 q_tile and, if the sequence reaches it, 2 q_tile + 1 cross it
      const int n_below = 2 * q_tile;
      for (int t = 0; t < n_below; t += 2) {
        process_tile(t, plain, sK0, sV0, sK1, sV1);
        process_tile(t + 1, plain, sK1, sV1, sK0, sV0);
      }
      process_tile(n_below, diagonal, sK0, sV0, sK1, sV1);
      if (n_below + 1 < n_tiles) process_tile(n_below + 1, diagonal, sK1, sV1, sK0, sV0);
    }

    // epilogue: normalise, store out (bf16) and lse (natural log)
    const float l_tot = l_run + xor32(l_run);
    const float inv = 1.0f / l_tot;
    if (q_valid) {
      __bf16* o_ptr = out + (size_t)(it.row0 + q_row) * row_stride + head_off;
#pragma unroll
      for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 pk = pack4(o[db][4 * g] * inv, o[db][4 * g + 1] * inv,
                                  o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
          *reinterpret_cast<bf16x4*>(o_ptr + 32 * db + 8 * g + 4 * hh) = pk;
        }
      if (hh == 0) lse[(size_t)it.head * T + it.row0 + q_row] = m_ref * scale + __logf(l_tot);
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

// instantiated in this order (the bidirectional kernels first)
#define KNAP_FWD_INSTANCE(D, CAUSAL)                                                                    \
  template __global__ void attn_fwd_kernel<D, CAUSAL>(const __bf16*, const __bf16*, const __bf16*,      \
                                                      const int32_t*, int, int, float, __bf16*, float*, \
                                                      unsigned*);
KNAP_FWD_INSTANCE(64, false)
KNAP_FWD_INSTANCE(128, false)
KNAP_FWD_INSTANCE(64, true)
KNAP_FWD_INSTANCE(128, true)
#undef KNAP_FWD_INSTANCE

// The forward entry point has no workspace argument, so the counters of its work queue live
// in the library's device image: kFwdQueueSlots sets of 8 (one per XCD), handed out in rotation
// by the host and zeroed on the launch stream right before the kernel that uses them.  Two
// launches share a set only if kFwdQueueSlots other forward launches were enqueued between
// them while the first was still running.
static __device__ __align__(256) unsigned g_fwd_queue[kFwdQueueSlots * 8];

__global__ void fwd_queue_reset_kernel(unsigned* __restrict__ counters) {
  if (threadIdx.x < 8) counters[threadIdx.x] = 0u;
}

int fwd_queue_slots() { return kFwdQueueSlots; }

unsigned* fwd_queue_base() {
  unsigned* p = nullptr;
  if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(g_fwd_queue)) != hipSuccess) {
    (void)hipGetLastError();
    return nullptr;
  }
  return p;
}

template <int D, bool CAUSAL>
static hipError_t launch_fwd_t(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq,
                               int H, float scale, void* out, float* lse, unsigned* counters, int grid,
                               hipStream_t stream) {
  hipLaunchKernelGGL(fwd_queue_reset_kernel, dim3(1), dim3(64), 0, stream, counters);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t dyn = (size_t)(2 * n_seq + 1) * sizeof(int);
  hipLaunchKernelGGL((attn_fwd_kernel<D, CAUSAL>), dim3(grid), dim3(kThreads), dyn, stream,
                     (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, cu, n_seq, H, scale,
                     (__bf16*)out, lse, counters);
  return hipGetLastError();
}

hipError_t launch_fwd(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq,
                      int H, int d, float scale, bool causal, void* out, float* lse, unsigned* counters, int grid,
                      hipStream_t stream) {
  if (!causal) {
    if (d == 64) return launch_fwd_t<64, false>(q, k, v, cu, n_seq, H, scale, out, lse, counters, grid, stream);
    return launch_fwd_t<128, false>(q, k, v, cu, n_seq, H, scale, out, lse, counters, grid, stream);
  }
  if (d == 64) return launch_fwd_t<64, true>(q, k, v, cu, n_seq, H, scale, out, lse, counters, grid, stream);
  return launch_fwd_t<128, true>(q, k, v, cu, n_seq, H, scale, out, lse, counters, grid, stream);
}

int fwd_workgroups_per_cu(int d) {
  int n = 0;
  hipError_t e = (d == 64)
      ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attn_fwd_kernel<64, false>, kThreads, 0)
      : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attn_fwd_kernel<128, false>, kThreads, 0);
  if (e != hipSuccess || n < 1) { (void)hipGetLastError(); n = 1; }
  return n;
}

}  // namespace knap
