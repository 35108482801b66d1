// Forward kernel: out = softmax(scale q k^T) v per (sequence, head) of a packed
// bag, with the row log-sum-exp (Sec. 3.4 / the attention listing of Sec. 3.5:
// full bidirectional attention inside each sequence, none across sequences).
//
// One persistent workgroup (4 waves) takes work items (sequence, head, 128-row
// query tile) from the longest-first schedule.  Wave w owns 32 query rows and
// streams the sequence's keys and values through LDS in tiles of 64 rows.
//
// Orientation: the scores are computed transposed, S^T = K Q^T, so that in the
// MFMA result layout a lane holds ONE query (column l % 32) and its registers
// run over keys.  Row max and row sum are then in-register reductions plus one
// exchange between lanes l and l ^ 32, the rescale factor is a per-lane scalar,
// and P^T in that layout is, unchanged, the B operand of O^T += V^T P^T.  V^T
// fragments come from the row-major V tile through transposing LDS reads.
#include "knap_device.h"
#include "knap_kernels.h"

namespace knap {

template <int D>
struct FwdCfg {
  static constexpr int BM = 128;         // query rows per work item
  static constexpr int BN = 64;          // key/value rows per LDS tile
  static constexpr int KS = D + 8;       // K tile row stride (elements): +16 B keeps 128-bit row reads conflict-free
  static constexpr int VS = D + 32;      // V tile row stride: +64 B spreads the 4-row transposing reads over all banks
  static constexpr int KC = D / 16;      // contraction chunks over d
  static constexpr int DB = D / 32;      // 32-wide blocks of d
};

template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
    const int32_t* __restrict__ cu, int n_seq, int H, float scale,
    __bf16* __restrict__ out, float* __restrict__ lse) {
  using C = FwdCfg<D>;
  extern __shared__ int s_dyn[];
  int* s_order = s_dyn;
  int* s_start = s_dyn + n_seq;
  __shared__ int s_part[kThreads];
  __shared__ __attribute__((aligned(16))) __bf16 sK[C::BN * C::KS];
  __shared__ __attribute__((aligned(16))) __bf16 sV[C::BN * C::VS];

  const int n_items = build_schedule<C::BM>(cu, n_seq, H, s_order, s_start, s_part);
  const int T = cu[n_seq];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hh = lane >> 5;
  const float c = scale * kLog2e;
  const size_t row_stride = (size_t)H * D;

  // global -> LDS tile copy geometry: 16 B per thread
  constexpr int TPR = D / 8;                 // threads per row
  constexpr int RPP = kThreads / TPR;        // rows per pass
  const int ld_row = tid / TPR;
  const int ld_col = (tid % TPR) * 8;

  for (int w = xcd_major_block_id(); w < n_items; w += gridDim.x) {
    const WorkItem it = decode_item<C::BM>(w, cu, n_seq, s_order, s_start);
    const int L = it.len;
    const int q_row = it.tile * C::BM + wave * 32 + l32;      // row inside the sequence
    const bool q_valid = q_row < L;
    const __bf16* q_ptr = q + (size_t)(it.row0 + q_row) * row_stride + (size_t)it.head * D;

    bf16x8 qf[C::KC];
#pragma unroll
    for (int cc = 0; cc < C::KC; ++cc)
      qf[cc] = q_valid ? *reinterpret_cast<const bf16x8*>(q_ptr + 16 * cc + 8 * hh) : zero_bf16x8();

    f32x16 o[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db) o[db] = zero16();
    float m_run = -INFINITY;   // running max of the raw scores
    float l_run = 0.f;         // this lane's share of the running sum (its 32 of the 64 keys per tile)

    const __bf16* k_base = k + (size_t)it.row0 * row_stride + (size_t)it.head * D;
    const __bf16* v_base = v + (size_t)it.row0 * row_stride + (size_t)it.head * D;

    for (int kv0 = 0; kv0 < L; kv0 += C::BN) {
      __syncthreads();   // the previous tile is no longer being read
#pragma unroll
      for (int p = 0; p < C::BN / RPP; ++p) {
        const int r = p * RPP + ld_row;
        const bool ok = kv0 + r < L;
        const size_t g = (size_t)(kv0 + r) * row_stride + ld_col;
        u32x4 kk = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
        if (ok) {
          kk = *reinterpret_cast<const u32x4*>(k_base + g);
          vv = *reinterpret_cast<const u32x4*>(v_base + g);
        }
        *reinterpret_cast<u32x4*>(&sK[r * C::KS + ld_col]) = kk;
        *reinterpret_cast<u32x4*>(&sV[r * C::VS + ld_col]) = vv;
      }
      __syncthreads();

      // S^T (64 keys x 32 queries) = K tile . Q^T
      f32x16 s[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        s[mb] = zero16();
#pragma unroll
        for (int cc = 0; cc < C::KC; ++cc) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(&sK[(32 * mb + l32) * C::KS + 16 * cc + 8 * hh]);
          s[mb] = mfma32(a, qf[cc], s[mb]);
        }
      }
      if (kv0 + C::BN > L) {   // ragged last tile: keys past the end of the sequence
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kv = kv0 + 32 * mb + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (kv >= L) s[mb][r] = -INFINITY;
          }
      }

      // online softmax, base 2
      float m_loc = s[0][0];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) m_loc = fmaxf(m_loc, s[mb][r]);
      m_loc = fmaxf(m_loc, xor32(m_loc));
      const float m_new = fmaxf(m_run, m_loc);      // finite: every tile holds at least one valid key
      const float alpha = fast_exp2((m_run - m_new) * c);
      const float mc = m_new * c;
      float l_loc = 0.f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = fast_exp2(__builtin_fmaf(s[mb][r], c, -mc));
          s[mb][r] = p;
          l_loc += p;
        }
      l_run = l_run * alpha + l_loc;
      m_run = m_new;
#pragma unroll
      for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;

      // O^T (d x 32 queries) += V^T P^T.  Chunk cc contracts 16 keys; element e of a
      // lane's operand is key 16 cc + 8 (e / 4) + 4 hh + e % 4 on both sides.
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const int mb = cc >> 1, r0 = 8 * (cc & 1);
        const bf16x8 pb = pack8(s[mb][r0], s[mb][r0 + 1], s[mb][r0 + 2], s[mb][r0 + 3],
                                s[mb][r0 + 4], s[mb][r0 + 5], s[mb][r0 + 6], s[mb][r0 + 7]);
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
          const bf16x8 a = lds_operand_tr(sV, C::VS, 16 * cc + 4 * hh, 16 * cc + 8 + 4 * hh, 32 * db, lane);
          o[db] = mfma32(a, pb, o[db]);
        }
      }
    }

    // epilogue: normalise, store out (bf16) and lse (natural log)
    const float l_tot = l_run + xor32(l_run);
    const float inv = 1.0f / l_tot;
    if (q_valid) {
      __bf16* o_ptr = out + (size_t)(it.row0 + q_row) * row_stride + (size_t)it.head * D;
#pragma unroll
      for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 pk = pack4(o[db][4 * g] * inv, o[db][4 * g + 1] * inv,
                                  o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
          *reinterpret_cast<bf16x4*>(o_ptr + 32 * db + 8 * g + 4 * hh) = pk;
        }
      if (hh == 0) lse[(size_t)it.head * T + it.row0 + q_row] = m_run * scale + __logf(l_tot);
    }
  }
}

template <int D>
static hipError_t launch_fwd_t(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq,
                               int H, float scale, void* out, float* lse, int grid, hipStream_t stream) {
  const size_t dyn = (size_t)(2 * n_seq + 1) * sizeof(int);
  hipLaunchKernelGGL(attn_fwd_kernel<D>, dim3(grid), dim3(kThreads), dyn, stream,
                     (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, cu, n_seq, H, scale,
                     (__bf16*)out, lse);
  return hipGetLastError();
}

hipError_t launch_fwd(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq,
                      int H, int d, float scale, void* out, float* lse, int grid, hipStream_t stream) {
  if (d == 64) return launch_fwd_t<64>(q, k, v, cu, n_seq, H, scale, out, lse, grid, stream);
  return launch_fwd_t<128>(q, k, v, cu, n_seq, H, scale, out, lse, grid, stream);
}

int fwd_workgroups_per_cu(int d) {
  int n = 0;
  hipError_t e = (d == 64)
      ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attn_fwd_kernel<64>, kThreads, 0)
      : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attn_fwd_kernel<128>, kThreads, 0);
  if (e != hipSuccess || n < 1) { (void)hipGetLastError(); n = 1; }
  return n;
}

}  // namespace knap
