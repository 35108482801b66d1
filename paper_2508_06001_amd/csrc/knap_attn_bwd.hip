// Backward kernels: gradients of sum(dout * out) with respect to q, k, v for
// packed block-diagonal attention, recomputing the probabilities from q, k and
// the forward's log-sum-exp (the training loop of Sec. 4 backpropagates through
// the attention of Sec. 3.4; Sec. 4.2 counts the backward as twice the forward,
// a recompute backward issues five contractions instead of four).
//
//   delta_i = sum_c dO_ic O_ic                       (preprocess kernel)
//   S = Q K^T, P = exp(scale S - LSE), dP = dO V^T, dS = P (dP - delta)
//   dV = P^T dO, dK = scale dS^T Q, dQ = scale dS K   (main kernel + dq convert)
//
// Main kernel: a persistent workgroup (4 waves) owns a 128-row key/value tile
// of one (sequence, head) and walks over that sequence's queries 64 rows at a
// time.  Wave w owns key columns [32 w, 32 w + 32): its K and V rows stay in
// registers as MFMA B operands, and its dK / dV rows accumulate in registers.
// With S = Q K^T in the MFMA result layout a lane holds one key column and its
// registers run over queries, so P and dS are, unchanged, the A operands of
// dV += P^T dO and dK += dS^T Q; dO and Q enter those as B operands through
// transposing LDS reads of the row-major tiles.  dQ contracts over keys, i.e.
// over lanes: dS takes one trip through LDS, after which wave w computes the
// dQ tile's 32-wide d slice over all 128 keys of the workgroup (K^T fragments
// for that slice stay in registers) and adds it to an fp32 accumulator in the
// workspace with hardware float atomics.
#include "knap_device.h"
#include "knap_kernels.h"

namespace knap {

template <int D>
struct BwdCfg {
  static constexpr int BM = 64;            // query rows per step
  static constexpr int BN = 128;           // key/value rows per workgroup
  static constexpr int MB = BM / 32;
  static constexpr int NB = D / 32;
  static constexpr int KC = D / 16;
  static constexpr int QS = D + 40;        // Q / dO tile row stride (elements); read both row-wise and transposed
  static constexpr int SS = BM + 40;       // dS tile [key][query] row stride
  static constexpr int KS = D + 32;        // K tile row stride (transposing reads only)
  static constexpr int DQ_BLOCKS = MB * NB;            // 32x32 blocks of the dQ tile
  static constexpr int DQ_PER_WAVE = DQ_BLOCKS / 4;    // blocks per wave (1 for d = 64, 2 for d = 128)
};

// delta[h][t] = sum_c dout[t][h][c] * out[t][h][c]; also clears the fp32 dq accumulator.
template <int D>
__global__ __launch_bounds__(kThreads) void attn_bwd_prep_kernel(
    const __bf16* __restrict__ out, const __bf16* __restrict__ dout, int64_t T, int H,
    float* __restrict__ delta, float* __restrict__ dq_acc) {
  constexpr int LPR = D / 8;   // lanes per (token, head) row, 8 elements each
  const int64_t n_rows = T * H;
  const int sub = threadIdx.x % LPR;
  for (int64_t row = (int64_t)blockIdx.x * (kThreads / LPR) + threadIdx.x / LPR; row < n_rows;
       row += (int64_t)gridDim.x * (kThreads / LPR)) {
    const size_t off = (size_t)row * D + sub * 8;
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(out + off);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(dout + off);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
#pragma unroll
    for (int s = 1; s < LPR; s <<= 1) acc += __shfl_xor(acc, s, 64);
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    *reinterpret_cast<f32x4*>(dq_acc + off) = z;
    *reinterpret_cast<f32x4*>(dq_acc + off + 4) = z;
    if (sub == 0) {
      const int64_t t = row / H;
      const int h = (int)(row - t * H);
      delta[(size_t)h * T + t] = acc;
    }
  }
}

// dq = bf16(scale * dq_acc)
__global__ __launch_bounds__(kThreads) void attn_bwd_dq_convert_kernel(
    const float* __restrict__ dq_acc, int64_t n8 /* groups of 8 elements */, float scale,
    __bf16* __restrict__ dq) {
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n8; i += (int64_t)gridDim.x * kThreads) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(dq_acc + i * 8);
    const f32x4 b = *reinterpret_cast<const f32x4*>(dq_acc + i * 8 + 4);
    *reinterpret_cast<bf16x8*>(dq + i * 8) =
        pack8(a[0] * scale, a[1] * scale, a[2] * scale, a[3] * scale,
              b[0] * scale, b[1] * scale, b[2] * scale, b[3] * scale);
  }
}

template <int D>
__global__ __launch_bounds__(kThreads, 1) void attn_bwd_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
    const __bf16* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ delta,
    const int32_t* __restrict__ cu, int n_seq, int H, float scale,
    float* __restrict__ dq_acc, __bf16* __restrict__ dk, __bf16* __restrict__ dv) {
  using C = BwdCfg<D>;
  extern __shared__ int s_dyn[];
  int* s_order = s_dyn;
  int* s_start = s_dyn + n_seq;
  __shared__ int s_part[kThreads];
  __shared__ __attribute__((aligned(16))) __bf16 sQ[C::BM * C::QS];
  __shared__ __attribute__((aligned(16))) __bf16 sdO[C::BM * C::QS];
  __shared__ __attribute__((aligned(16))) __bf16 sdS[C::BN * C::SS];
  __shared__ __attribute__((aligned(16))) __bf16 sK[C::BN * C::KS];
  __shared__ __attribute__((aligned(16))) float sLse[C::BM];     // LSE in base 2; +inf for rows past the end
  __shared__ __attribute__((aligned(16))) float sDelta[C::BM];

  const int n_items = build_schedule<C::BN>(cu, n_seq, H, s_order, s_start, s_part);
  const int T = cu[n_seq];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hh = lane >> 5;
  const float c = scale * kLog2e;
  const size_t row_stride = (size_t)H * D;

  constexpr int TPR = D / 8;
  constexpr int RPP = kThreads / TPR;
  const int ld_row = tid / TPR;
  const int ld_col = (tid % TPR) * 8;

  // dQ tile blocks of this wave: d slice nb, query blocks mb0 + j * MB_STEP
  const int dq_nb = wave % C::NB;
  const int dq_mb0 = wave / C::NB;
  constexpr int MB_STEP = 4 / C::NB > 0 ? 4 / C::NB : 1;   // 2 for d = 64, 1 for d = 128

  for (int w = xcd_major_block_id(); w < n_items; w += gridDim.x) {
    const WorkItem it = decode_item<C::BN>(w, cu, n_seq, s_order, s_start);
    const int L = it.len;
    const int kv0 = it.tile * C::BN;
    const size_t head_off = (size_t)it.head * D;
    const __bf16* q_base = q + (size_t)it.row0 * row_stride + head_off;
    const __bf16* do_base = dout + (size_t)it.row0 * row_stride + head_off;
    const __bf16* k_base = k + (size_t)it.row0 * row_stride + head_off;
    const __bf16* v_base = v + (size_t)it.row0 * row_stride + head_off;
    const float* lse_base = lse + (size_t)it.head * T + it.row0;
    const float* delta_base = delta + (size_t)it.head * T + it.row0;

    // this wave's key rows as B operands of S = Q K^T and dP = dO V^T
    const int kv_row = kv0 + 32 * wave + l32;
    const bool kv_valid = kv_row < L;
    bf16x8 kf[C::KC], vf[C::KC];
#pragma unroll
    for (int cc = 0; cc < C::KC; ++cc) {
      kf[cc] = kv_valid ? *reinterpret_cast<const bf16x8*>(k_base + (size_t)kv_row * row_stride + 16 * cc + 8 * hh)
                        : zero_bf16x8();
      vf[cc] = kv_valid ? *reinterpret_cast<const bf16x8*>(v_base + (size_t)kv_row * row_stride + 16 * cc + 8 * hh)
                        : zero_bf16x8();
    }

    // whole K tile through LDS once, to pick up K^T fragments for the dQ product
    __syncthreads();   // previous item no longer reads sK / sQ / sdO / sdS
#pragma unroll
    for (int p = 0; p < C::BN / RPP; ++p) {
      const int r = p * RPP + ld_row;
      u32x4 kk = {0u, 0u, 0u, 0u};
      if (kv0 + r < L) kk = *reinterpret_cast<const u32x4*>(k_base + (size_t)(kv0 + r) * row_stride + ld_col);
      *reinterpret_cast<u32x4*>(&sK[r * C::KS + ld_col]) = kk;
    }
    __syncthreads();
    bf16x8 ktf[C::BN / 16];   // element e of chunk ck: K[16 ck + 8 hh + e][32 dq_nb + l32]
#pragma unroll
    for (int ck = 0; ck < C::BN / 16; ++ck)
      ktf[ck] = lds_operand_tr(sK, C::KS, 16 * ck + 8 * hh, 16 * ck + 8 * hh + 4, 32 * dq_nb, lane);

    f32x16 dk_acc[C::NB], dv_acc[C::NB];
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb) { dk_acc[nb] = zero16(); dv_acc[nb] = zero16(); }

    for (int q0 = 0; q0 < L; q0 += C::BM) {
      __syncthreads();   // (A) the previous step's tiles are no longer being read
#pragma unroll
      for (int p = 0; p < C::BM / RPP; ++p) {
        const int r = p * RPP + ld_row;
        u32x4 qq = {0u, 0u, 0u, 0u}, dd = {0u, 0u, 0u, 0u};
        if (q0 + r < L) {
          const size_t g = (size_t)(q0 + r) * row_stride + ld_col;
          qq = *reinterpret_cast<const u32x4*>(q_base + g);
          dd = *reinterpret_cast<const u32x4*>(do_base + g);
        }
        *reinterpret_cast<u32x4*>(&sQ[r * C::QS + ld_col]) = qq;
        *reinterpret_cast<u32x4*>(&sdO[r * C::QS + ld_col]) = dd;
      }
      if (tid < C::BM) {
        const bool ok = q0 + tid < L;
        sLse[tid] = ok ? lse_base[q0 + tid] * kLog2e : INFINITY;   // +inf makes P = 0 on rows past the end
        sDelta[tid] = ok ? delta_base[q0 + tid] : 0.f;
      }
      __syncthreads();   // (B)

      // S and dP: (64 queries) x (this wave's 32 keys)
      f32x16 s[C::MB], dp[C::MB];
#pragma unroll
      for (int mb = 0; mb < C::MB; ++mb) {
        s[mb] = zero16();
        dp[mb] = zero16();
#pragma unroll
        for (int cc = 0; cc < C::KC; ++cc) {
          const int off = (32 * mb + l32) * C::QS + 16 * cc + 8 * hh;
          const bf16x8 aq = *reinterpret_cast<const bf16x8*>(&sQ[off]);
          const bf16x8 ad = *reinterpret_cast<const bf16x8*>(&sdO[off]);
          s[mb] = mfma32(aq, kf[cc], s[mb]);
          dp[mb] = mfma32(ad, vf[cc], dp[mb]);
        }
      }

      // P = exp2(c S - LSE2), dS = P (dP - delta); register r is query 32 mb + 8 (r / 4) + 4 hh + r % 4
#pragma unroll
      for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int qi = 32 * mb + 8 * g + 4 * hh;
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(&sLse[qi]);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(&sDelta[qi]);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p = fast_exp2(__builtin_fmaf(s[mb][4 * g + e], c, -l4[e]));
            s[mb][4 * g + e] = p;
            dp[mb][4 * g + e] = p * (dp[mb][4 * g + e] - d4[e]);
          }
          // dS to LDS as [key][query]: 4 consecutive queries per lane
          *reinterpret_cast<bf16x4*>(&sdS[(32 * wave + l32) * C::SS + qi]) =
              pack4(dp[mb][4 * g], dp[mb][4 * g + 1], dp[mb][4 * g + 2], dp[mb][4 * g + 3]);
        }

      // dV += P^T dO and dK += dS^T Q: contraction over queries in chunks of 16;
      // element e of chunk cq is query 16 cq + 8 (e / 4) + 4 hh + e % 4 on both sides
#pragma unroll
      for (int cq = 0; cq < C::BM / 16; ++cq) {
        const int mb = cq >> 1, r0 = 8 * (cq & 1);
        const bf16x8 pa = pack8(s[mb][r0], s[mb][r0 + 1], s[mb][r0 + 2], s[mb][r0 + 3],
                                s[mb][r0 + 4], s[mb][r0 + 5], s[mb][r0 + 6], s[mb][r0 + 7]);
        const bf16x8 da = pack8(dp[mb][r0], dp[mb][r0 + 1], dp[mb][r0 + 2], dp[mb][r0 + 3],
                                dp[mb][r0 + 4], dp[mb][r0 + 5], dp[mb][r0 + 6], dp[mb][r0 + 7]);
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) {
          const bf16x8 bo = lds_operand_tr(sdO, C::QS, 16 * cq + 4 * hh, 16 * cq + 8 + 4 * hh, 32 * nb, lane);
          const bf16x8 bq = lds_operand_tr(sQ, C::QS, 16 * cq + 4 * hh, 16 * cq + 8 + 4 * hh, 32 * nb, lane);
          dv_acc[nb] = mfma32(pa, bo, dv_acc[nb]);
          dk_acc[nb] = mfma32(da, bq, dk_acc[nb]);
        }
      }

      __syncthreads();   // (C) every wave's dS columns are in LDS

      // dQ tile block (query block mb, d slice dq_nb) = dS[:, all 128 keys] . K[:, slice]
#pragma unroll
      for (int j = 0; j < C::DQ_PER_WAVE; ++j) {
        const int mb = dq_mb0 + j * MB_STEP;
        f32x16 acc = zero16();
#pragma unroll
        for (int ck = 0; ck < C::BN / 16; ++ck) {
          const bf16x8 a = lds_operand_tr(sdS, C::SS, 16 * ck + 8 * hh, 16 * ck + 8 * hh + 4, 32 * mb, lane);
          acc = mfma32(a, ktf[ck], acc);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qi = q0 + 32 * mb + 8 * (r >> 2) + 4 * hh + (r & 3);
          if (qi < L)
            unsafeAtomicAdd(dq_acc + (size_t)(it.row0 + qi) * row_stride + head_off + 32 * dq_nb + l32, acc[r]);
        }
      }
    }

    // dK (scaled) and dV rows of this wave: register r is key 8 (r / 4) + 4 hh + r % 4, lane is d
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kv = kv0 + 32 * wave + 8 * (r >> 2) + 4 * hh + (r & 3);
        if (kv < L) {
          const size_t g = (size_t)(it.row0 + kv) * row_stride + head_off + 32 * nb + l32;
          dk[g] = (__bf16)(dk_acc[nb][r] * scale);
          dv[g] = (__bf16)dv_acc[nb][r];
        }
      }
  }
}

template <int D>
static hipError_t launch_bwd_t(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq, int H,
                               float scale, const void* out, const float* lse, const void* dout,
                               void* dq, void* dk, void* dv, int64_t T, float* delta, float* dq_acc,
                               int grid, int aux_grid, hipStream_t stream,
                               hipEvent_t ev_start, hipEvent_t ev_stop) {
  hipLaunchKernelGGL(attn_bwd_prep_kernel<D>, dim3(aux_grid), dim3(kThreads), 0, stream,
                     (const __bf16*)out, (const __bf16*)dout, T, H, delta, dq_acc);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t dyn = (size_t)(2 * n_seq + 1) * sizeof(int);
  if (ev_start && ev_stop && (e = hipEventRecord(ev_start, stream)) != hipSuccess) return e;
  hipLaunchKernelGGL(attn_bwd_kernel<D>, dim3(grid), dim3(kThreads), dyn, stream,
                     (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)dout, lse,
                     (const float*)delta, cu, n_seq, H, scale, dq_acc, (__bf16*)dk, (__bf16*)dv);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev_start && ev_stop && (e = hipEventRecord(ev_stop, stream)) != hipSuccess) return e;
  hipLaunchKernelGGL(attn_bwd_dq_convert_kernel, dim3(aux_grid), dim3(kThreads), 0, stream,
                     (const float*)dq_acc, T * H * D / 8, scale, (__bf16*)dq);
  return hipGetLastError();
}

hipError_t launch_bwd(const void* q, const void* k, const void* v, const int32_t* cu, int n_seq, int H, int d,
                      float scale, const void* out, const float* lse, const void* dout,
                      void* dq, void* dk, void* dv, int64_t T, float* delta, float* dq_acc,
                      int grid, int aux_grid, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (d == 64)
    return launch_bwd_t<64>(q, k, v, cu, n_seq, H, scale, out, lse, dout, dq, dk, dv, T, delta, dq_acc,
                            grid, aux_grid, stream, ev_start, ev_stop);
  return launch_bwd_t<128>(q, k, v, cu, n_seq, H, scale, out, lse, dout, dq, dk, dv, T, delta, dq_acc,
                           grid, aux_grid, stream, ev_start, ev_stop);
}

int bwd_workgroups_per_cu(int d) {
  int n = 0;
  hipError_t e = (d == 64)
      ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attn_bwd_kernel<64>, kThreads, 0)
      : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attn_bwd_kernel<128>, kThreads, 0);
  if (e != hipSuccess || n < 1) { (void)hipGetLastError(); n = 1; }
  return n;
}

}  // namespace knap
