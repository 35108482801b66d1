/* libknapattn: packed variable-length joint self-attention for MI355X (gfx950),
 * forward and backward, plus the host-side workload model and greedy balancer
 * of KnapFormer (arXiv 2508.06001).
 *
 * Plain C ABI.  No C++ or framework types cross this boundary.
 *
 * Conventions for every function that returns int: 0 (KNAP_OK) on success, a
 * negative KNAP_ERR_* otherwise.  Nothing aborts, throws or prints.
 */
#ifndef KNAPATTN_H
#define KNAPATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KNAP_OK                        0
#define KNAP_ERR_INVALID_ARG          -1  /* null pointer, bad size, unsupported head dim, misaligned pointer */
#define KNAP_ERR_WORKSPACE_TOO_SMALL  -2
#define KNAP_ERR_LAUNCH_FAILED        -3  /* the HIP runtime refused a launch; see knap_last_hip_error() */
#define KNAP_ERR_TOO_MANY_SEQS        -4  /* n_seq above KNAP_MAX_SEQS */
#define KNAP_ERR_CAPACITY             -5  /* an output array of a host function is too small */
#define KNAP_ERR_PARSE                -6  /* malformed topology string */
#define KNAP_ERR_SCRATCH_TOO_SMALL    -7  /* the bag exceeds the library's own scratch (knap_varlen_attn_bwd_noalloc) */

/* Largest number of sequences in one packed bag.  Every workgroup rebuilds the
 * tile schedule from cu_seqlens in LDS, which bounds the bag size. */
#define KNAP_MAX_SEQS 2048

/* ------------------------------------------------------------------------
 * Attention.  Defined by Sec. 3.4 and the attention listing of Sec. 3.5 of
 * the paper: packed q, k, v of shape (l1+...+ln, h, d) and the list of
 * sequence lengths; each sequence attends only to itself (bidirectional, no
 * mask inside a sequence; "Limitations" paragraph).  Eq. 1's 4 l^2 d term is
 * this operation's FLOP count.
 *
 * Layout.  q, k, v, out, dout, dq, dk, dv: bf16, shape (T, H, d), d fastest,
 * contiguous, T = cu_seqlens[n_seq].  lse: fp32, shape (H, T): the natural
 * log of sum_j exp(scale * q_i . k_j) over the keys of row i's sequence.
 * cu_seqlens: int32[n_seq + 1], cu[0] = 0, non-decreasing (zero-length
 * sequences are legal and skipped).  Its contents live on the device and are
 * NOT validated (that would need a synchronisation): a non-monotone array is
 * a caller error with undefined results.
 *
 * Memory.  Every pointer is a DEVICE pointer owned by the caller, 16-byte
 * aligned.  The library never allocates, frees or synchronises: all work is
 * enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 * stream) and the call returns at once.  Outputs are fully overwritten for
 * rows < T; inputs are never modified; outputs must not alias inputs.
 *
 * Supported: d in {64, 128}; 0 <= n_seq <= KNAP_MAX_SEQS; H >= 1; scale positive
 * and finite; T < 2^31.
 * n_seq == 0 succeeds and enqueues nothing.  With n_seq > 0 every pointer must be
 * non-null even if all sequences are empty (T = 0): the host cannot see T.
 * ------------------------------------------------------------------------ */

/* out = softmax(scale * q k^T) v per (sequence, head); also writes lse.
 *
 * Concurrency.  The kernel draws its work items from counters that live in the
 * library's device image: 256 sets, each cleared on `stream` right before the
 * kernel that uses it.  Eager launches take sets 0..127 in rotation: calls from
 * several threads and on several streams may overlap freely as long as no more
 * than 128 eager forward launches are in flight on a device at the same time.
 * A launch recorded under stream capture takes one of sets 128..255 and keeps
 * it for every replay of its graph, so replays never share a set with eager
 * launches; two captured launches share a set only once more than 128 forward
 * launches have been captured in the process, and graphs that hold such a pair
 * must then not be replayed at the same time.  The first call on a device (it
 * looks up device properties, once, under a lock) must not be made under
 * stream capture; later calls may be captured. */
int knap_varlen_attn_fwd(const void* q, const void* k, const void* v,
                         const int32_t* cu_seqlens, int n_seq,
                         int H, int d, float scale,
                         void* out, float* lse,
                         void* stream);

/* Gradients of sum(dout * out) with respect to q, k, v, recomputing the
 * probabilities from q, k and lse (as produced by the forward call).
 *
 * `total_tokens` must equal cu_seqlens[n_seq]; it sizes the launches and the
 * workspace because the host cannot read cu_seqlens without synchronising.
 * `workspace` is caller-owned device scratch of at least
 * knap_varlen_attn_bwd_workspace_bytes(total_tokens, n_seq, H, d) bytes,
 * 256-byte aligned; its contents on entry are ignored and on return are
 * unspecified.  It holds the per-row dot products of dout and out, the
 * log-sum-exp in base 2 and the counters of the kernels' work queues, so two
 * calls that may run at the same time (different streams) need a workspace
 * each. */
int knap_varlen_attn_bwd(const void* q, const void* k, const void* v,
                         const int32_t* cu_seqlens, int n_seq,
                         int H, int d, float scale,
                         const void* out, const float* lse,
                         const void* dout,
                         void* dq, void* dk, void* dv,
                         int64_t total_tokens,
                         void* workspace, size_t workspace_bytes,
                         void* stream);

size_t knap_varlen_attn_bwd_workspace_bytes(int64_t total_tokens, int n_seq, int H, int d);

/* knap_varlen_attn_bwd for callers that cannot allocate a workspace: code under
 * HIP graph capture, tight serving or training loops, harnesses that forbid
 * hipMalloc.  Same arguments without `workspace`, same kernels, same results
 * bit for bit.  The scratch (the per-row dot products of dout and out and the
 * log-sum-exp in base 2, two floats per (row, head), plus 256 bytes of
 * work-queue counters) is an array in the library's device image,
 * 2 * KNAP_NOALLOC_MAX_ROWS floats + 256 bytes = 32 MiB + 256 bytes that every
 * GPU the library runs on holds until the process ends.
 * The call allocates and frees nothing and synchronises nothing.
 * Limit: total_tokens * H <= KNAP_NOALLOC_MAX_ROWS, else
 * KNAP_ERR_SCRATCH_TOO_SMALL (nothing is enqueued).
 * Every call on a GPU shares that GPU's array, which keeps the previous call's
 * contents (each call overwrites all it reads): calls that may overlap on one
 * GPU (different streams, or graphs replayed at the same time) race on it and
 * must use knap_varlen_attn_bwd with a workspace each instead.  As for the
 * forward, the first call of the library on a device must not be captured. */
#define KNAP_NOALLOC_MAX_ROWS (4 * 1024 * 1024)
int knap_varlen_attn_bwd_noalloc(const void* q, const void* k, const void* v,
                                 const int32_t* cu_seqlens, int n_seq,
                                 int H, int d, float scale,
                                 const void* out, const float* lse,
                                 const void* dout,
                                 void* dq, void* dk, void* dv,
                                 int64_t total_tokens,
                                 void* stream);

/* The same two calls under the other homogeneous mask the paper admits inside a
 * datum (Limitations paragraph: bidirectional full attention or causal
 * attention): row i of a sequence attends to rows 0..i of that sequence only,
 * i counted from the sequence's first row; lse is the log-sum over those keys.
 * Arguments, layouts, workspace (same size query), concurrency and error
 * behaviour are exactly those of knap_varlen_attn_fwd / knap_varlen_attn_bwd;
 * `out` and `lse` given to the backward must come from the causal forward. */
int knap_varlen_attn_causal_fwd(const void* q, const void* k, const void* v,
                                const int32_t* cu_seqlens, int n_seq,
                                int H, int d, float scale,
                                void* out, float* lse,
                                void* stream);
int knap_varlen_attn_causal_bwd(const void* q, const void* k, const void* v,
                                const int32_t* cu_seqlens, int n_seq,
                                int H, int d, float scale,
                                const void* out, const float* lse,
                                const void* dout,
                                void* dq, void* dk, void* dv,
                                int64_t total_tokens,
                                void* workspace, size_t workspace_bytes,
                                void* stream);

/* ------------------------------------------------------------------------
 * Local data movement of the Ulysses layout switch (Sec. 3.4).  A g-GPU bag
 * goes from (partial sequences, full heads) to (full sequences, partial heads)
 * with one all-to-all before attention and back with one after it.  Around
 * each all-to-all (which is the caller's, e.g. RCCL) every GPU of the bag
 * rearranges its own data so that what it sends to one peer is contiguous.
 * Element type: any two-byte type (bf16); (H / g) * d must be a multiple of 8
 * so that a (token, head-group) row is a whole number of 16-byte units.
 * Device pointers, 16-byte aligned, caller-owned; in and out must not alias;
 * nothing allocates or synchronises; a tensor may hold at most 2^31 units.
 *
 * Layouts.  GPU r of the bag holds chunk r of every sequence of the bag (second
 * pass of Sec. 3.3: g contiguous chunks as even as possible, the first L mod g
 * one token longer), packed in the bag's sequence order: (T_r, H, d).
 *   pack_heads    x (T_r, H, d) -> y (g, T_r, H/g, d); slab r' = heads
 *                 [r' H/g, (r'+1) H/g) of every local token = what GPU r' gets.
 *   unpack_heads  the inverse (after the second all-to-all).
 * After the first all-to-all a GPU holds g slabs, from GPU 0 .. g-1 in that
 * order, slab r being (T_r, H/g, d): `recv`, T = sum_r T_r rows in all.
 *   gather_chunks   recv -> z (T, H/g, d), every sequence whole and in the
 *                   bag's order (the input of knap_varlen_attn_* with H/g heads
 *                   and the bag's cu_seqlens).
 *   scatter_chunks  the inverse (before the second all-to-all).
 * Both use row_map (int32[T], device): z[t] = recv[row_map[t]].  It depends
 * only on the bag's cu_seqlens and g; knap_ulysses_plan builds it on the device
 * (workspace: knap_ulysses_plan_workspace_bytes(n_seq, g) bytes of scratch, free
 * to reuse once the plan kernels have run) and it serves q, k, v, the attention
 * output and their gradients in every layer until the bag changes.
 * ------------------------------------------------------------------------ */
#define KNAP_ULYSSES_MAX_GPUS 64

int knap_ulysses_pack_heads(const void* x, int64_t local_tokens, int H, int d, int g, void* y, void* stream);
int knap_ulysses_unpack_heads(const void* y, int64_t local_tokens, int H, int d, int g, void* x, void* stream);

size_t knap_ulysses_plan_workspace_bytes(int n_seq, int g);
/* cu_seqlens: device int32[n_seq + 1] of the WHOLE sequences of the bag;
 * total_tokens must equal cu_seqlens[n_seq]; 1 <= g <= KNAP_ULYSSES_MAX_GPUS. */
int knap_ulysses_plan(const int32_t* cu_seqlens, int n_seq, int64_t total_tokens, int g,
                      int32_t* row_map, void* workspace, size_t workspace_bytes, void* stream);

int knap_ulysses_gather_chunks(const void* recv, const int32_t* row_map, int64_t total_tokens,
                               int heads_local, int d, void* z, void* stream);
int knap_ulysses_scatter_chunks(const void* z, const int32_t* row_map, int64_t total_tokens,
                                int heads_local, int d, void* send, void* stream);

/* Message for a KNAP_ERR_* code (static string, never NULL). */
const char* knap_strerror(int code);

/* The hipError_t (as int) of the most recent failed launch on this thread, 0 if none. */
int knap_last_hip_error(void);

/* ------------------------------------------------------------------------
 * Host-side workload model and balancer (pure C, host pointers, no GPU).
 * ------------------------------------------------------------------------ */

/* a L^2 + b L: the semi-empirical per-sequence cost (Sec. 3.1, Eq. 2 with
 * a = k gamma 4 d and b = k 24 d^2). */
double knap_seq_cost(int64_t L, double a, double b);

/* 24 l d^2 + gamma 4 l^2 d with d = d_model (Eq. 1 for gamma = 1, Eq. 2
 * without the hardware constant otherwise). */
double knap_flux_workload(int64_t l, int64_t d_model, double gamma);

/* Fit t ~ a sumL2 + b sumL over n measurements by least squares on the
 * relative error, no intercept (Sec. 3.1: the correction is obtained by
 * fitting the model to measured (l, t) pairs).  Writes a, b and the largest
 * relative residual.  n >= 2, every t > 0. */
int knap_fit_cost_model(const double* sum_l2, const double* sum_l, const double* t, int n,
                        double* a, double* b, double* max_rel_resid);

/* "g1n2+g2n1+g4n1" -> bag_gpus = {1, 1, 2, 4}, *n_bags = 4 (Sec. 3.2).
 * `cap` is the capacity of bag_gpus. */
int knap_parse_topology(const char* spec, int* bag_gpus, int cap, int* n_bags);

/* First pass of the greedy balancer (Sec. 3.3) with cost a L^2 + b L:
 * sequences in descending cost (stable), each to the bag of lowest occupancy
 * among those with enough remaining capacity; if none has, among all bags.
 * Writes bag_of_seq[n_seq] and bag_load[n_bags]. */
int knap_greedy_assign(const int64_t* seq_len, int n_seq,
                       const int* bag_gpus, int n_bags,
                       double a, double b,
                       int* bag_of_seq, double* bag_load);

/* The same pass on caller-computed weights (e.g. knap_flux_workload). */
int knap_greedy_assign_weights(const double* weight, int n_seq,
                               const int* bag_gpus, int n_bags,
                               int* bag_of_seq, double* bag_load);

/* Second pass (Sec. 3.3): lengths of the g contiguous chunks of a sequence,
 * the first (L mod g) one token longer.  Writes chunk_len[g]. */
int knap_chunk_lengths(int64_t L, int g, int64_t* chunk_len);

/* Tokens every GPU of a g-GPU bag holds after the second pass: tokens_of_gpu[r] =
 * sum over the bag's sequences of the length of chunk r (the T_r above, and the
 * split sizes of the all-to-all).  Writes tokens_of_gpu[g]. */
int knap_ulysses_local_tokens(const int64_t* seq_len, int n_seq, int g, int64_t* tokens_of_gpu);

/* Workload imbalance ratio (Sec. 4.2): max / min over bags of load_j / gpus_j. */
double knap_wir(const double* bag_load, const int* bag_gpus, int n_bags);

/* Packed list of one bag: writes the lengths of the sequences assigned to
 * `bag` (original order) to out_len[cap], their count to *n_out, and, if
 * cu_seqlens is not NULL, their prefix sums to cu_seqlens[*n_out + 1]. */
int knap_bag_cu_seqlens(const int64_t* seq_len, const int* bag_of_seq, int n_seq, int bag,
                        int64_t* out_len, int cap, int* n_out, int32_t* cu_seqlens);

#ifdef __cplusplus
}
#endif
#endif /* KNAPATTN_H */
