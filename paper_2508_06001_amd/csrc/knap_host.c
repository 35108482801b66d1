/* Host side of libknapattn: the semi-empirical workload model (Sec. 3.1),
 * the compute-bag topology string (Sec. 3.2), the greedy balancer's first and
 * second pass (Sec. 3.3) and the workload imbalance ratio (Sec. 4.2).
 * Pure C, no GPU. */
#include "knapattn.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

double knap_seq_cost(int64_t L, double a, double b) {
  const double l = (double)L;
  return a * l * l + b * l;
}

double knap_flux_workload(int64_t l, int64_t d_model, double gamma) {
  const double x = (double)l, d = (double)d_model;
  return 24.0 * x * d * d + gamma * 4.0 * x * x * d;
}

/* Relative least squares without intercept: minimise sum_i ((a x2_i + b x1_i - t_i) / t_i)^2.
 * With u_i = x2_i / t_i and v_i = x1_i / t_i this is the 2x2 normal system
 *   [ sum u^2  sum uv ] [a]   [ sum u ]
 *   [ sum uv   sum v^2 ] [b] = [ sum v ]. */
int knap_fit_cost_model(const double* sum_l2, const double* sum_l, const double* t, int n,
                        double* a, double* b, double* max_rel_resid) {
  if (!sum_l2 || !sum_l || !t || !a || !b || n < 2) return KNAP_ERR_INVALID_ARG;
  /* columns are scaled to unit magnitude first: sum_l2 is ~1e4..1e5 times sum_l */
  double s2 = 0.0, s1 = 0.0;
  for (int i = 0; i < n; ++i) {
    if (!(t[i] > 0.0)) return KNAP_ERR_INVALID_ARG;
    const double u = sum_l2[i] / t[i], v = sum_l[i] / t[i];
    if (fabs(u) > s2) s2 = fabs(u);
    if (fabs(v) > s1) s1 = fabs(v);
  }
  if (s2 == 0.0 || s1 == 0.0) return KNAP_ERR_INVALID_ARG;
  double uu = 0.0, uv = 0.0, vv = 0.0, ru = 0.0, rv = 0.0;
  for (int i = 0; i < n; ++i) {
    const double u = sum_l2[i] / t[i] / s2, v = sum_l[i] / t[i] / s1;
    uu += u * u; uv += u * v; vv += v * v; ru += u; rv += v;
  }
  const double det = uu * vv - uv * uv;
  if (!(fabs(det) > 1e-300) || fabs(det) < 1e-14 * uu * vv) return KNAP_ERR_INVALID_ARG;
  *a = (ru * vv - rv * uv) / det / s2;
  *b = (rv * uu - ru * uv) / det / s1;
  if (max_rel_resid) {
    double worst = 0.0;
    for (int i = 0; i < n; ++i) {
      const double r = fabs((*a) * sum_l2[i] + (*b) * sum_l[i] - t[i]) / t[i];
      if (r > worst) worst = r;
    }
    *max_rel_resid = worst;
  }
  return KNAP_OK;
}

/* Parses one positive decimal integer at *p; advances *p.  Returns -1 on failure. */
static long parse_uint(const char** p) {
  const char* s = *p;
  if (*s < '0' || *s > '9') return -1;
  long v = 0;
  while (*s >= '0' && *s <= '9') {
    v = v * 10 + (*s - '0');
    if (v > 1000000) return -1;
    ++s;
  }
  *p = s;
  return v;
}

int knap_parse_topology(const char* spec, int* bag_gpus, int cap, int* n_bags) {
  if (!spec || !bag_gpus || !n_bags || cap < 0) return KNAP_ERR_INVALID_ARG;
  const char* p = spec;
  int count = 0;
  for (;;) {
    while (*p == ' ') ++p;
    if (*p != 'g') return KNAP_ERR_PARSE;
    ++p;
    const long g = parse_uint(&p);
    if (g <= 0 || *p != 'n') return KNAP_ERR_PARSE;
    ++p;
    const long n = parse_uint(&p);
    if (n <= 0) return KNAP_ERR_PARSE;
    for (long i = 0; i < n; ++i) {
      if (count >= cap) return KNAP_ERR_CAPACITY;
      bag_gpus[count++] = (int)g;
    }
    while (*p == ' ') ++p;
    if (*p == '+') { ++p; continue; }
    if (*p == '\0') break;
    return KNAP_ERR_PARSE;
  }
  *n_bags = count;
  return KNAP_OK;
}

typedef struct { double w; int idx; } knap_item;

/* descending weight; equal weights keep their original order */
static int item_cmp(const void* pa, const void* pb) {
  const knap_item* a = (const knap_item*)pa;
  const knap_item* b = (const knap_item*)pb;
  if (a->w > b->w) return -1;
  if (a->w < b->w) return 1;
  return (a->idx > b->idx) - (a->idx < b->idx);
}

int knap_greedy_assign_weights(const double* weight, int n_seq,
                               const int* bag_gpus, int n_bags,
                               int* bag_of_seq, double* bag_load) {
  if (n_seq < 0 || n_bags <= 0 || !bag_gpus || !bag_load || (n_seq > 0 && (!weight || !bag_of_seq)))
    return KNAP_ERR_INVALID_ARG;
  long total_gpus = 0;
  for (int j = 0; j < n_bags; ++j) {
    if (bag_gpus[j] <= 0) return KNAP_ERR_INVALID_ARG;
    total_gpus += bag_gpus[j];
    bag_load[j] = 0.0;
  }
  if (n_seq == 0) return KNAP_OK;
  knap_item* items = (knap_item*)malloc(sizeof(knap_item) * (size_t)n_seq);
  double* capacity = (double*)malloc(sizeof(double) * (size_t)n_bags);
  if (!items || !capacity) { free(items); free(capacity); return KNAP_ERR_INVALID_ARG; }
  double total = 0.0;
  for (int i = 0; i < n_seq; ++i) {
    if (!(weight[i] >= 0.0)) { free(items); free(capacity); return KNAP_ERR_INVALID_ARG; }
    items[i].w = weight[i];
    items[i].idx = i;
    total += weight[i];
  }
  const double per_gpu_target = total / (double)total_gpus;
  for (int j = 0; j < n_bags; ++j) capacity[j] = per_gpu_target * (double)bag_gpus[j];
  qsort(items, (size_t)n_seq, sizeof(knap_item), item_cmp);

  for (int r = 0; r < n_seq; ++r) {
    const double w = items[r].w;
    int pick = -1, pick_any = -1;
    double occ = 0.0, occ_any = 0.0;
    for (int j = 0; j < n_bags; ++j) {
      const double o = capacity[j] > 0.0 ? bag_load[j] / capacity[j] : 0.0;
      if (pick_any < 0 || o < occ_any) { pick_any = j; occ_any = o; }
      if (capacity[j] - bag_load[j] >= w && (pick < 0 || o < occ)) { pick = j; occ = o; }
    }
    if (pick < 0) pick = pick_any;   /* nothing fits: lowest occupancy over all bags */
    bag_load[pick] += w;
    bag_of_seq[items[r].idx] = pick;
  }
  free(items);
  free(capacity);
  return KNAP_OK;
}

int knap_greedy_assign(const int64_t* seq_len, int n_seq,
                       const int* bag_gpus, int n_bags,
                       double a, double b,
                       int* bag_of_seq, double* bag_load) {
  if (n_seq < 0 || (n_seq > 0 && !seq_len)) return KNAP_ERR_INVALID_ARG;
  double* w = (double*)malloc(sizeof(double) * (size_t)(n_seq > 0 ? n_seq : 1));
  if (!w) return KNAP_ERR_INVALID_ARG;
  for (int i = 0; i < n_seq; ++i) {
    if (seq_len[i] < 0) { free(w); return KNAP_ERR_INVALID_ARG; }
    w[i] = knap_seq_cost(seq_len[i], a, b);
  }
  const int rc = knap_greedy_assign_weights(w, n_seq, bag_gpus, n_bags, bag_of_seq, bag_load);
  free(w);
  return rc;
}

int knap_chunk_lengths(int64_t L, int g, int64_t* chunk_len) {
  if (L < 0 || g <= 0 || !chunk_len) return KNAP_ERR_INVALID_ARG;
  const int64_t base = L / g, rem = L % g;
  for (int c = 0; c < g; ++c) chunk_len[c] = base + (c < rem ? 1 : 0);
  return KNAP_OK;
}

int knap_ulysses_local_tokens(const int64_t* seq_len, int n_seq, int g, int64_t* tokens_of_gpu) {
  if (n_seq < 0 || g <= 0 || !tokens_of_gpu || (n_seq > 0 && !seq_len)) return KNAP_ERR_INVALID_ARG;
  for (int r = 0; r < g; ++r) tokens_of_gpu[r] = 0;
  for (int s = 0; s < n_seq; ++s) {
    if (seq_len[s] < 0) return KNAP_ERR_INVALID_ARG;
    const int64_t base = seq_len[s] / g, rem = seq_len[s] % g;
    for (int r = 0; r < g; ++r) tokens_of_gpu[r] += base + (r < rem ? 1 : 0);
  }
  return KNAP_OK;
}

double knap_wir(const double* bag_load, const int* bag_gpus, int n_bags) {
  if (!bag_load || !bag_gpus || n_bags <= 0) return NAN;
  double hi = 0.0, lo = 0.0;
  for (int j = 0; j < n_bags; ++j) {
    if (bag_gpus[j] <= 0) return NAN;
    const double per_gpu = bag_load[j] / (double)bag_gpus[j];
    if (j == 0 || per_gpu > hi) hi = per_gpu;
    if (j == 0 || per_gpu < lo) lo = per_gpu;
  }
  return lo > 0.0 ? hi / lo : INFINITY;
}

int knap_bag_cu_seqlens(const int64_t* seq_len, const int* bag_of_seq, int n_seq, int bag,
                        int64_t* out_len, int cap, int* n_out, int32_t* cu_seqlens) {
  if (n_seq < 0 || !n_out || cap < 0 || (n_seq > 0 && (!seq_len || !bag_of_seq))) return KNAP_ERR_INVALID_ARG;
  int count = 0;
  int64_t total = 0;
  if (cu_seqlens) cu_seqlens[0] = 0;
  for (int i = 0; i < n_seq; ++i) {
    if (bag_of_seq[i] != bag) continue;
    if (count >= cap || !out_len) return KNAP_ERR_CAPACITY;
    total += seq_len[i];
    if (total > INT32_MAX) return KNAP_ERR_INVALID_ARG;
    out_len[count++] = seq_len[i];
    if (cu_seqlens) cu_seqlens[count] = (int32_t)total;
  }
  *n_out = count;
  return KNAP_OK;
}
