/* Fuzz driver for the host side of libknapattn (csrc/knap_host.c), built by
 * tests/test_host_sanitizers.py with -fsanitize=address,undefined.  It calls
 * every host function on seeded random and degenerate inputs (malformed
 * topology strings, empty bags, zero weights, zero capacities, undersized
 * output arrays) and checks the few properties that hold for any input.  A
 * sanitizer report or a failed check ends the process with a non-zero status. */
#include "knapattn.h"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>

static unsigned long long g_state = 0x9E3779B97F4A7C15ull;
static unsigned rnd(void) {
  g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
  return (unsigned)(g_state >> 33);
}
static int rnd_in(int lo, int hi) { return lo + (int)(rnd() % (unsigned)(hi - lo + 1)); }

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond);   \
      exit(3);                                                             \
    }                                                                      \
  } while (0)

static void fuzz_topology(void) {
  static const char alphabet[] = "gn+0123456789 x-";
  const char* fixed[] = {"", "g", "g1", "g1n", "g1n1+", "+g1n1", "g0n1", "g1n0", "g1n2+g2n1+g4n1", "g8n4",
                         "g1n1 + g2n2", "g99999999n1", "g1n99999999", "G1N1", "g1n1x", "g-1n1", " g2n3 "};
  int bags[64];
  for (size_t i = 0; i < sizeof(fixed) / sizeof(fixed[0]); ++i) {
    int n = -1;
    const int rc = knap_parse_topology(fixed[i], bags, 64, &n);
    if (rc == KNAP_OK) { CHECK(n >= 1 && n <= 64); for (int j = 0; j < n; ++j) CHECK(bags[j] >= 1); }
    else CHECK(rc == KNAP_ERR_PARSE || rc == KNAP_ERR_CAPACITY);
  }
  { int n = 0; CHECK(knap_parse_topology("g1n2+g2n1+g4n1", bags, 64, &n) == KNAP_OK && n == 4 && bags[3] == 4); }
  { int n = 0; CHECK(knap_parse_topology("g1n5", bags, 4, &n) == KNAP_ERR_CAPACITY); }
  { int n = 0; CHECK(knap_parse_topology("g1n1", bags, 0, &n) == KNAP_ERR_CAPACITY); }
  { int n = 0; CHECK(knap_parse_topology(NULL, bags, 4, &n) == KNAP_ERR_INVALID_ARG); }
  for (int it = 0; it < 4000; ++it) {
    const int len = rnd_in(0, 24);
    char* s = (char*)malloc((size_t)len + 1);      /* exactly sized: an overread is caught */
    for (int i = 0; i < len; ++i) s[i] = alphabet[rnd() % (sizeof(alphabet) - 1)];
    s[len] = '\0';
    const int cap = rnd_in(0, 16);
    int* out = (int*)malloc(sizeof(int) * (size_t)(cap > 0 ? cap : 1));
    int n = -1;
    const int rc = knap_parse_topology(s, out, cap, &n);
    if (rc == KNAP_OK) CHECK(n >= 1 && n <= cap);
    free(out);
    free(s);
  }
}

static void fuzz_greedy(void) {
  for (int it = 0; it < 3000; ++it) {
    const int n_seq = rnd_in(0, 40), n_bags = rnd_in(1, 9);
    int64_t* len = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_seq > 0 ? n_seq : 1));
    double* w = (double*)malloc(sizeof(double) * (size_t)(n_seq > 0 ? n_seq : 1));
    int* gpus = (int*)malloc(sizeof(int) * (size_t)n_bags);
    int* bag_of = (int*)malloc(sizeof(int) * (size_t)(n_seq > 0 ? n_seq : 1));
    double* load = (double*)malloc(sizeof(double) * (size_t)n_bags);
    const int mode = it % 5;     /* 0: random, 1: all zero lengths, 2: equal, 3: one giant, 4: zero model */
    for (int i = 0; i < n_seq; ++i) {
      len[i] = mode == 1 ? 0 : mode == 2 ? 777 : (mode == 3 && i == 0) ? 1000000 : rnd_in(0, 70000);
      w[i] = mode == 1 ? 0.0 : (double)len[i] * 1.5;
    }
    for (int j = 0; j < n_bags; ++j) gpus[j] = 1 << rnd_in(0, 3);
    const double a = mode == 4 ? 0.0 : 1e-6, b = mode == 4 ? 0.0 : 3e-3;
    CHECK(knap_greedy_assign(len, n_seq, gpus, n_bags, a, b, bag_of, load) == KNAP_OK);
    double sum_load = 0.0, sum_w = 0.0;
    for (int j = 0; j < n_bags; ++j) sum_load += load[j];
    for (int i = 0; i < n_seq; ++i) {
      CHECK(bag_of[i] >= 0 && bag_of[i] < n_bags);
      sum_w += knap_seq_cost(len[i], a, b);
    }
    CHECK(fabs(sum_load - sum_w) <= 1e-9 * (1.0 + sum_w));
    CHECK(knap_greedy_assign_weights(w, n_seq, gpus, n_bags, bag_of, load) == KNAP_OK);
    for (int i = 0; i < n_seq; ++i) CHECK(bag_of[i] >= 0 && bag_of[i] < n_bags);
    const double r = knap_wir(load, gpus, n_bags);
    CHECK(isnan(r) || r >= 1.0 - 1e-12);      /* inf when a bag stays empty */
    /* one bag's packed list, with an output array that may be too small */
    const int bag = rnd_in(0, n_bags - 1), cap = rnd_in(0, n_seq + 1);
    int64_t* out_len = (int64_t*)malloc(sizeof(int64_t) * (size_t)(cap > 0 ? cap : 1));
    int32_t* cu = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cap + 1));
    int n_out = -1;
    const int rc = knap_bag_cu_seqlens(len, bag_of, n_seq, bag, out_len, cap, &n_out, cu);
    if (rc == KNAP_OK) {
      CHECK(n_out >= 0 && n_out <= cap && cu[0] == 0);
      for (int i = 0; i < n_out; ++i) CHECK(cu[i + 1] - cu[i] == (int32_t)out_len[i]);
    } else {
      CHECK(rc == KNAP_ERR_CAPACITY);
    }
    free(cu); free(out_len);
    /* bad arguments */
    gpus[0] = 0;
    CHECK(knap_greedy_assign_weights(w, n_seq, gpus, n_bags, bag_of, load) == KNAP_ERR_INVALID_ARG);
    CHECK(isnan(knap_wir(load, gpus, n_bags)));
    gpus[0] = 1;
    if (n_seq > 0) {
      w[0] = -1.0;
      CHECK(knap_greedy_assign_weights(w, n_seq, gpus, n_bags, bag_of, load) == KNAP_ERR_INVALID_ARG);
      w[0] = NAN;
      CHECK(knap_greedy_assign_weights(w, n_seq, gpus, n_bags, bag_of, load) == KNAP_ERR_INVALID_ARG);
      len[0] = -5;
      CHECK(knap_greedy_assign(len, n_seq, gpus, n_bags, a, b, bag_of, load) == KNAP_ERR_INVALID_ARG);
    }
    CHECK(knap_greedy_assign_weights(w, n_seq, gpus, 0, bag_of, load) == KNAP_ERR_INVALID_ARG);
    free(len); free(w); free(gpus); free(bag_of); free(load);
  }
}

static void fuzz_chunks(void) {
  for (int it = 0; it < 3000; ++it) {
    const int g = rnd_in(1, 64);
    const int64_t L = it % 7 == 0 ? 0 : (int64_t)rnd_in(0, 300000);
    int64_t* c = (int64_t*)malloc(sizeof(int64_t) * (size_t)g);
    CHECK(knap_chunk_lengths(L, g, c) == KNAP_OK);
    int64_t sum = 0;
    for (int r = 0; r < g; ++r) { sum += c[r]; CHECK(c[r] == L / g || c[r] == L / g + 1); CHECK(r == 0 || c[r] <= c[r - 1]); }
    CHECK(sum == L);
    const int n_seq = rnd_in(0, 12);
    int64_t* len = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_seq > 0 ? n_seq : 1));
    int64_t total = 0;
    for (int i = 0; i < n_seq; ++i) { len[i] = rnd_in(0, 5000); total += len[i]; }
    CHECK(knap_ulysses_local_tokens(len, n_seq, g, c) == KNAP_OK);
    sum = 0;
    for (int r = 0; r < g; ++r) sum += c[r];
    CHECK(sum == total);
    free(len); free(c);
  }
  int64_t one;
  CHECK(knap_chunk_lengths(10, 0, &one) == KNAP_ERR_INVALID_ARG);
  CHECK(knap_chunk_lengths(-1, 2, &one) == KNAP_ERR_INVALID_ARG);
  CHECK(knap_chunk_lengths(10, 1, NULL) == KNAP_ERR_INVALID_ARG);
}

static void fuzz_fit(void) {
  for (int it = 0; it < 2000; ++it) {
    const int n = rnd_in(0, 12);
    double* s2 = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double* s1 = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double* t = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    const double a0 = 1e-7 * (1 + rnd_in(0, 9)), b0 = 1e-4 * (1 + rnd_in(0, 9));
    const int mode = it % 4;     /* 0: exact model, 1: one length only (singular), 2: a zero time, 3: all zero */
    for (int i = 0; i < n; ++i) {
      const double L = mode == 1 ? 1024.0 : (double)rnd_in(64, 70000);
      const double m = (double)rnd_in(1, 20);
      s2[i] = mode == 3 ? 0.0 : m * L * L;
      s1[i] = mode == 3 ? 0.0 : m * L;
      t[i] = a0 * s2[i] + b0 * s1[i];
      if (mode == 2 && i == n / 2) t[i] = 0.0;
    }
    double a = 0, b = 0, r = 0;
    const int rc = knap_fit_cost_model(s2, s1, t, n, &a, &b, &r);
    if (rc == KNAP_OK) {
      CHECK(mode == 0 && n >= 2);
      CHECK(fabs(a - a0) <= 1e-6 * a0 && fabs(b - b0) <= 1e-5 * b0 && r <= 1e-8);
    } else {
      CHECK(rc == KNAP_ERR_INVALID_ARG);
    }
    free(s2); free(s1); free(t);
  }
}

int main(void) {
  fuzz_topology();
  fuzz_greedy();
  fuzz_chunks();
  fuzz_fit();
  CHECK(knap_seq_cost(0, 1.0, 1.0) == 0.0);
  CHECK(knap_flux_workload(0, 3072, 0.49) == 0.0);
  puts("host fuzz ok");
  return 0;
}
