/* Drives the CPU oracle under AddressSanitizer / UBSan (built and run by
 * tests/test_oracle_sanitize.py).  Exercises ordinary batches, every status path, fanout -1,
 * exact capacities and the label / mean-aggregation helpers on a small random graph. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int32_t oracle_sample_mfg(int64_t, const int64_t *, const int32_t *, const void *, int64_t, int64_t,
                          const int32_t *, int32_t, const int32_t *, int32_t, uint64_t, int32_t *, int64_t,
                          const int64_t *, int32_t *, int32_t *const *, int32_t *const *, void *, int64_t *);
int32_t oracle_slice_labels(const void *, int32_t, int64_t, const int32_t *, int32_t, void *);
int32_t oracle_mean_aggregate(const int32_t *, const int32_t *, int64_t, const void *, int32_t, int32_t,
                              double *, double *);
int32_t oracle_sage_layer(const int32_t *, const int32_t *, int64_t, const void *, int32_t, int32_t,
                          const double *, const double *, int32_t, int32_t, double *, double *, double *,
                          double *);
int32_t oracle_sample_positions(uint32_t, int32_t, uint64_t, uint32_t, uint32_t, uint32_t *);

static uint64_t rng_state = 88172645463325252ull;
static uint32_t rnd(void) {
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (uint32_t)(rng_state >> 16);
}

#define N 400
#define L_MAX 4

int main(void) {
  /* random graph with rows of 0..40 neighbours (repeats allowed) */
  int64_t *indptr = malloc(sizeof(int64_t) * (N + 1));
  indptr[0] = 0;
  for (int v = 0; v < N; ++v) indptr[v + 1] = indptr[v] + (v % 11 == 0 ? 0 : rnd() % 41);
  int64_t m = indptr[N];
  int32_t *indices = malloc(sizeof(int32_t) * (size_t)(m > 0 ? m : 1));
  for (int64_t e = 0; e < m; ++e) indices[e] = (int32_t)(rnd() % N);
  float *feat = malloc(sizeof(float) * N * 6);
  for (int i = 0; i < N * 6; ++i) feat[i] = (float)(rnd() % 1000) / 37.0f;
  int32_t *local_of = malloc(sizeof(int32_t) * N);
  for (int v = 0; v < N; ++v) local_of[v] = -1;

  const int32_t fan_sets[6][L_MAX] = {{3, 2, 0, 0}, {32, 0, 0, 0}, {1, 1, 1, 1}, {-1, 2, 0, 0}, {5, -1, -1, 0}, {100, 7, 0, 0}};
  const int32_t fan_len[6] = {2, 1, 4, 2, 3, 2};
  int checked = 0;
  for (int f = 0; f < 6; ++f) {
    for (int trial = 0; trial < 6; ++trial) {
      int32_t L = fan_len[f];
      int32_t ns = 1 + (int32_t)(rnd() % 40);
      int32_t seeds[41];
      for (int i = 0; i < ns; ++i) {       /* distinct seeds */
        int again = 1;
        while (again) {
          seeds[i] = (int32_t)(rnd() % N);
          again = 0;
          for (int q = 0; q < i; ++q) if (seeds[q] == seeds[i]) again = 1;
        }
      }
      if (trial == 4) seeds[ns - 1] = seeds[0] + (ns > 1 ? 0 : N);   /* duplicate (or out of range) */
      if (trial == 5) seeds[0] = -3;                                  /* out of range */
      /* exact-fit buffers: first run with roomy capacities to learn the sizes */
      int64_t node_cap = N, edge_cap[L_MAX];
      for (int h = 0; h < L; ++h) edge_cap[h] = m > 0 ? m : 1;
      for (int pass = 0; pass < 3; ++pass) {
        int32_t *node_ids = malloc(sizeof(int32_t) * (size_t)node_cap);
        int32_t *bp[L_MAX], *bi[L_MAX];
        for (int h = 0; h < L; ++h) {
          bp[h] = malloc(sizeof(int32_t) * (size_t)(node_cap + 1));
          bi[h] = malloc(sizeof(int32_t) * (size_t)(edge_cap[h] > 0 ? edge_cap[h] : 1));
        }
        float *out_feat = malloc(sizeof(float) * 6 * (size_t)node_cap);
        int64_t counts[2 * L_MAX + 2];
        int32_t st = oracle_sample_mfg(N, indptr, indices, feat, 24, 24, seeds, ns, fan_sets[f], L,
                                       0x1234567ull * (uint64_t)(trial + 1), local_of, node_cap, edge_cap,
                                       node_ids, bp, bi, out_feat, counts);
        for (int v = 0; v < N; ++v) if (local_of[v] != -1) { printf("scratch not restored\n"); return 1; }
        if (st == 0) {
          for (int64_t j = 0; j < counts[L]; ++j)
            if (memcmp(out_feat + 6 * j, feat + 6 * node_ids[j], 24) != 0) { printf("bad row\n"); return 1; }
          /* consumers of the result */
          int64_t labels[N], ys[41];
          for (int v = 0; v < N; ++v) labels[v] = v * 3;
          if (oracle_slice_labels(labels, 8, N, seeds, ns, ys) != 0 || ys[0] != seeds[0] * 3) return 1;
          double *mean = malloc(sizeof(double) * 6 * (size_t)(counts[L - 1] + 1));
          double *mag = malloc(sizeof(double) * 6 * (size_t)(counts[L - 1] + 1));
          if (oracle_mean_aggregate(bp[L - 1], bi[L - 1], counts[L - 1], out_feat, 6, 4, mean, mag) != 0) return 1;
          {                       /* a layer with 5 outputs over the same block */
            double w[5 * 12], bias[5];
            for (int q = 0; q < 5 * 12; ++q) w[q] = (double)(rnd() % 17) - 8.0;
            for (int q = 0; q < 5; ++q) bias[q] = (double)(rnd() % 5) - 2.0;
            double *lo = malloc(sizeof(double) * 5 * (size_t)(counts[L - 1] + 1));
            double *lm = malloc(sizeof(double) * 5 * (size_t)(counts[L - 1] + 1));
            if (oracle_sage_layer(bp[L - 1], bi[L - 1], counts[L - 1], out_feat, 6, 4, w, bias, 5, 1, mean, mag,
                                  lo, lm) != 0) return 1;
            free(lo); free(lm);
          }
          free(mean); free(mag);
          ++checked;
        }
        int64_t n_final = counts[L];
        int64_t e_now[L_MAX];
        for (int h = 0; h < L; ++h) e_now[h] = counts[L + 1 + h];
        free(node_ids); free(out_feat);
        for (int h = 0; h < L; ++h) { free(bp[h]); free(bi[h]); }
        if (st != 0) break;
        if (pass == 0) {            /* second pass: exact capacities must succeed */
          node_cap = n_final > 0 ? n_final : 1;
          for (int h = 0; h < L; ++h) edge_cap[h] = e_now[h];
        } else if (pass == 1) {     /* third pass: one short of the nodes must report, not overrun */
          if (n_final > ns) node_cap = n_final - 1; else break;
        }
      }
    }
  }
  uint32_t p[8];
  if (oracle_sample_positions(5, 8, 1, 2, 3, p) != 5 || oracle_sample_positions(1000000, 8, 1, 2, 3, p) != 8) return 1;
  printf("ok %d\n", checked);
  free(indptr); free(indices); free(feat); free(local_of);
  return 0;
}
