/*
 * CPU oracle for sampled mini-batch preparation.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, single-threaded, deliberately slow statement of what the hot path computes:
 * node-wise neighbour sampling (paper section 2.2 and section 4.1, first paragraph), the
 * one-hop message-flow-graph construction with its ordered global->local map (the MFG
 * construction algorithm, procedure OneHopMFG), chained over hops (section 4.1), and the
 * slice xs = x[ids] of Listing 1; plus the label slice of Listing 1 and, as a consumer of the
 * blocks, the mean aggregation and the whole GraphSAGE layer (mean, linear layer on the
 * concatenation, ReLU) of equation 1 / section 2.1 / the GraphSAGE listing of Appendix C.
 *
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may use this file.
 * It shares nothing with the HIP library: no header, no table, no helper.
 *
 * Readings where the paper is silent (the same ones the HIP library documents):
 *  - fanouts[0] belongs to hop 0, whose destinations are the seeds;
 *  - a node with deg <= fanout contributes its whole row in CSR order, no random draw;
 *  - otherwise k = fanout distinct row positions are chosen with Floyd's subset algorithm,
 *    the "set" being an array searched linearly (the array set of section 4.1);
 *  - random words are Philox4x32-10 (Salmon et al., SC'11): key = rng_key split into
 *    (low, high) 32-bit words, counter = (dst node, hop, draw / 4, 0), word draw % 4;
 *  - an index in [0, m) is drawn from a 32-bit word r as floor(r * m / 2^32);
 *  - the destinations of hop h+1 are ALL nodes known after hop h (old prefix included).
 *
 * Parity pins: tests/test_oracle_*.py (library Philox, exhaustive Floyd, brute-force
 * invariants, BFS special case, chi-square).  Every exported function is pinned.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
  ORACLE_OK = 0,
  ORACLE_ERR_ARG = -1,
  /* conditions found while walking the data, reported in counts[2L+1] and returned */
  ORACLE_ST_NODE_CAPACITY = 1,
  ORACLE_ST_EDGE_CAPACITY = 2,
  ORACLE_ST_SEED_RANGE = 4,
  ORACLE_ST_DUP_SEED = 5
};

/* ---- Philox4x32-10 -------------------------------------------------------------------- */

static void philox_round(uint32_t c[4], const uint32_t k[2]) {
  uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
  uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
  uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
  uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
  uint32_t n0 = hi1 ^ c[1] ^ k[0];
  uint32_t n2 = hi0 ^ c[3] ^ k[1];
  c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;
}

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
  uint32_t k[2] = {key[0], key[1]};
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k[0] += 0x9E3779B9u; k[1] += 0xBB67AE85u; }
    philox_round(c, k);
  }
  out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

/* The s-th random word of destination node v at hop h. */
static uint32_t draw_word(uint64_t rng_key, uint32_t v, uint32_t h, uint32_t s) {
  uint32_t ctr[4] = {v, h, s >> 2, 0u};
  uint32_t key[2] = {(uint32_t)rng_key, (uint32_t)(rng_key >> 32)};
  uint32_t out[4];
  oracle_philox4x32_10(ctr, key, out);
  return out[s & 3u];
}

/* ---- one destination's sampled row positions ------------------------------------------- */

/* Floyd's algorithm with caller-supplied words: for s = 0..k-1, j = deg-k+s, t = an index in
 * [0, j]; position t is taken unless already taken, in which case j is.  Returns k. */
int32_t oracle_floyd_positions(uint32_t deg, uint32_t k, const uint32_t *words, uint32_t *p) {
  for (uint32_t s = 0; s < k; ++s) {
    uint32_t j = deg - k + s;
    uint32_t t = (uint32_t)(((uint64_t)words[s] * (uint64_t)(j + 1u)) >> 32);
    int taken = 0;
    for (uint32_t q = 0; q < s; ++q) if (p[q] == t) taken = 1;
    p[s] = taken ? j : t;
  }
  return (int32_t)k;
}

/* Positions within the CSR row of v chosen at hop h with fanout d; returns their number.
 * d = -1 stands for the full neighbourhood (section 5 compares sampled fanouts with "all"). */
int32_t oracle_sample_positions(uint32_t deg, int32_t d, uint64_t rng_key, uint32_t v, uint32_t h,
                                uint32_t *p) {
  if (d < -1) return ORACLE_ERR_ARG;
  if (d == -1 || deg <= (uint32_t)d) {
    for (uint32_t s = 0; s < deg; ++s) p[s] = s;
    return (int32_t)deg;
  }
  uint32_t *words = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(d > 0 ? d : 1));
  if (!words) return ORACLE_ERR_ARG;
  for (int32_t s = 0; s < d; ++s) words[s] = draw_word(rng_key, v, h, (uint32_t)s);
  int32_t k = oracle_floyd_positions(deg, (uint32_t)d, words, p);
  free(words);
  return k;
}

/* ---- label slice ---------------------------------------------------------------------------- */

/* ys = y[ids[:batch_size]] (Listing 1): the first batch_size ids are the seeds themselves, so
 * out[i] = y[seeds[i]], elem_bytes bytes each, copied verbatim. */
int32_t oracle_slice_labels(const void *labels, int32_t elem_bytes, int64_t num_nodes,
                            const int32_t *seeds, int32_t num_seeds, void *out) {
  if (!labels || !seeds || !out || elem_bytes < 1) return ORACLE_ERR_ARG;
  for (int32_t i = 0; i < num_seeds; ++i) {
    if (seeds[i] < 0 || (int64_t)seeds[i] >= num_nodes) return ORACLE_ST_SEED_RANGE;
    memcpy((char *)out + (int64_t)i * elem_bytes, (const char *)labels + (int64_t)seeds[i] * elem_bytes,
           (size_t)elem_bytes);
  }
  return ORACLE_OK;
}

/* ---- mean aggregation over one block (a consumer of the MFG) ------------------------------- */

/* IEEE 754 binary16 bit pattern -> double (exact). */
double oracle_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1, ex = (h >> 10) & 0x1F, man = h & 0x3FF;
  double v;
  if (ex == 0) {
    v = (double)man / 1024.0 / 16384.0;              /* subnormal: man * 2^-24 */
  } else if (ex == 31) {
    v = man ? (0.0 / 0.0) : (1.0 / 0.0);
  } else {
    v = 1.0 + (double)man / 1024.0;
    int e = ex - 15;
    while (e > 0) { v *= 2.0; --e; }
    while (e < 0) { v *= 0.5; ++e; }
  }
  return sign ? -v : v;
}

/* Equation 1 with agg = mean, as the GraphSAGE listing of Appendix C uses a block:
 * mean[i, c] = (1/k_i) sum_e x[indices[e], c] over the row i of the block, 0 for an empty row;
 * also mag[i, c] = (1/k_i) sum_e |x[indices[e], c]| (the scale of the float error bound).
 * x: row-major [num_src x dim] of elem_bytes 2 (half) or 4 (float).  All sums in double. */
int32_t oracle_mean_aggregate(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                              const void *x, int32_t dim, int32_t elem_bytes, double *mean, double *mag) {
  if (!indptr || !indices || !x || !mean || !mag || dim < 1 || (elem_bytes != 2 && elem_bytes != 4))
    return ORACLE_ERR_ARG;
  for (int64_t i = 0; i < num_dst; ++i) {
    int32_t k = indptr[i + 1] - indptr[i];
    for (int32_t c = 0; c < dim; ++c) {
      double s = 0.0, a = 0.0;
      for (int32_t e = indptr[i]; e < indptr[i + 1]; ++e) {
        int64_t at = (int64_t)indices[e] * dim + c;
        double v = elem_bytes == 2 ? oracle_half_to_double(((const uint16_t *)x)[at])
                                   : (double)((const float *)x)[at];
        s += v;
        a += v < 0 ? -v : v;
      }
      mean[i * dim + c] = k > 0 ? s / k : 0.0;
      mag[i * dim + c] = k > 0 ? a / k : 0.0;
    }
  }
  return ORACLE_OK;
}

/* One GraphSAGE layer over a block (equation 1 with the choices section 2.1 names for GraphSAGE:
 * agg = mean of the sampled neighbours, upd = a linear layer on the concatenation of the node's
 * own row and that mean; the model listing of Appendix C applies a ReLU after every layer but the
 * last).  The destinations of a block are its first num_dst source rows, so the node's own row is
 * x[i]:
 *   out[i, j] = act(bias[j] + sum_c w[j, c] x[i, c] + sum_c w[j, dim + c] mean[i, c]),
 * w row-major [out_dim x 2 dim] (the layout of a linear layer's weight), bias [out_dim] or NULL,
 * act = max(., 0) if relu else the identity.  mag[i, j] = |bias[j]| + sum_c |w[j, c]| |x[i, c]| +
 * sum_c |w[j, dim + c]| mag_mean[i, c] is the scale for a float error bound.  All in double;
 * mean_tmp, mag_tmp: caller scratch [num_dst x dim]. */
int32_t oracle_sage_layer(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                          const void *x, int32_t dim, int32_t elem_bytes, const double *w,
                          const double *bias, int32_t out_dim, int32_t relu, double *mean_tmp,
                          double *mag_tmp, double *out, double *mag) {
  if (!w || !out || !mag || !mean_tmp || !mag_tmp || out_dim < 1) return ORACLE_ERR_ARG;
  int32_t rc = oracle_mean_aggregate(indptr, indices, num_dst, x, dim, elem_bytes, mean_tmp, mag_tmp);
  if (rc != ORACLE_OK) return rc;
  for (int64_t i = 0; i < num_dst; ++i) {
    for (int32_t j = 0; j < out_dim; ++j) {
      const double *wj = w + (int64_t)j * 2 * dim;
      double s = bias ? bias[j] : 0.0;
      double a = s < 0 ? -s : s;
      for (int32_t c = 0; c < dim; ++c) {
        int64_t at = i * dim + c;
        double own = elem_bytes == 2 ? oracle_half_to_double(((const uint16_t *)x)[at])
                                     : (double)((const float *)x)[at];
        double w_own = wj[c], w_agg = wj[dim + c];
        s += w_own * own + w_agg * mean_tmp[at];
        a += (w_own < 0 ? -w_own : w_own) * (own < 0 ? -own : own) +
             (w_agg < 0 ? -w_agg : w_agg) * mag_tmp[at];
      }
      out[i * out_dim + j] = (relu && s < 0.0) ? 0.0 : s;
      mag[i * out_dim + j] = a;
    }
  }
  return ORACLE_OK;
}

/* ---- multi-hop MFG + feature slice ------------------------------------------------------- */

/*
 * local_of: caller scratch [num_nodes], every entry -1 on entry; restored to -1 on return.
 * node_ids [node_capacity]; blk_indptr[h] [node_capacity + 1]; blk_indices[h] [edge_capacity[h]];
 * out_feat [node_capacity * row_bytes] or NULL; counts [2L+2] = n_0..n_L, E_0..E_{L-1}, status.
 * Returns ORACLE_ERR_ARG for malformed arguments, else the status (0 = ok).
 */
int32_t oracle_sample_mfg(int64_t num_nodes, const int64_t *indptr, const int32_t *indices,
                          const void *feat, int64_t row_bytes, int64_t row_stride,
                          const int32_t *seeds, int32_t num_seeds,
                          const int32_t *fanouts, int32_t L, uint64_t rng_key,
                          int32_t *local_of, int64_t node_capacity, const int64_t *edge_capacity,
                          int32_t *node_ids, int32_t *const *blk_indptr, int32_t *const *blk_indices,
                          void *out_feat, int64_t *counts) {
  if (!indptr || !seeds || !fanouts || !local_of || !node_ids || !blk_indptr || !blk_indices ||
      !edge_capacity || !counts || L < 1 || num_seeds < 0 || num_nodes < 0)
    return ORACLE_ERR_ARG;
  int32_t status = ORACLE_OK;
  int64_t n = 0; /* size of the ordered map M */
  for (int32_t q = 0; q < 2 * L + 2; ++q) counts[q] = 0;

  /* M starts with the destination nodes of hop 0, in the order given. */
  for (int32_t i = 0; i < num_seeds && status == ORACLE_OK; ++i) {
    int32_t v = seeds[i];
    if (v < 0 || (int64_t)v >= num_nodes) { status = ORACLE_ST_SEED_RANGE; break; }
    if (local_of[v] >= 0) { status = ORACLE_ST_DUP_SEED; break; }
    if (n >= node_capacity) { status = ORACLE_ST_NODE_CAPACITY; break; }
    local_of[v] = (int32_t)n;
    node_ids[n++] = v;
  }
  counts[0] = n;

  uint32_t *p = NULL;
  for (int32_t h = 0; h < L && status == ORACLE_OK; ++h) {
    int32_t d = fanouts[h];
    if (d < 1 && d != -1) { status = ORACLE_ERR_ARG; break; }
    size_t p_cap = 0;
    int64_t n_dst = n; /* snapshot: nodes met during this hop are not expanded in it */
    int64_t e = 0;
    int32_t *bp = blk_indptr[h], *bi = blk_indices[h];
    bp[0] = 0;
    for (int64_t i = 0; i < n_dst && status == ORACLE_OK; ++i) {
      int32_t v = node_ids[i];
      int64_t a = indptr[v];
      uint32_t deg = (uint32_t)(indptr[v + 1] - a);
      size_t need = (d == -1 || deg <= (uint32_t)d) ? deg : (size_t)d;
      if (need > p_cap) { p_cap = need; p = (uint32_t *)realloc(p, sizeof(uint32_t) * p_cap); }
      int32_t k = oracle_sample_positions(deg, d, rng_key, (uint32_t)v, (uint32_t)h, p);
      for (int32_t s = 0; s < k; ++s) {
        int32_t g = indices[a + (int64_t)p[s]];
        if (local_of[g] < 0) { /* first encounter: next local id */
          if (n >= node_capacity) { status = ORACLE_ST_NODE_CAPACITY; break; }
          local_of[g] = (int32_t)n;
          node_ids[n++] = g;
        }
        if (e >= edge_capacity[h]) { status = ORACLE_ST_EDGE_CAPACITY; break; }
        bi[e++] = local_of[g];
      }
      bp[i + 1] = (int32_t)e;
    }
    counts[h + 1] = n;
    counts[L + 1 + h] = e;
  }
  free(p);

  if (status == ORACLE_OK && out_feat && feat) {
    for (int64_t j = 0; j < n; ++j)
      memcpy((char *)out_feat + j * row_bytes, (const char *)feat + (int64_t)node_ids[j] * row_stride,
             (size_t)row_bytes);
  }
  for (int64_t j = 0; j < n; ++j) local_of[node_ids[j]] = -1;
  counts[2 * L + 1] = status;
  return status;
}
