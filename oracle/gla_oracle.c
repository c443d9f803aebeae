/*
 * CPU oracle for decode attention over a paged latent / tied-state cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and is
 * only ever loaded by the tests, the smoke check and the benchmark's CPU
 * baseline leg.
 *
 * What it computes (written from the paper, in its notation):
 *
 *   GLA, absorbed decode (Section 3.3.2; the score with the decoupled RoPE
 *   term is the sum form given for MLA in Section 2.1): the query heads are
 *   split into h_c groups of g_q = h_q / h_c consecutive heads; head h of group
 *   g = h / g_q attends to latent head c_g only,
 *        s_j  = scale * ( q_nope . c_g[j]  +  q_rope . k_rope[j] )
 *        p    = softmax_j(s)
 *        out  = sum_j p_j * c_g[j]                       (latent-space output)
 *   The RoPE key k_rope[j] is ONE vector per token shared by every head.
 *
 *   GTA (Section 3.3.1): the tied state of group g is the value V; the key is
 *   concat(first d_n = d_h/2 dims of the tied state, shared RoPE key); so the
 *   same formula applies with the dot product q_nope . c_g[j] running over the
 *   first d_n dims only while the output uses all d_v dims.
 *
 *   Visible keys: key j of sequence b is visible to query row t (0-based, of T
 *   rows that are the LAST T cached positions) iff j < L_b - T + 1 + t when
 *   causal, j < L_b otherwise.  A row with no visible key yields out = 0 and
 *   lse = -infinity.
 *
 *   lse = m + ln( sum_j exp(s_j - m) ),  m = max_j s_j   (natural log).
 *
 * Everything is two-pass and accumulated in fp64; bf16 inputs are widened
 * exactly.  No blocking, no online softmax, no fusion.
 *
 * The two projections around the attention (gla_oracle_project, at the end of
 * this file): the key up-projection absorbed on the query side (Section 2.1)
 * and the grouped output projection with the value up-projection absorbed
 * (Section 3.3.2), both as plain fp64 sums.
 *
 * Pins (tests/test_oracle_pins.py): equality with explicit up-projected
 * attention, with an assembled-K GQA for GTA, closed forms, paging invariance,
 * split/merge identity; for the projections: the whole absorbed block against
 * explicit per-head attention with separate W_UK, W_UV, W_O, numpy products,
 * identity weights; for the grouped-query baseline: textbook attention on the
 * gathered keys and values, and GTA as the special case whose key is assembled
 * from the tied state and the shared RoPE key.  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_to_f64(uint16_t v) {
  uint32_t u = ((uint32_t)v) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* Number of threads the parallel loops will use. */
int gla_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * One decode call.
 *
 *  q_nope      [B, T, h_q, d_n]   bf16 bits
 *  q_rope      [B, T, h_q, d_r]   bf16 bits (ignored when d_r == 0)
 *  state       [n_pages, h_c, P, d_v] bf16 bits
 *  rope        [n_pages, P, d_r]  bf16 bits
 *  page_table  [B, max_pages]     int32; entries past ceil(L_b / P) never read
 *  seq_lens    [B]                int32
 *  key_begin, key_end             only keys j in [key_begin, key_end) take part
 *                                 (pass 0 and INT64_MAX for the whole context);
 *                                 used to produce the partial results of a
 *                                 split over the key axis
 *  sel, n_sel                     optional list of (b, t, h) int32 triples; when
 *                                 given only those rows are computed and the
 *                                 outputs are indexed by list position
 *  out         [rows, d_v] fp64, lse [rows] fp64
 *  weights     optional [rows, w_stride] fp64 softmax weights (0 beyond the
 *              visible range), for the row-sum pin
 *
 *  returns 0, or -1 on a bad argument.
 */
int gla_oracle_decode(const uint16_t* q_nope, const uint16_t* q_rope, const uint16_t* state,
                      const uint16_t* rope, const int32_t* page_table, const int32_t* seq_lens,
                      int B, int T, int h_q, int h_c, int d_v, int d_n, int d_r, int P,
                      int max_pages, double scale, int causal, int64_t key_begin,
                      int64_t key_end, const int32_t* sel, int64_t n_sel, double* out,
                      double* lse, double* weights, int64_t w_stride) {
  if (B < 0 || T < 1 || h_q < 1 || h_c < 1 || h_q % h_c != 0 || d_v < 1 || d_n < 0 ||
      d_n > d_v || d_r < 0 || P < 1)
    return -1;
  const int g_q = h_q / h_c;
  const int64_t rows = sel ? n_sel : (int64_t)B * T * h_q;
  int64_t max_len = 0;
  for (int b = 0; b < B; ++b)
    if (seq_lens[b] > max_len) max_len = seq_lens[b];
  int failed = 0;

#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
    if (!s) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
      if (!s) continue;
      int b, t, h;
      if (sel) {
        b = sel[3 * r + 0];
        t = sel[3 * r + 1];
        h = sel[3 * r + 2];
      } else {
        b = (int)(r / ((int64_t)T * h_q));
        t = (int)((r / h_q) % T);
        h = (int)(r % h_q);
      }
      const int g = h / g_q;
      const int64_t L = seq_lens[b];
      int64_t n_vis = causal ? L - T + 1 + t : L;
      int64_t j0 = key_begin > 0 ? key_begin : 0;
      int64_t j1 = key_end < n_vis ? key_end : n_vis;
      double* o = out + r * d_v;
      for (int d = 0; d < d_v; ++d) o[d] = 0.0;
      if (weights)
        for (int64_t j = 0; j < w_stride; ++j) weights[r * w_stride + j] = 0.0;
      if (j1 <= j0) {
        lse[r] = -INFINITY;
        continue;
      }
      const uint16_t* qn = q_nope + (((int64_t)b * T + t) * h_q + h) * d_n;
      const uint16_t* qr = q_rope ? q_rope + (((int64_t)b * T + t) * h_q + h) * d_r : NULL;

      /* pass 1: scores and their maximum */
      double m = -INFINITY;
      for (int64_t j = j0; j < j1; ++j) {
        const int64_t page = page_table[(int64_t)b * max_pages + j / P];
        const int64_t off = j % P;
        const uint16_t* c = state + ((page * h_c + g) * P + off) * d_v;
        double acc = 0.0;
        for (int d = 0; d < d_n; ++d) acc += bf16_to_f64(qn[d]) * bf16_to_f64(c[d]);
        if (d_r > 0) {
          const uint16_t* k = rope + (page * P + off) * d_r;
          for (int d = 0; d < d_r; ++d) acc += bf16_to_f64(qr[d]) * bf16_to_f64(k[d]);
        }
        const double sj = scale * acc;
        s[j - j0] = sj;
        if (sj > m) m = sj;
      }
      /* pass 2: normaliser */
      double l = 0.0;
      for (int64_t j = j0; j < j1; ++j) l += exp(s[j - j0] - m);
      lse[r] = m + log(l);
      /* pass 3: weighted sum of the SAME cached vectors (all d_v dims) */
      for (int64_t j = j0; j < j1; ++j) {
        const double p = exp(s[j - j0] - m) / l;
        if (weights && j < w_stride) weights[r * w_stride + j] = p;
        const int64_t page = page_table[(int64_t)b * max_pages + j / P];
        const int64_t off = j % P;
        const uint16_t* c = state + ((page * h_c + g) * P + off) * d_v;
        for (int d = 0; d < d_v; ++d) o[d] += p * bf16_to_f64(c[d]);
      }
    }
    free(s);
  }
  return failed ? -1 : 0;
}

/*
 * Merge of partial results taken over disjoint key ranges.  Softmax over a
 * union of ranges, written in terms of each range's own normalised output O_s
 * and log-sum-exp lse_s:
 *      lse = ln sum_s exp(lse_s)
 *      out = sum_s exp(lse_s - lse) * O_s
 * A part with lse_s = -inf (no keys) contributes nothing; if every part is
 * empty the result is out = 0, lse = -inf.
 *
 *  part_out [n_parts, rows, d_v], part_lse [n_parts, rows]
 */
int gla_oracle_merge(const double* part_out, const double* part_lse, int n_parts, int64_t rows,
                     int d_v, double* out, double* lse) {
  if (n_parts < 1 || rows < 0 || d_v < 1) return -1;
  for (int64_t r = 0; r < rows; ++r) {
    double m = -INFINITY;
    for (int s = 0; s < n_parts; ++s)
      if (part_lse[(int64_t)s * rows + r] > m) m = part_lse[(int64_t)s * rows + r];
    double* o = out + r * d_v;
    for (int d = 0; d < d_v; ++d) o[d] = 0.0;
    if (m == -INFINITY) {
      lse[r] = -INFINITY;
      continue;
    }
    double z = 0.0;
    for (int s = 0; s < n_parts; ++s) z += exp(part_lse[(int64_t)s * rows + r] - m);
    const double total = m + log(z);
    lse[r] = total;
    for (int s = 0; s < n_parts; ++s) {
      const double ls = part_lse[(int64_t)s * rows + r];
      if (ls == -INFINITY) continue;
      const double w = exp(ls - total);
      const double* po = part_out + ((int64_t)s * rows + r) * d_v;
      for (int d = 0; d < d_v; ++d) o[d] += w * po[d];
    }
  }
  return 0;
}

/*
 * The projections on either side of the attention, both instances of
 *
 *      C[m][g][n] = sum_k A[m][g][k] * W[g][n][k]          (sum_groups == 0)
 *      C[m][n]    = sum_g sum_k A[m][g][k] * W[g][n][k]    (sum_groups != 0)
 *
 * Query side (Section 2.1): with W = W_UK of head g (latent dim n, head dim k)
 * and A the raw per-head queries, C is the absorbed query that scores directly
 * against the latent: q . (W_UK^T c) == (W_UK q) . c.
 * Output side (Section 3.3.2): with A the latent-space attention output of group
 * g (its heads' outputs side by side, k over g_q * d_c) and W = W_g^vo stored
 * output-major, the sum over groups is the block's output; with several devices
 * that sum is the all-reduce.
 *
 * a: bf16 bits, element strides (row m, group g), k contiguous
 * w: bf16 bits [G][N][K] contiguous
 * c: fp64 [M][G][N] or [M][N] contiguous
 * returns 0, or -1 on a bad argument.
 */
int gla_oracle_project(const uint16_t* a, int64_t a_row_stride, int64_t a_group_stride,
                       const uint16_t* w, int M, int G, int N, int K, int sum_groups, double* c) {
  if (M < 0 || G < 1 || N < 1 || K < 1) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t mn = 0; mn < (int64_t)M * N; ++mn) {
    const int m = (int)(mn / N), n = (int)(mn % N);
    double total = 0.0;
    for (int g = 0; g < G; ++g) {
      const uint16_t* ar = a + m * a_row_stride + g * a_group_stride;
      const uint16_t* wr = w + ((int64_t)g * N + n) * K;
      double acc = 0.0;
      for (int k = 0; k < K; ++k) acc += bf16_to_f64(ar[k]) * bf16_to_f64(wr[k]);
      if (sum_groups) total += acc;
      else c[((int64_t)m * G + g) * N + n] = acc;
    }
    if (sum_groups) c[(int64_t)m * N + n] = total;
  }
  return 0;
}

/*
 * Grouped-query attention decode with keys and values in separate paged caches:
 * the baseline Grouped-Tied Attention is measured against (Section 3.3.1: the
 * tied state replaces the separate key and value of a GQA group, halving the
 * cache).  Plain definition, two-pass, fp64:
 *
 *      s_j = scale * q . K[j],   p = softmax_j(s),   out = sum_j p_j V[j]
 *
 * for query head h with its group's key / value head g = h / (h_q / h_kv); the
 * rotary embedding is already part of q and of the cached keys.  Visible keys
 * and empty rows as in gla_oracle_decode.
 *
 *  q        [B, T, h_q, d_k]       bf16 bits
 *  kcache   [n_pages, h_kv, P, d_k], vcache [n_pages, h_kv, P, d_v]   bf16 bits
 *  sel / n_sel, out [rows, d_v], lse [rows] as in gla_oracle_decode
 */
int gla_oracle_gqa_decode(const uint16_t* q, const uint16_t* kcache, const uint16_t* vcache,
                          const int32_t* page_table, const int32_t* seq_lens, int B, int T, int h_q,
                          int h_kv, int d_k, int d_v, int P, int max_pages, double scale, int causal,
                          const int32_t* sel, int64_t n_sel, double* out, double* lse) {
  if (B < 0 || T < 1 || h_q < 1 || h_kv < 1 || h_q % h_kv != 0 || d_k < 1 || d_v < 1 || P < 1) return -1;
  const int g_q = h_q / h_kv;
  const int64_t rows = sel ? n_sel : (int64_t)B * T * h_q;
  int64_t max_len = 0;
  for (int b = 0; b < B; ++b)
    if (seq_lens[b] > max_len) max_len = seq_lens[b];
  int failed = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
    if (!s) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
      if (!s) continue;
      const int b = sel ? sel[3 * r] : (int)(r / ((int64_t)T * h_q));
      const int t = sel ? sel[3 * r + 1] : (int)((r / h_q) % T);
      const int h = sel ? sel[3 * r + 2] : (int)(r % h_q);
      const int g = h / g_q;
      const int64_t L = seq_lens[b];
      const int64_t n_vis = causal ? L - T + 1 + t : L;
      double* o = out + r * d_v;
      for (int d = 0; d < d_v; ++d) o[d] = 0.0;
      if (n_vis <= 0) {
        lse[r] = -INFINITY;
        continue;
      }
      const uint16_t* qv = q + (((int64_t)b * T + t) * h_q + h) * d_k;
      double m = -INFINITY;
      for (int64_t j = 0; j < n_vis; ++j) {
        const int64_t page = page_table[(int64_t)b * max_pages + j / P];
        const uint16_t* k = kcache + ((page * h_kv + g) * P + j % P) * d_k;
        double acc = 0.0;
        for (int d = 0; d < d_k; ++d) acc += bf16_to_f64(qv[d]) * bf16_to_f64(k[d]);
        s[j] = scale * acc;
        if (s[j] > m) m = s[j];
      }
      double l = 0.0;
      for (int64_t j = 0; j < n_vis; ++j) l += exp(s[j] - m);
      lse[r] = m + log(l);
      for (int64_t j = 0; j < n_vis; ++j) {
        const double pj = exp(s[j] - m) / l;
        const int64_t page = page_table[(int64_t)b * max_pages + j / P];
        const uint16_t* v = vcache + ((page * h_kv + g) * P + j % P) * d_v;
        for (int d = 0; d < d_v; ++d) o[d] += pj * bf16_to_f64(v[d]);
      }
    }
    free(s);
  }
  return failed ? -1 : 0;
}
