/*
 * fp64 CPU oracle for the forward pass of a partitioned, computation-dropping MoE FFN layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the layer computes,
 * written token by token with no grouping, tiling or reordering of work.  It shares no code with
 * the GPU library and must never be called from the product path; only the test-suite, the smoke
 * check and the CPU-baseline leg of the benchmark use it.
 *
 * What it follows (DualSparse-MoE, arXiv 2508.18376):
 *   - gating: softmax over all E router logits (Sec. 2.1.1, Eq. 1; Sec. 3.1 score formula),
 *     Top-K selection (Sec. 2.1.1, Eq. 2), weighted sum of expert outputs (Eq. 3);
 *   - SwiGLU expert f(x) = (Swish(x W1) * (x W3)) W2 with Swish(a) = a * sigmoid(a) (Eq. 4);
 *   - partial transformation: each expert's (reordered) neurons are split evenly into P
 *     contiguous sub-experts, the gate score of the expert is repeated for its sub-experts and
 *     W2 is not rescaled (Sec. 3.2);
 *   - reconstruction: neuron order inside an expert is given by a static permutation, partition 0
 *     holding the most important neurons (Sec. 4.2 b);
 *   - dropping: the K selected scores are normalised to sum to one; unit (token, expert,
 *     partition p) is computed iff the normalised score is not below that partition's threshold;
 *     a kept unit is still weighted by the original gate score (Sec. 4.1, Sec. 4.2 c).  With
 *     renorm != 0 the combine weight is the normalised score, for models that normalise anyway.
 *   - load-aware thresholds enter only as a per-expert threshold table (Sec. 4.3).
 *   - shared experts are always on, weight 1, never partitioned or dropped (Sec. 5.3.1 text).
 *   - neuron importance profiling: the four accumulated metrics of Sec. 4.2 b.
 *
 * Readings where the text leaves a choice: Top-K is taken on the logits, ordered by value
 * descending then index ascending (ties go to the lower index); a unit is kept iff n >= tau
 * (only scores strictly below the threshold are dropped); the normalised score is not divided by
 * P; the keep decision is taken after rounding n to float, the precision the GPU kernel decides
 * in, against the float threshold.
 *
 * The weights are indexed in their ORIGINAL layout through perm; no partitioned copy is built.
 * Element type of x / weights: dtype 0 = float, 1 = bf16 bit patterns (widened exactly).
 * All arithmetic is double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double ld_elem(const void* p, int dtype, size_t i) {
  if (dtype == 0) return (double)((const float*)p)[i];
  uint32_t u = ((uint32_t)((const uint16_t*)p)[i]) << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

int dsmoe_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * Gating of one token.  logits: E floats.  Outputs for the K slots, in selection order:
 * idx (expert id), s (softmax score), n (score normalised over the K selected).
 */
static void gate_token(const float* logits, int E, int K, int32_t* idx, double* s, double* n) {
  /* Top-K on the logits: K rounds, each taking the largest not yet taken; a later index only
   * wins if strictly larger, so equal values go to the lower index (Eq. 2). */
  for (int k = 0; k < K; ++k) {
    int best = -1;
    for (int e = 0; e < E; ++e) {
      int taken = 0;
      for (int j = 0; j < k; ++j) taken |= (idx[j] == e);
      if (taken) continue;
      if (best < 0 || logits[e] > logits[best]) best = e;
    }
    idx[k] = best;
  }
  /* softmax over all E (Eq. 1), shifted by the maximum */
  double m = (double)logits[0];
  for (int e = 1; e < E; ++e)
    if ((double)logits[e] > m) m = (double)logits[e];
  double z = 0.0;
  for (int e = 0; e < E; ++e) z += exp((double)logits[e] - m);
  double sel = 0.0;
  for (int k = 0; k < K; ++k) {
    s[k] = exp((double)logits[idx[k]] - m) / z;
    sel += s[k];
  }
  /* normalise the K selected scores (Sec. 4.1) */
  for (int k = 0; k < K; ++k) n[k] = s[k] / sel;
}

/*
 * Routing and drop mask for all tokens.
 *   logits [T][E] float; tau [E][P] float (row = global expert id, column = partition).
 *   Experts outside [lo, hi) are not resident: their units are never kept here.
 * Outputs (any may be NULL): idx [T][K]; s, n, g [T][K] double; keep [T][K][P] (0/1);
 *   group_count [E*P] kept units per sub-expert e*P+p (Sec. 3.2 index remap);
 *   min_margin: smallest |n - tau| over all (token, slot, partition) of resident experts.
 */
int dsmoe_oracle_route(const float* logits, int T, int E, int K, int P, const float* tau, int lo, int hi,
                       int renorm, int32_t* idx, double* s, double* n, double* g, uint8_t* keep,
                       int64_t* group_count, double* min_margin) {
  if (T < 0 || E < 1 || K < 1 || K > E || P < 1 || lo < 0 || hi > E || lo > hi) return -1;
  if (group_count) memset(group_count, 0, sizeof(int64_t) * (size_t)E * P);
  double margin = INFINITY;
  int32_t* ti = (int32_t*)malloc(sizeof(int32_t) * K);
  double* ts = (double*)malloc(sizeof(double) * K);
  double* tn = (double*)malloc(sizeof(double) * K);
  for (int t = 0; t < T; ++t) {
    gate_token(logits + (size_t)t * E, E, K, ti, ts, tn);
    for (int k = 0; k < K; ++k) {
      size_t o = (size_t)t * K + k;
      int e = ti[k];
      if (idx) idx[o] = e;
      if (s) s[o] = ts[k];
      if (n) n[o] = tn[k];
      if (g) g[o] = renorm ? tn[k] : ts[k];
      for (int p = 0; p < P; ++p) {
        int kept = 0;
        if (e >= lo && e < hi) {
          float thr = tau[(size_t)e * P + p];
          kept = ((float)tn[k] >= thr);
          double d = fabs(tn[k] - (double)thr);
          if (d < margin) margin = d;
        }
        if (keep) keep[o * P + p] = (uint8_t)kept;
        if (kept && group_count) group_count[(size_t)e * P + p] += 1;
      }
    }
  }
  free(ti);
  free(ts);
  free(tn);
  if (min_margin) *min_margin = margin;
  return 0;
}

/* a[q] = sum_d x[d] * W[d][q] for all q (W is [D][F], row d contiguous) */
static void xw(const void* x, size_t xoff, const void* w, size_t woff, int D, int F, int dtype, double* a) {
  for (int q = 0; q < F; ++q) a[q] = 0.0;
  for (int d = 0; d < D; ++d) {
    double xd = ld_elem(x, dtype, xoff + d);
    size_t row = woff + (size_t)d * F;
    for (int q = 0; q < F; ++q) a[q] += xd * ld_elem(w, dtype, row + q);
  }
}

static inline double swish(double a) { return a / (1.0 + exp(-a)); }

/*
 * Layer output for a list of tokens.
 *   x [T][D]; logits [T][E]; w1, w3 [hi-lo][D][F]; w2 [hi-lo][F][D] (resident experts only, in
 *   id order); sh_w1, sh_w3 [n_shared][D][F_sh]; sh_w2 [n_shared][F_sh][D];
 *   perm [hi-lo][F] (perm[e][j] = original neuron at new position j; NULL = identity);
 *   tau [E][P]; tokens: n_tokens token ids (NULL = 0..n_tokens-1).
 *   y [n_tokens][D] double: row i is the output of token tokens[i].
 * Returns 0, or -1 on a bad argument.
 */
int dsmoe_oracle_forward(const void* x, const float* logits, const void* w1, const void* w3, const void* w2,
                         const void* sh_w1, const void* sh_w3, const void* sh_w2, const int32_t* perm,
                         const float* tau, int T, int D, int F, int E, int K, int P, int n_shared, int F_sh,
                         int lo, int hi, int renorm, int dtype, const int32_t* tokens, int n_tokens, double* y) {
  if (T < 0 || D < 1 || F < 1 || E < 1 || K < 1 || K > E || P < 1 || F % P != 0) return -1;
  if (lo < 0 || hi > E || lo > hi || n_shared < 0 || (n_shared > 0 && F_sh < 1)) return -1;
  if (dtype != 0 && dtype != 1) return -1;
  const int Fp = F / P;
  const int Fmax = F > F_sh ? F : F_sh;
  int bad = 0;
#pragma omp parallel
  {
    double* a = (double*)malloc(sizeof(double) * Fmax);
    double* b = (double*)malloc(sizeof(double) * Fmax);
    int32_t* ti = (int32_t*)malloc(sizeof(int32_t) * K);
    double* ts = (double*)malloc(sizeof(double) * K);
    double* tn = (double*)malloc(sizeof(double) * K);
#pragma omp for schedule(dynamic, 1)
    for (int i = 0; i < n_tokens; ++i) {
      int t = tokens ? tokens[i] : i;
      double* yt = y + (size_t)i * D;
      for (int d = 0; d < D; ++d) yt[d] = 0.0;
      if (t < 0 || t >= T) {
#pragma omp atomic write
        bad = 1;
        continue;
      }
      gate_token(logits + (size_t)t * E, E, K, ti, ts, tn);
      for (int k = 0; k < K; ++k) {
        int e = ti[k];
        if (e < lo || e >= hi) continue; /* computed on another device */
        double gk = renorm ? tn[k] : ts[k];
        int any = 0;
        for (int p = 0; p < P; ++p) any |= ((float)tn[k] >= tau[(size_t)e * P + p]);
        if (!any) continue;
        size_t r = (size_t)(e - lo);
        xw(x, (size_t)t * D, w1, r * D * F, D, F, dtype, a); /* gate projection, all neurons */
        xw(x, (size_t)t * D, w3, r * D * F, D, F, dtype, b); /* up projection */
        for (int p = 0; p < P; ++p) {
          if (!((float)tn[k] >= tau[(size_t)e * P + p])) continue; /* unit dropped */
          for (int j = p * Fp; j < (p + 1) * Fp; ++j) {
            int q = perm ? perm[r * F + j] : j; /* original neuron sitting at position j */
            double h = swish(a[q]) * b[q];
            size_t row = (r * F + q) * (size_t)D;
            for (int d = 0; d < D; ++d) yt[d] += gk * h * ld_elem(w2, dtype, row + d);
          }
        }
      }
      for (int sidx = 0; sidx < n_shared; ++sidx) {
        size_t r = (size_t)sidx;
        xw(x, (size_t)t * D, sh_w1, r * D * F_sh, D, F_sh, dtype, a);
        xw(x, (size_t)t * D, sh_w3, r * D * F_sh, D, F_sh, dtype, b);
        for (int q = 0; q < F_sh; ++q) {
          double h = swish(a[q]) * b[q];
          size_t row = (r * F_sh + q) * (size_t)D;
          for (int d = 0; d < D; ++d) yt[d] += h * ld_elem(sh_w2, dtype, row + d);
        }
      }
    }
    free(a);
    free(b);
    free(ti);
    free(ts);
    free(tn);
  }
  return bad ? -1 : 0;
}

/*
 * Neuron importance profiling on calibration tokens (Sec. 4.2 b, the four accumulated metrics):
 * for every resident expert e and ORIGINAL neuron q, the sum over the calibration tokens that
 * route to e (Top-K of Eq. 2, nothing dropped) of
 *   metric 0: Swish(x . W1[:, q])                      accumulated gate value
 *   metric 1: |Swish(x . W1[:, q])|                    accumulated absolute gate value
 *   metric 2: Swish(x . W1[:, q]) * (x . W3[:, q])     accumulated gate-up value
 *   metric 3: |Swish(x . W1[:, q]) * (x . W3[:, q])|   accumulated absolute gate-up value
 * imp [hi-lo][F] double.  abs_sum (may be NULL) [hi-lo][F]: the sum of the absolute values of the
 * same terms (the scale rounding errors of a reduced-precision implementation live on).
 */
int dsmoe_oracle_importance(const void* x, const float* logits, const void* w1, const void* w3, int T, int D, int F,
                            int E, int K, int lo, int hi, int dtype, int metric, double* imp, double* abs_sum) {
  if (T < 0 || D < 1 || F < 1 || E < 1 || K < 1 || K > E || lo < 0 || hi > E || lo > hi) return -1;
  if (metric < 0 || metric > 3 || (dtype != 0 && dtype != 1)) return -1;
  const size_t n = (size_t)(hi - lo) * F;
  for (size_t i = 0; i < n; ++i) imp[i] = 0.0;
  if (abs_sum)
    for (size_t i = 0; i < n; ++i) abs_sum[i] = 0.0;
  double* a = (double*)malloc(sizeof(double) * F);
  double* b = (double*)malloc(sizeof(double) * F);
  int32_t* ti = (int32_t*)malloc(sizeof(int32_t) * K);
  double* ts = (double*)malloc(sizeof(double) * K);
  double* tn = (double*)malloc(sizeof(double) * K);
  for (int t = 0; t < T; ++t) {
    gate_token(logits + (size_t)t * E, E, K, ti, ts, tn);
    for (int k = 0; k < K; ++k) {
      int e = ti[k];
      if (e < lo || e >= hi) continue;
      size_t r = (size_t)(e - lo);
      xw(x, (size_t)t * D, w1, r * D * F, D, F, dtype, a);
      if (metric >= 2) xw(x, (size_t)t * D, w3, r * D * F, D, F, dtype, b);
      for (int q = 0; q < F; ++q) {
        double v = swish(a[q]);
        if (metric >= 2) v *= b[q];
        imp[r * F + q] += (metric & 1) ? fabs(v) : v;
        if (abs_sum) abs_sum[r * F + q] += fabs(v);
      }
    }
  }
  free(a);
  free(b);
  free(ti);
  free(ts);
  free(tn);
  return 0;
}
