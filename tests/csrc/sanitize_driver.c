/*
 * Driver for the sanitizer run of the CPU oracle (tests/test_oracle_sanitizers.py builds this file
 * together with oracle/dsmoe_oracle.c under -fsanitize=address,undefined and runs it).  It walks the
 * grid of tiny layers the oracle's brute-force pins use, with every buffer allocated at exactly its
 * size, so that an access one element past any argument is reported.  It also checks three facts that
 * need no second implementation: outputs are finite, thresholds of 2 give an all-zero routed output,
 * and with nothing dropped the output does not depend on the number of partitions.
 * Prints "sanitize_driver: ok <cases>" and returns 0 unless a check fails.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int dsmoe_oracle_route(const float* logits, int T, int E, int K, int P, const float* tau, int lo, int hi, int renorm,
                       int32_t* idx, double* s, double* n, double* g, uint8_t* keep, int64_t* group_count, double* min_margin);
int dsmoe_oracle_forward(const void* x, const float* logits, const void* w1, const void* w3, const void* w2, const void* sh_w1,
                         const void* sh_w3, const void* sh_w2, const int32_t* perm, const float* tau, int T, int D, int F, int E,
                         int K, int P, int n_shared, int F_sh, int lo, int hi, int renorm, int dtype, const int32_t* tokens,
                         int n_tokens, double* y);
int dsmoe_oracle_importance(const void* x, const float* logits, const void* w1, const void* w3, int T, int D, int F, int E, int K,
                            int lo, int hi, int dtype, int metric, double* imp, double* abs_sum);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform(void) { /* (0, 1), a 64-bit linear congruential generator */
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return ((double)(rng_state >> 11) + 0.5) / 9007199254740992.0;
}
static double normal(void) { return sqrt(-2.0 * log(uniform())) * cos(6.283185307179586 * uniform()); }

static uint16_t to_bf16(float f) { /* round to nearest even */
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

/* n values ~ N(0, std) in the layer's element type (dtype 0: float, 1: bf16 bits) */
static void* tensor(size_t n, double std, int dtype) {
  void* p = malloc(n ? n * (dtype ? 2 : 4) : 1);
  if (!p) exit(3);
  for (size_t i = 0; i < n; ++i) {
    const float v = (float)(std * normal());
    if (dtype) ((uint16_t*)p)[i] = to_bf16(v);
    else ((float*)p)[i] = v;
  }
  return p;
}

static int check(int ok, const char* what, int T, int D, int F, int E, int K, int P) {
  if (!ok) fprintf(stderr, "sanitize_driver: %s failed at T=%d D=%d F=%d E=%d K=%d P=%d\n", what, T, D, F, E, K, P);
  return ok ? 0 : 1;
}

int main(void) {
  static const int Ts[] = {0, 1, 3, 64}, Ds[] = {8, 24}, Fs[] = {8, 48}, Es[] = {1, 2, 8}, Ps[] = {1, 2, 4};
  int cases = 0, bad = 0;
  for (int ti = 0; ti < 4; ++ti)
    for (int di = 0; di < 2; ++di)
      for (int fi = 0; fi < 2; ++fi)
        for (int ei = 0; ei < 3; ++ei)
          for (int kk = 0; kk < 3; ++kk)
            for (int dtype = 0; dtype < 2; ++dtype) {
              const int T = Ts[ti], D = Ds[di], F = Fs[fi], E = Es[ei];
              const int K = kk == 0 ? 1 : kk == 1 ? (E < 2 ? E : 2) : E;
              if (kk == 1 && K == 1) continue;
              if (kk == 2 && K <= 2 && E <= 2 && kk != E) continue;
              const int n_shared = (ei == 2 && di == 1) ? 2 : 0, F_sh = 12;
              const int lo = (E == 8 && fi == 1) ? 2 : 0, hi = (E == 8 && fi == 1) ? 7 : E, E_res = hi - lo;
              void* x = tensor((size_t)T * D, 1.0, dtype);
              float* logits = (float*)tensor((size_t)T * E, 1.0, 0);
              void* w1 = tensor((size_t)E_res * D * F, 0.3, dtype);
              void* w3 = tensor((size_t)E_res * D * F, 0.3, dtype);
              void* w2 = tensor((size_t)E_res * F * D, 0.3, dtype);
              void* s1 = n_shared ? tensor((size_t)n_shared * D * F_sh, 0.3, dtype) : NULL;
              void* s3 = n_shared ? tensor((size_t)n_shared * D * F_sh, 0.3, dtype) : NULL;
              void* s2 = n_shared ? tensor((size_t)n_shared * F_sh * D, 0.3, dtype) : NULL;
              int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)E_res * F);
              for (int e = 0; e < E_res; ++e)
                for (int j = 0; j < F; ++j) perm[(size_t)e * F + j] = (j * 5 + 3 + e) % F; /* a bijection: F is 8 or 48, 5 is coprime */
              double* y_first = NULL;
              for (int pi = 0; pi < 3; ++pi) {
                const int P = Ps[pi];
                ++cases;
                float* tau = (float*)malloc(sizeof(float) * (size_t)E * P);
                int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T * K ? T * K : 1));
                double* sc = (double*)malloc(sizeof(double) * (size_t)(T * K ? T * K : 1));
                double* nn = (double*)malloc(sizeof(double) * (size_t)(T * K ? T * K : 1));
                double* gg = (double*)malloc(sizeof(double) * (size_t)(T * K ? T * K : 1));
                uint8_t* keep = (uint8_t*)malloc((size_t)(T * K * P ? T * K * P : 1));
                int64_t* gc = (int64_t*)malloc(sizeof(int64_t) * (size_t)E * P);
                double* y = (double*)malloc(sizeof(double) * (size_t)(T * D ? T * D : 1));
                double margin = 0;
                /* per-partition thresholds that drop some units */
                for (int i = 0; i < E * P; ++i) tau[i] = 0.15f + 0.1f * (float)(i % P);
                bad += check(dsmoe_oracle_route(logits, T, E, K, P, tau, lo, hi, pi & 1, idx, sc, nn, gg, keep, gc, &margin) == 0,
                             "route", T, D, F, E, K, P);
                bad += check(dsmoe_oracle_forward(x, logits, w1, w3, w2, s1, s3, s2, perm, tau, T, D, F, E, K, P, n_shared, F_sh, lo,
                                                  hi, pi & 1, dtype, NULL, T, y) == 0,
                             "forward", T, D, F, E, K, P);
                for (int i = 0; i < T * D; ++i) bad += check(isfinite(y[i]), "finite output", T, D, F, E, K, P);
                /* a token subset, in reverse order */
                if (T >= 3) {
                  int32_t tok[2] = {T - 1, 0};
                  double* ys = (double*)malloc(sizeof(double) * 2 * (size_t)D);
                  bad += check(dsmoe_oracle_forward(x, logits, w1, w3, w2, s1, s3, s2, perm, tau, T, D, F, E, K, P, n_shared, F_sh,
                                                    lo, hi, pi & 1, dtype, tok, 2, ys) == 0,
                               "forward on a token list", T, D, F, E, K, P);
                  for (int d = 0; d < D; ++d)
                    bad += check(ys[d] == y[(size_t)(T - 1) * D + d] && ys[D + d] == y[d], "token list rows", T, D, F, E, K, P);
                  free(ys);
                }
                /* everything dropped: the routed output is exactly zero (shared experts aside) */
                for (int i = 0; i < E * P; ++i) tau[i] = 2.0f;
                dsmoe_oracle_forward(x, logits, w1, w3, w2, NULL, NULL, NULL, perm, tau, T, D, F, E, K, P, 0, 0, lo, hi, 0, dtype,
                                     NULL, T, y);
                for (int i = 0; i < T * D; ++i) bad += check(y[i] == 0.0, "all dropped -> zero", T, D, F, E, K, P);
                /* nothing dropped: the same output for every P */
                for (int i = 0; i < E * P; ++i) tau[i] = 0.0f;
                dsmoe_oracle_forward(x, logits, w1, w3, w2, s1, s3, s2, perm, tau, T, D, F, E, K, P, n_shared, F_sh, lo, hi, 0, dtype,
                                     NULL, T, y);
                if (!y_first) {
                  y_first = (double*)malloc(sizeof(double) * (size_t)(T * D ? T * D : 1));
                  memcpy(y_first, y, sizeof(double) * (size_t)T * D);
                } else {
                  for (int i = 0; i < T * D; ++i)
                    bad += check(fabs(y[i] - y_first[i]) <= 1e-11 * (1.0 + fabs(y_first[i])), "partition invariance", T, D, F, E, K, P);
                }
                free(tau), free(idx), free(sc), free(nn), free(gg), free(keep), free(gc), free(y);
              }
              /* importance of the calibration tokens, the four metrics */
              for (int metric = 0; metric < 4; ++metric) {
                double* imp = (double*)malloc(sizeof(double) * (size_t)E_res * F);
                double* ab = (double*)malloc(sizeof(double) * (size_t)E_res * F);
                bad += check(dsmoe_oracle_importance(x, logits, w1, w3, T, D, F, E, K, lo, hi, dtype, metric, imp, ab) == 0,
                             "importance", T, D, F, E, K, 1);
                for (int i = 0; i < E_res * F; ++i) bad += check(isfinite(imp[i]) && fabs(imp[i]) <= ab[i] * (1 + 1e-12) + 1e-300, "importance bound", T, D, F, E, K, 1);
                free(imp), free(ab);
              }
              free(y_first), free(x), free(logits), free(w1), free(w3), free(w2), free(s1), free(s3), free(s2), free(perm);
            }
  if (bad) {
    fprintf(stderr, "sanitize_driver: %d checks failed\n", bad);
    return 1;
  }
  printf("sanitize_driver: ok %d\n", cases);
  return 0;
}
