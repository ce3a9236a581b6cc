/*
 * Sanitizer driver for the oracle (test helper, CPU only): built by tests/test_oracle_sanitizers.py together with
 * oracle/flexspec_oracle.c under -fsanitize=address,undefined and run once.  It walks every entry point of the oracle
 * on a tiny model with awkward sizes (ragged vocabulary, GQA, a cache exactly as long as needed, rank-3 adapters,
 * bf16 and float weights, every storage-rounding mask, the top-k / top-p cuts, greedy and sampled modes), so that an
 * out-of-bounds index, a use after free or an overflowing shift anywhere in it ends the run with a report.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../oracle/flexspec_oracle.c"

static uint64_t rng = 0x9E3779B97F4A7C15ull;
static double unif(void) {   /* splitmix64 -> (0,1) */
  uint64_t z = (rng += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return ((double)(z >> 11) + 0.5) / 9007199254740992.0;
}
static double normal(void) { return sqrt(-2.0 * log(unif())) * cos(6.283185307179586 * unif()); }

/* a matrix of n values ~ N(mean, std) in the storage type of the model */
static void *matrix(size_t n, double mean, double std, int bf16) {
  if (bf16) {
    uint16_t *p = malloc(sizeof(uint16_t) * n);
    for (size_t i = 0; i < n; ++i) {
      float f = (float)(mean + std * normal());
      uint32_t b;
      memcpy(&b, &f, 4);
      p[i] = (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
    }
    return p;
  }
  float *p = malloc(sizeof(float) * n);
  for (size_t i = 0; i < n; ++i) p[i] = (float)(mean + std * normal());
  return p;
}

static int run(int bf16, double *checksum) {
  enum { NL = 3, D = 24, H = 4, HKV = 2, HD = 6, F = 40, V = 53, L0 = 19, N = 5, RANK = 3, DH = 17, DP = 11 };
  const int QD = H * HD, QKVD = QD + 2 * HKV * HD, CAP = L0 + N;
  orc_model mo = {NL, D, H, HKV, HD, F, V, bf16, 1e-5, 10000.0};
  const void *an[NL], *wqkv[NL], *wo[NL], *mn[NL], *wgu[NL], *wd[NL];
  const void *aq[NL - 1], *bq[NL - 1], *ao[NL - 1], *bo[NL - 1];
  for (int l = 0; l < NL; ++l) {
    an[l] = matrix(D, 1.0, 0.02, bf16); wqkv[l] = matrix((size_t)QKVD * D, 0, 0.2, bf16); wo[l] = matrix((size_t)D * QD, 0, 0.2, bf16);
    mn[l] = matrix(D, 1.0, 0.02, bf16); wgu[l] = matrix((size_t)2 * F * D, 0, 0.2, bf16); wd[l] = matrix((size_t)D * F, 0, 0.2, bf16);
  }
  for (int l = 0; l < NL - 1; ++l) {
    aq[l] = matrix((size_t)RANK * D, 0, 0.2, bf16); bq[l] = matrix((size_t)QKVD * RANK, 0, 0.2, bf16);
    ao[l] = matrix((size_t)RANK * QD, 0, 0.2, bf16); bo[l] = matrix((size_t)D * RANK, 0, 0.2, bf16);
  }
  orc_weights w = {matrix((size_t)V * D, 0, 1.0, bf16), matrix(D, 1.0, 0.02, bf16), matrix((size_t)V * D, 0, 0.3, bf16),
                   an, wqkv, wo, mn, wgu, wd};
  orc_lora lora = {RANK, 0.5, aq, bq, ao, bo};
  orc_draft_head head = {DH, DP, matrix((size_t)DH * D, 0, 0.3, bf16), matrix((size_t)DP * DH, 0, 0.3, bf16),
                         matrix((size_t)V * DP, 0, 0.5, bf16)};
  const size_t csz = (size_t)NL * CAP * HKV * HD;
  double *kc = malloc(sizeof(double) * csz), *vc = malloc(sizeof(double) * csz);
  double *logits = malloc(sizeof(double) * N * V), *hidden = malloc(sizeof(double) * N * D);
  int32_t tokens[N];
  double sum = 0.0;
  for (int mask = 0; mask < 64; mask += (mask < 8 ? 1 : 7)) {   /* every single point, several sets, all points */
    for (size_t i = 0; i < csz; ++i) { kc[i] = normal(); vc[i] = normal(); }
    for (int i = 0; i < N; ++i) tokens[i] = (int32_t)(unif() * V);
    if (orc_forward_lora(&mo, &w, (mask & 1) ? &lora : (const orc_lora *)0, kc, vc, CAP, L0, tokens, N, logits, hidden, mask)) return 1;
    for (int i = 0; i < N * V; ++i) sum += logits[i];
    if (orc_forward_lora(&mo, &w, &lora, kc, vc, CAP, L0, tokens, N, (double *)0, hidden, mask)) return 2;   /* no logits asked */
  }
  if (orc_forward(&mo, &w, kc, vc, CAP, L0, tokens, N, logits, hidden) || orc_forward_stored(&mo, &w, kc, vc, CAP, L0, tokens, N, logits, hidden, 63))
    return 3;
  if (orc_forward(&mo, &w, kc, vc, CAP, L0 + 1, tokens, N, logits, hidden) != -1) return 4;   /* one position too many: refused */
  {
    const size_t c1 = (size_t)CAP * HKV * HD;
    double *k1 = malloc(sizeof(double) * c1), *v1 = malloc(sizeof(double) * c1), *z = malloc(sizeof(double) * N * V);
    for (size_t i = 0; i < c1; ++i) { k1[i] = normal(); v1[i] = normal(); }
    if (orc_draft_forward(&mo, &w, &head, k1, v1, CAP, L0, tokens, N, z, 0) || orc_draft_forward(&mo, &w, &head, k1, v1, CAP, L0, tokens, N, z, 63))
      return 5;
    for (int i = 0; i < N * V; ++i) sum += z[i];
    free(k1); free(v1); free(z);
  }
  /* the accept / resample step on those logits: gamma = N - 1 drafts, every mode */
  {
    const int G = N - 1;
    float *q = malloc(sizeof(float) * G * V), u[N];
    int32_t d[N];
    for (int i = 0; i < G; ++i) {
      double s = 0.0;
      for (int x = 0; x < V; ++x) { q[i * V + x] = (float)exp(normal()); s += q[i * V + x]; }
      for (int x = 0; x < V; ++x) q[i * V + x] = (float)(q[i * V + x] / s);
      d[i] = (int32_t)(unif() * V);
      u[i] = (float)(floor(unif() * 16777216.0) / 16777216.0);
    }
    const double Ts[] = {0.0, 0.7, 1.0};
    const int ks[] = {0, 1, 7, V, V + 5};
    const double ps[] = {1.0, 0.9, 0.05, 1e-9};
    for (int ti = 0; ti < 3; ++ti)
      for (int ki = 0; ki < 5; ++ki)
        for (int pi = 0; pi < 4; ++pi)
          for (int g = 0; g <= G; ++g) {
            orc_sample_out o;
            double a[N];
            if (orc_sample_cut(logits, V, g, d, q, u, (float)(floor(unif() * 16777216.0) / 16777216.0), Ts[ti], ks[ki], ps[pi], &o, a))
              return 6;
            if (o.tau < 0 || o.tau > g || o.next_token < 0 || o.next_token >= V) return 7;
            int32_t nl, pr;
            if (orc_rollback(L0, g, o.tau, 16, &nl, &pr) || nl != L0 + 1 + o.tau) return 8;
            sum += o.tau + o.next_token;
          }
    orc_sample_out o;
    if (orc_sample(logits, V, G, d, q, u, 0.5f, 1.0, &o, (double *)0) || orc_sample_warp(logits, V, G, d, q, u, 0.5f, 1.0, 0.8, &o, (double *)0))
      return 9;
    free(q);
  }
  {
    double y[4], x[6] = {1, 2, 3, 4, 5, 6};
    float W[6] = {1, 0, -1, 0.5f, 0.25f, 2};
    orc_linear(W, 0, 2, 3, x, 2, y);
    if (y[0] != -2.0 || y[1] != 7.0 || y[2] != -2.0 || y[3] != 15.25) return 10;
    if (orc_round_bf16(1.00390625) != 1.0 || orc_round_bf16(1.01171875) != 1.015625) return 11;   /* ties to even, both ways */
  }
  for (int l = 0; l < NL; ++l) { free((void *)an[l]); free((void *)wqkv[l]); free((void *)wo[l]); free((void *)mn[l]); free((void *)wgu[l]); free((void *)wd[l]); }
  for (int l = 0; l < NL - 1; ++l) { free((void *)aq[l]); free((void *)bq[l]); free((void *)ao[l]); free((void *)bo[l]); }
  free((void *)w.embed); free((void *)w.final_norm); free((void *)w.lm_head);
  free((void *)head.w1); free((void *)head.w2); free((void *)head.wv);
  free(kc); free(vc); free(logits); free(hidden);
  *checksum = sum;
  return 0;
}

int main(void) {
  double c0 = 0, c1 = 0;
  int rc = run(0, &c0);
  if (rc) { printf("float weights: step %d failed\n", rc); return 1; }
  rc = run(1, &c1);
  if (rc) { printf("bf16 weights: step %d failed\n", rc); return 1; }
  if (!isfinite(c0) || !isfinite(c1)) { printf("non-finite checksum\n"); return 1; }
  printf("ok %.6e %.6e\n", c0, c1);
  return 0;
}
