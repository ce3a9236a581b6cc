/*
 * Exhaustive driver for the oracle's sampler (test helper, CPU only).
 *
 * For a table-defined target law p(. | prefix) and draft law q(. | prefix) over a tiny
 * vocabulary it enumerates every draft sequence (weighted by the draft chain), a midpoint
 * grid over every uniform the step consumes, runs orc_sample on each combination and
 * accumulates the probability mass of every emitted token sequence.  The Python test then
 * checks that each emitted token, given the tokens emitted before it, follows p.
 *
 * Tables are indexed by prefix code: prefix (t1..tn) -> sum_{k<=n} V^(k-1) + base-V value,
 * i.e. level offsets 0, 1, 1+V, 1+V+V^2 ...; every row holds V entries.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct {
  int32_t tau, next_token, used_residual, pad_;
  double accept_margin, cdf_margin, nucleus_margin;
} orc_sample_out;
int orc_sample_cut(const double *logits, int V, int gamma, const int32_t *draft, const float *q,
                   const float *u_acc, float u_smp, double T, int top_k, double top_p, orc_sample_out *out, double *a_out);

static int level_offset(int V, int n) { int off = 0, p = 1; for (int k = 0; k < n; ++k) { off += p; p *= V; } return off; }

static int prefix_code(int V, const int32_t *t, int n) {
  int v = 0;
  for (int k = 0; k < n; ++k) v = v * V + t[k];
  return level_offset(V, n) + v;
}

/* hist is indexed by the code of the emitted sequence (length 1..gamma+1). */
int brute_force_cut(int V, int gamma, int N, double T, int top_k, double top_p, const double *target_logits,
                    const float *q_table, double *hist);
int brute_force(int V, int gamma, int N, double T, const double *target_logits, const float *q_table, double *hist) {
  return brute_force_cut(V, gamma, N, T, 0, 1.0, target_logits, q_table, hist);
}
int brute_force_warp(int V, int gamma, int N, double T, double top_p, const double *target_logits, const float *q_table,
                     double *hist) {
  return brute_force_cut(V, gamma, N, T, 0, top_p, target_logits, q_table, hist);
}

int brute_force_cut(int V, int gamma, int N, double T, int top_k, double top_p, const double *target_logits,
                    const float *q_table, double *hist) {
  int nseq = 1;
  for (int k = 0; k < gamma; ++k) nseq *= V;
  double *logits = malloc(sizeof(double) * (gamma + 1) * V);
  float *q = malloc(sizeof(float) * (gamma > 0 ? gamma : 1) * V);
  int32_t d[8], emit[9];
  float u[8];
  if (gamma > 8) return -1;
  long ngrid = 1;
  for (int k = 0; k < gamma; ++k) ngrid *= N;
  for (int s = 0; s < nseq; ++s) {
    int v = s;
    for (int k = gamma - 1; k >= 0; --k) { d[k] = v % V; v /= V; }
    double wseq = 1.0;
    for (int i = 0; i <= gamma; ++i) {
      int code = prefix_code(V, d, i);
      for (int x = 0; x < V; ++x) logits[i * V + x] = target_logits[code * V + x];
      if (i < gamma) {
        for (int x = 0; x < V; ++x) q[i * V + x] = q_table[code * V + x];
        wseq *= (double)q_table[code * V + d[i]];
      }
    }
    if (wseq == 0.0) continue;
    for (long g = 0; g < ngrid; ++g) {
      long gg = g;
      for (int k = 0; k < gamma; ++k) { u[k] = (float)(((gg % N) + 0.5) / N); gg /= N; }
      for (int ks = 0; ks < N; ++ks) {
        orc_sample_out out;
        if (orc_sample_cut(logits, V, gamma, d, q, u, (float)((ks + 0.5) / N), T, top_k, top_p, &out, 0) != 0) return -2;
        for (int k = 0; k < out.tau; ++k) emit[k] = d[k];
        emit[out.tau] = out.next_token;
        hist[prefix_code(V, emit, out.tau + 1)] += wseq / ((double)ngrid * N);
      }
    }
  }
  free(logits); free(q);
  return 0;
}
