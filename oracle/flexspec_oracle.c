/*
 * CPU oracle for the cloud-side verification step of FlexSpec
 * (Alg. 2 step 2 and the KV-session / rollback paragraph of Sec. IV-C).
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must
 * compute; it is slow on purpose, shares no code with the GPU path and must
 * never be called from it.  Everything floating point is fp64; weights are
 * widened exactly from their storage type (fp32 or bf16 bit patterns).
 *
 * What is written out here:
 *   - orc_forward : the target model M_t' scoring a block of new tokens on top
 *                   of a restored per-user KV cache (Alg. 2 "q <- M_t'(x_draft,
 *                   context)"; Sec. IV-C: KV pairs are computed only for the
 *                   newly received tokens).  Llama-style pre-norm decoder,
 *                   textbook definitions, no blocking or fusion.
 *   - orc_sample  : the acceptance loop of Alg. 2 (greedy: longest prefix with
 *                   draft == argmax) and, for temperature > 0, the speculative
 *                   sampling rule of the works the paper builds on (accept with
 *                   probability min(1, p/q), on rejection resample from the
 *                   normalised positive part of p - q, bonus token from p when
 *                   every draft is accepted), which keeps the output law equal
 *                   to the target model's (Sec. II, Regime B of Sec. V).  With
 *                   top_p < 1 and / or top_k > 0 the target law is first cut to its
 *                   most probable tokens (Regime B samples with top-p 0.9): the rule
 *                   then keeps the output law equal to the cut target law.
 *   - orc_rollback: the KV rollback of Sec. IV-C (positions from the first
 *                   rejected draft onward are discarded).
 *   - orc_forward_stored : the same forward with chosen intermediate tensors ROUNDED TO
 *                   bf16 where a bf16 deployment stores them between steps (the
 *                   configurations run the 1B / 8B targets "in bf16": weights, the KV
 *                   cache and the activations handed from one step to the next are
 *                   bf16 tensors).  All arithmetic stays fp64; only the named tensors
 *                   are rounded (round to nearest, ties to even).  With mask 0 it IS
 *                   orc_forward.  The difference between the two is the error that
 *                   bf16 storage alone causes, whatever computes the steps.
 *   - orc_forward_lora : the same forward for an EVOLVED target (Sec. IV-A: the target's parameters are the frozen
 *                   backbone plus PEFT adapters injected into the transformer layers; the head -- the last
 *                   transformer block and the LM head -- stays invariant).  The adapters are LoRA pairs on the
 *                   attention projections of every layer but the last: y = W x + s B (A x).  Without
 *                   adapters it IS orc_forward_stored.
 *   - orc_draft_forward : the edge draft model of Sec. IV-A, M_d(x) = H_small(B_shared(x)): a frozen copy of the
 *                   anchor block (the target's last transformer block) followed by a two-layer MLP and a
 *                   vocabulary projection.  The cloud holds all of it, so it can recompute the draft's law
 *                   for the tokens it receives instead of having it sent over the uplink.
 *
 * Parity pins for every function live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int weights_bf16; /* 1: weight arrays hold bf16 bit patterns (uint16_t), 0: float */
  double rms_eps, rope_theta;
} orc_model;

/* All matrices are [out_features][in_features], row-major. */
typedef struct {
  const void *embed;             /* [vocab][d_model]                          */
  const void *final_norm;        /* [d_model]                                 */
  const void *lm_head;           /* [vocab][d_model]                          */
  const void *const *attn_norm;  /* per layer [d_model]                       */
  const void *const *w_qkv;      /* per layer [(H+2*Hkv)*hd][d_model]: Wq|Wk|Wv */
  const void *const *w_o;        /* per layer [d_model][H*hd]                 */
  const void *const *mlp_norm;   /* per layer [d_model]                       */
  const void *const *w_gate_up;  /* per layer [2*d_ffn][d_model]: gate|up     */
  const void *const *w_down;     /* per layer [d_model][d_ffn]                */
} orc_weights;

static inline double widen(const void *w, int bf16, size_t idx) {
  if (bf16) {
    uint32_t bits = ((uint32_t)((const uint16_t *)w)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
  }
  return (double)((const float *)w)[idx];
}

/* Storage points of a bf16 deployment (orc_forward_stored): which tensors are rounded to bf16.  The two tensors that
 * are bounded whatever the model (a normalised activation is at most sqrt(d_model) times its gain, an attention output is a
 * convex combination of cached values) may instead be kept in fp16, which has the same 16 bits but 11 significant ones:
 * ORC_ST_A16 / ORC_ST_O16 round them to fp16; where both the bf16 and the fp16 bit of a tensor are set, bf16 wins. */
enum {
  ORC_ST_A = 1,    /* normalised activations entering the QKV, gate|up and LM-head projections */
  ORC_ST_Q = 2,    /* rotated queries                                                          */
  ORC_ST_KV = 4,   /* rotated keys and values of the new rows, as written to the KV cache       */
  ORC_ST_P = 8,    /* attention probabilities relative to the row maximum, exp(s - max)         */
  ORC_ST_O = 16,   /* attention output entering the O projection                                */
  ORC_ST_ACT = 32, /* SwiGLU output entering the down projection                                */
  ORC_ST_A16 = 64, /* the tensor of ORC_ST_A, rounded to fp16                                  */
  ORC_ST_O16 = 128 /* the tensor of ORC_ST_O, rounded to fp16                                  */
};

/* Nearest bf16 (8 significant bits, fp32 exponent range), ties to even, of a double; returned as a double. */
double orc_round_bf16(double x) {
  if (x == 0.0 || x != x || isinf(x)) return x;
  int e;
  (void)frexp(x, &e);                    /* x = m 2^e, 0.5 <= |m| < 1 */
  int qe = e - 8;                        /* quantum 2^(e-8): 8 significant bits */
  if (qe < -133) qe = -133;              /* subnormal range of the fp32 exponent: fixed quantum 2^-133 */
  double r = ldexp(nearbyint(ldexp(x, -qe)), qe);   /* default rounding mode: nearest, ties to even */
  if (fabs(r) >= ldexp(1.0, 128)) r = (x > 0) ? INFINITY : -INFINITY;
  return r;
}
static void round_rows(double *v, size_t n) {
  for (size_t i = 0; i < n; ++i) v[i] = orc_round_bf16(v[i]);
}

/* Nearest fp16 (11 significant bits, normal range from 2^-14, subnormal quantum 2^-24), ties to even, of a double;
 * a value that would round beyond the largest finite fp16 number is held at +-65504 (a saturating conversion). */
double orc_round_f16(double x) {
  if (x == 0.0 || x != x) return x;
  if (isinf(x)) return x > 0 ? 65504.0 : -65504.0;
  int e;
  (void)frexp(x, &e);                    /* x = m 2^e, 0.5 <= |m| < 1 */
  int qe = e - 11;                       /* quantum 2^(e-11): 11 significant bits */
  if (qe < -24) qe = -24;
  double r = ldexp(nearbyint(ldexp(x, -qe)), qe);
  if (r > 65504.0) r = 65504.0;
  if (r < -65504.0) r = -65504.0;
  return r;
}
static void round_rows_f16(double *v, size_t n) {
  for (size_t i = 0; i < n; ++i) v[i] = orc_round_f16(v[i]);
}
/* one storage point: its bf16 bit, else its fp16 bit, else left alone */
static void store_point(double *v, size_t n, int stored, int bit_bf16, int bit_f16) {
  if (stored & bit_bf16) round_rows(v, n);
  else if (stored & bit_f16) round_rows_f16(v, n);
}

/* Dense projection, the definition: y[m][o] = sum_k x[m][k] * W[o][k]   (x: [n][in], y: [n][out]) */
void orc_linear(const void *W, int bf16, int out, int in, const double *x, int n, double *y) {
#pragma omp parallel for schedule(static)
  for (int o = 0; o < out; ++o) {
    for (int m = 0; m < n; ++m) {
      double acc = 0.0;
      for (int k = 0; k < in; ++k) acc += x[(size_t)m * in + k] * widen(W, bf16, (size_t)o * in + k);
      y[(size_t)m * out + o] = acc;
    }
  }
}

/* RMSNorm: y = x * g / sqrt(mean(x^2) + eps) */
static void rmsnorm(const double *x, const void *g, int bf16, int d, double eps, int n, double *y) {
  for (int m = 0; m < n; ++m) {
    double ss = 0.0;
    for (int k = 0; k < d; ++k) ss += x[(size_t)m * d + k] * x[(size_t)m * d + k];
    double r = 1.0 / sqrt(ss / d + eps);
    for (int k = 0; k < d; ++k) y[(size_t)m * d + k] = x[(size_t)m * d + k] * r * widen(g, bf16, k);
  }
}

/* Rotary embedding, half-split pairing (i, i + hd/2), angle = pos * theta^(-2i/hd). */
static void rope(double *vec, int hd, int pos, double theta) {
  int half = hd / 2;
  for (int i = 0; i < half; ++i) {
    double ang = (double)pos * pow(theta, -2.0 * i / hd);
    double c = cos(ang), s = sin(ang);
    double a = vec[i], b = vec[i + half];
    vec[i] = a * c - b * s;
    vec[i + half] = a * s + b * c;
  }
}

/*
 * Attention of a block of n queries over one session's cache (one layer), the definition:
 * query i (rotated, at position L+i) attends to keys 0 .. L+i, i.e. the restored context plus the
 * block up to itself (causal only inside the block); query head hh reads KV head hh / (H/Hkv).
 *   q   : [n][q_stride] with head hh at q[i*q_stride + hh*hd]
 *   kl,vl: [>= L+n][Hkv*hd] keys / values of this layer
 *   out : [n][H*hd]
 */
static void attention_impl(const double *q, int q_stride, const double *kl, const double *vl, int L, int n, int H,
                           int Hkv, int hd, double *out, int round_p) {
  const int kvdim = Hkv * hd, group = H / Hkv;
  double *sc = malloc(sizeof(double) * (L + n));
  for (int i = 0; i < n; ++i) {
    int nkeys = L + i + 1;
    for (int hh = 0; hh < H; ++hh) {
      const double *qv = q + (size_t)i * q_stride + hh * hd;
      int kvh = hh / group;
      double mx = -INFINITY;
      for (int j = 0; j < nkeys; ++j) {
        const double *kv = kl + (size_t)j * kvdim + kvh * hd;
        double s = 0.0;
        for (int e = 0; e < hd; ++e) s += qv[e] * kv[e];
        sc[j] = s / sqrt((double)hd);
        if (sc[j] > mx) mx = sc[j];
      }
      double den = 0.0;
      for (int j = 0; j < nkeys; ++j) { sc[j] = exp(sc[j] - mx); den += sc[j]; }
      double *o = out + (size_t)i * H * hd + hh * hd;
      for (int e = 0; e < hd; ++e) o[e] = 0.0;
      for (int j = 0; j < nkeys; ++j) {
        const double *vv = vl + (size_t)j * kvdim + kvh * hd;
        /* ORC_ST_P: the numerator uses the stored (rounded) exp(s - max), the normaliser the exact sum */
        double p = (round_p ? orc_round_bf16(sc[j]) : sc[j]) / den;
        for (int e = 0; e < hd; ++e) o[e] += p * vv[e];
      }
    }
  }
  free(sc);
}

void orc_attention(const double *q, int q_stride, const double *kl, const double *vl, int L, int n, int H, int Hkv,
                   int hd, double *out) {
  attention_impl(q, q_stride, kl, vl, L, n, H, Hkv, hd, out, 0);
}

/*
 * Score n new tokens that sit at positions L .. L+n-1 of one user's session.
 *   kc, vc : the session's KV cache, [n_layers][cap][n_kv_heads][head_dim] doubles;
 *            positions < L hold the restored context, positions L..L+n-1 are
 *            written here (the KV pairs of the newly received tokens).
 *   logits : [n][vocab], row i = target logits for the token FOLLOWING tokens[i].
 *   hidden : optional [n][d_model], final residual stream before the last norm.
 * Query i attends to keys 0 .. L+i (context plus the block up to itself).
 * Returns 0, or -1 on bad arguments / out of memory.
 */
/*
 * One request's LoRA adapter (Sec. IV-A, PEFT parameterisation of the evolving target): for every layer l but the last,
 * low-rank pairs on the fused q|k|v projection and on the output projection,
 *   qkv = W_qkv a + scale * B_qkv (A_qkv a),    o_proj = W_o att + scale * B_o (A_o att).
 * Matrices are [out][in] row-major in the model's weight storage type: A_qkv [rank][d_model], B_qkv [(H+2Hkv)hd][rank],
 * A_o [rank][H hd], B_o [d_model][rank]; the arrays hold n_layers - 1 pointers each.  The low-rank product is never
 * rounded (it is not a stored tensor); its input is the same (possibly stored) activation the main projection reads.
 */
typedef struct {
  int rank;
  double scale;
  const void *const *a_qkv, *const *b_qkv, *const *a_o, *const *b_o;
} orc_lora;

/* y[m][:] += scale * B (A x[m][:]) */
static void lora_add(const void *A, const void *B, int bf16, int out, int in, int rank, double scale, const double *x, int n,
                     double *y) {
  double *t = malloc(sizeof(double) * n * rank), *u = malloc(sizeof(double) * n * out);
  orc_linear(A, bf16, rank, in, x, n, t);
  orc_linear(B, bf16, out, rank, t, n, u);
  for (size_t i = 0; i < (size_t)n * out; ++i) y[i] += scale * u[i];
  free(t); free(u);
}

int orc_forward_lora(const orc_model *mo, const orc_weights *w, const orc_lora *lora, double *kc, double *vc, int cap, int L,
                     const int32_t *tokens, int n, double *logits, double *hidden, int stored) {
  const int d = mo->d_model, H = mo->n_heads, Hkv = mo->n_kv_heads, hd = mo->head_dim;
  const int F = mo->d_ffn, V = mo->vocab, bf = mo->weights_bf16;
  if (n <= 0 || L < 0 || L + n > cap || H % Hkv != 0 || hd % 2 != 0) return -1;
  for (int i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= V) return -1;
  const int qdim = H * hd, kvdim = Hkv * hd, qkvdim = qdim + 2 * kvdim;
  double *h = malloc(sizeof(double) * n * d), *a = malloc(sizeof(double) * n * d);
  double *qkv = malloc(sizeof(double) * n * qkvdim), *att = malloc(sizeof(double) * n * qdim);
  double *gu = malloc(sizeof(double) * n * 2 * F), *act = malloc(sizeof(double) * n * F);
  double *upd = malloc(sizeof(double) * n * d);
  if (!h || !a || !qkv || !att || !gu || !act || !upd) return -1;

  for (int i = 0; i < n; ++i)
    for (int k = 0; k < d; ++k) h[(size_t)i * d + k] = widen(w->embed, bf, (size_t)tokens[i] * d + k);

  for (int l = 0; l < mo->n_layers; ++l) {
    double *kl = kc + (size_t)l * cap * kvdim, *vl = vc + (size_t)l * cap * kvdim;
    rmsnorm(h, w->attn_norm[l], bf, d, mo->rms_eps, n, a);
    store_point(a, (size_t)n * d, stored, ORC_ST_A, ORC_ST_A16);
    orc_linear(w->w_qkv[l], bf, qkvdim, d, a, n, qkv);
    const int adapted = lora && lora->rank > 0 && l < mo->n_layers - 1;   /* the last block is part of the invariant head */
    if (adapted) lora_add(lora->a_qkv[l], lora->b_qkv[l], bf, qkvdim, d, lora->rank, lora->scale, a, n, qkv);
    for (int i = 0; i < n; ++i) {
      double *row = qkv + (size_t)i * qkvdim;
      int pos = L + i;
      for (int hh = 0; hh < H; ++hh) rope(row + hh * hd, hd, pos, mo->rope_theta);
      for (int hh = 0; hh < Hkv; ++hh) rope(row + qdim + hh * hd, hd, pos, mo->rope_theta);
      if (stored & ORC_ST_Q) round_rows(row, qdim);
      if (stored & ORC_ST_KV) round_rows(row + qdim, 2 * (size_t)kvdim);
      memcpy(kl + (size_t)pos * kvdim, row + qdim, sizeof(double) * kvdim);
      memcpy(vl + (size_t)pos * kvdim, row + qdim + kvdim, sizeof(double) * kvdim);
    }
    attention_impl(qkv, qkvdim, kl, vl, L, n, H, Hkv, hd, att, stored & ORC_ST_P);
    store_point(att, (size_t)n * qdim, stored, ORC_ST_O, ORC_ST_O16);
    orc_linear(w->w_o[l], bf, d, qdim, att, n, upd);
    if (adapted) lora_add(lora->a_o[l], lora->b_o[l], bf, d, qdim, lora->rank, lora->scale, att, n, upd);
    for (size_t t = 0; t < (size_t)n * d; ++t) h[t] += upd[t];
    rmsnorm(h, w->mlp_norm[l], bf, d, mo->rms_eps, n, a);
    store_point(a, (size_t)n * d, stored, ORC_ST_A, ORC_ST_A16);
    orc_linear(w->w_gate_up[l], bf, 2 * F, d, a, n, gu);
    for (int i = 0; i < n; ++i)
      for (int f = 0; f < F; ++f) {
        double g = gu[(size_t)i * 2 * F + f], u = gu[(size_t)i * 2 * F + F + f];
        act[(size_t)i * F + f] = g / (1.0 + exp(-g)) * u; /* silu(g) * u */
      }
    if (stored & ORC_ST_ACT) round_rows(act, (size_t)n * F);
    orc_linear(w->w_down[l], bf, d, F, act, n, upd);
    for (size_t t = 0; t < (size_t)n * d; ++t) h[t] += upd[t];
  }
  if (hidden) memcpy(hidden, h, sizeof(double) * n * d);
  if (logits) {
    rmsnorm(h, w->final_norm, bf, d, mo->rms_eps, n, a);
    store_point(a, (size_t)n * d, stored, ORC_ST_A, ORC_ST_A16);
    orc_linear(w->lm_head, bf, V, d, a, n, logits);
  }
  free(h); free(a); free(qkv); free(att); free(gu); free(act); free(upd);
  return 0;
}

int orc_forward_stored(const orc_model *mo, const orc_weights *w, double *kc, double *vc, int cap, int L,
                       const int32_t *tokens, int n, double *logits, double *hidden, int stored) {
  return orc_forward_lora(mo, w, (const orc_lora *)0, kc, vc, cap, L, tokens, n, logits, hidden, stored);
}

int orc_forward(const orc_model *mo, const orc_weights *w, double *kc, double *vc, int cap, int L,
                const int32_t *tokens, int n, double *logits, double *hidden) {
  return orc_forward_lora(mo, w, (const orc_lora *)0, kc, vc, cap, L, tokens, n, logits, hidden, 0);
}

/*
 * The draft model of Sec. IV-A (structural definition): M_d(x) = H_small(B_shared(x)).
 *   B_shared : a frozen copy of the anchor block, i.e. the LAST transformer block of the base target (weights taken from
 *              layer n_layers - 1 of `w`), applied to the embeddings of the tokens (the base model's embedding table)
 *              with a KV session of its own (kc, vc: ONE layer, [cap][n_kv_heads][head_dim]);
 *   H_small  : a two-layer MLP followed by a vocabulary projection, on the block's output h (the residual stream):
 *              z = W_v ( W_2 silu( W_1 h ) ),  W_1 [d_hidden][d_model], W_2 [d_proj][d_hidden], W_v [vocab][d_proj].
 * logits: [n][vocab], row i = the draft's logits for the token following tokens[i]; its law is softmax(z / T).
 * With `stored` != 0 the block rounds its storage points as the target forward does, and the three inputs of the head's
 * projections (h, the activation, the second layer's output) are rounded to bf16 as well.
 */
typedef struct {
  int d_hidden, d_proj;
  const void *w1, *w2, *wv;   /* weight storage type of the model */
} orc_draft_head;

int orc_draft_forward(const orc_model *mo, const orc_weights *w, const orc_draft_head *head, double *kc, double *vc, int cap,
                      int L, const int32_t *tokens, int n, double *logits, int stored) {
  if (mo->n_layers < 1 || !head || head->d_hidden <= 0 || head->d_proj <= 0) return -1;
  const int last = mo->n_layers - 1, d = mo->d_model, bf = mo->weights_bf16, dh = head->d_hidden, dp = head->d_proj;
  orc_model m1 = *mo;
  m1.n_layers = 1;
  orc_weights w1 = *w;   /* the one-layer model whose only block is the anchor block */
  const void *an = w->attn_norm[last], *qkv = w->w_qkv[last], *wo = w->w_o[last], *mn = w->mlp_norm[last],
             *gu = w->w_gate_up[last], *dn = w->w_down[last];
  w1.attn_norm = &an; w1.w_qkv = &qkv; w1.w_o = &wo; w1.mlp_norm = &mn; w1.w_gate_up = &gu; w1.w_down = &dn;
  double *h = malloc(sizeof(double) * n * d), *t1 = malloc(sizeof(double) * n * dh), *t2 = malloc(sizeof(double) * n * dp);
  if (!h || !t1 || !t2) return -1;
  int rc = orc_forward_lora(&m1, &w1, (const orc_lora *)0, kc, vc, cap, L, tokens, n, (double *)0, h, stored);
  if (rc == 0) {
    if (stored) round_rows(h, (size_t)n * d);
    orc_linear(head->w1, bf, dh, d, h, n, t1);
    for (size_t i = 0; i < (size_t)n * dh; ++i) t1[i] = t1[i] / (1.0 + exp(-t1[i]));   /* silu */
    if (stored) round_rows(t1, (size_t)n * dh);
    orc_linear(head->w2, bf, dp, dh, t1, n, t2);
    if (stored) round_rows(t2, (size_t)n * dp);
    orc_linear(head->wv, bf, mo->vocab, dp, t2, n, logits);
  }
  free(h); free(t1); free(t2);
  return rc;
}

typedef struct {
  int32_t tau;          /* accepted drafts, 0..gamma                                        */
  int32_t next_token;   /* correction token (tau < gamma) or bonus token (tau == gamma)     */
  int32_t used_residual;/* 1 if next_token was drawn from the residual distribution         */
  int32_t pad_;
  double accept_margin; /* min over tested drafts of |u_i - min(1, p/q)|; +inf if none      */
  double cdf_margin;    /* distance of u_sample from the chosen token's CDF edges (normalised) */
  double nucleus_margin;/* min over the rows used of the distance of top_p from the cumulative masses at the cut */
} orc_sample_out;

static void softmax_row(const double *lg, int V, double T, double *p) {
  double mx = -INFINITY, den = 0.0;
  for (int x = 0; x < V; ++x) if (lg[x] / T > mx) mx = lg[x] / T;
  for (int x = 0; x < V; ++x) { p[x] = exp(lg[x] / T - mx); den += p[x]; }
  for (int x = 0; x < V; ++x) p[x] /= den;
}

/*
 * Cut of a probability row to its most probable tokens, as Regime B of Sec. V samples (top-p 0.9; top-k is the other
 * common form of the same cut).  Order the tokens by probability.
 *   top_k > 0 : keep the top_k most probable tokens and every token tied with the last of them; renormalise.
 *   top_p < 1 : of what is left, keep the most probable tokens up to and including the one with which the kept mass
 *               first reaches top_p (of the renormalised row), and every token tied with that last one; renormalise.
 * Ties are always kept together, so the set never depends on an order among equal probabilities.  top_k <= 0 or >= V
 * and top_p >= 1 keep the row.  *margin (may be NULL) gets, for the top-p step, min(top_p - mass strictly above the
 * last kept value, mass at or above it - top_p) in units of the row the step works on.
 */
typedef struct { double p; int x; } orc_px;
static int px_desc(const void *a, const void *b) {
  const orc_px *u = a, *v = b;
  if (u->p != v->p) return (u->p < v->p) ? 1 : -1;
  return (u->x > v->x) - (u->x < v->x);
}
static int cut_row(double *p, int V, int top_k, double top_p, double *margin) {
  if (margin) *margin = INFINITY;
  const int use_k = top_k > 0 && top_k < V, use_p = top_p < 1.0;
  if (!use_k && !use_p) return 0;
  orc_px *s = malloc(sizeof(orc_px) * V);
  if (!s) return -1;
  if (use_k) {
    for (int x = 0; x < V; ++x) { s[x].p = p[x]; s[x].x = x; }
    qsort(s, V, sizeof(orc_px), px_desc);
    const double cut = s[top_k - 1].p;
    double ge = 0.0;
    for (int x = 0; x < V; ++x) if (p[x] >= cut) ge += p[x];
    for (int x = 0; x < V; ++x) p[x] = (p[x] >= cut) ? p[x] / ge : 0.0;
  }
  if (use_p) {
    for (int x = 0; x < V; ++x) { s[x].p = p[x]; s[x].x = x; }
    qsort(s, V, sizeof(orc_px), px_desc);
    double cum = 0.0;
    int k = V - 1;
    for (int i = 0; i < V; ++i) { cum += s[i].p; if (cum >= top_p) { k = i; break; } }
    const double cut = s[k].p;
    double gt = 0.0, ge = 0.0;
    for (int i = 0; i < V; ++i) { if (s[i].p > cut) gt += s[i].p; if (s[i].p >= cut) ge += s[i].p; }
    if (margin) { double a = top_p - gt, b = ge - top_p; *margin = (a < b) ? a : b; }
    for (int x = 0; x < V; ++x) p[x] = (p[x] >= cut) ? p[x] / ge : 0.0;
  }
  free(s);
  return 0;
}

static int argmax_row(const double *lg, int V) { /* lowest index wins ties */
  int best = 0;
  for (int x = 1; x < V; ++x) if (lg[x] > lg[best]) best = x;
  return best;
}

/* Smallest x whose inclusive running sum of mass exceeds u * total; the last
 * index with positive mass if rounding leaves none. */
static int inverse_cdf(const double *mass, int V, double u, double *margin) {
  double total = 0.0;
  for (int x = 0; x < V; ++x) total += mass[x];
  double target = u * total, run = 0.0;
  int pick = -1, last_pos = 0;
  double lo = 0.0, hi = 0.0;
  for (int x = 0; x < V; ++x) {
    if (mass[x] > 0.0) last_pos = x;
    double prev = run;
    run += mass[x];
    if (pick < 0 && run > target) { pick = x; lo = prev; hi = run; }
  }
  if (pick < 0) { pick = last_pos; lo = hi = total; }
  if (margin) {
    double a = fabs(target - lo), b = fabs(hi - target);
    *margin = (a < b ? a : b) / total;
  }
  return pick;
}

/*
 * Accept / reject one request's drafts and emit the next token.
 *   logits : [gamma+1][V] target logits; row i scores the token after input row i
 *            (row 0 = after last_token, row i = after draft i).
 *   q      : [gamma][V] draft probabilities, q[i-1] is the law draft i was drawn from
 *            (ignored when T == 0).
 *   u_acc  : [gamma] uniforms in [0,1); u_smp: one uniform for the emitted token.
 *   a_out  : optional [gamma], acceptance probabilities of the drafts that were tested.
 * T == 0 is greedy decoding (Alg. 2): accept while draft == argmax, emit argmax.
 */
int orc_sample_cut(const double *logits, int V, int gamma, const int32_t *draft, const float *q,
                   const float *u_acc, float u_smp, double T, int top_k, double top_p, orc_sample_out *out,
                   double *a_out) {
  if (V <= 0 || gamma < 0 || T < 0.0 || !(top_p > 0.0) || top_k < 0) return -1;
  out->tau = 0; out->used_residual = 0; out->accept_margin = INFINITY; out->cdf_margin = INFINITY;
  out->nucleus_margin = INFINITY;
  double nm;
  if (T == 0.0) {
    int tau = 0;
    while (tau < gamma && draft[tau] == argmax_row(logits + (size_t)tau * V, V)) ++tau;
    out->tau = tau;
    out->next_token = argmax_row(logits + (size_t)tau * V, V);
    return 0;
  }
  double *p = malloc(sizeof(double) * V), *r = malloc(sizeof(double) * V);
  if (!p || !r) return -1;
  int tau = 0;
  for (int i = 1; i <= gamma; ++i) {
    int dtok = draft[i - 1];
    if (dtok < 0 || dtok >= V) { free(p); free(r); return -1; }
    softmax_row(logits + (size_t)(i - 1) * V, V, T, p);
    if (cut_row(p, V, top_k, top_p, &nm)) { free(p); free(r); return -1; }
    if (nm < out->nucleus_margin) out->nucleus_margin = nm;
    double qd = (double)q[(size_t)(i - 1) * V + dtok];
    double ratio = p[dtok] / qd;              /* qd == 0 gives +inf (or NaN for 0/0) */
    double a = (ratio >= 1.0) ? 1.0 : ratio;
    if (!(a == a)) a = 0.0;                   /* p = q = 0: a token the draft cannot have produced */
    if (a_out) a_out[i - 1] = a;
    double mg = fabs((double)u_acc[i - 1] - a);
    if (mg < out->accept_margin) out->accept_margin = mg;
    if ((double)u_acc[i - 1] < a) ++tau; else break;
  }
  out->tau = tau;
  softmax_row(logits + (size_t)tau * V, V, T, p);
  if (cut_row(p, V, top_k, top_p, &nm)) { free(p); free(r); return -1; }
  if (nm < out->nucleus_margin) out->nucleus_margin = nm;
  if (tau < gamma) {
    double Z = 0.0;
    for (int x = 0; x < V; ++x) {
      double dlt = p[x] - (double)q[(size_t)tau * V + x];
      r[x] = dlt > 0.0 ? dlt : 0.0;
      Z += r[x];
    }
    if (Z > 0.0) {
      out->used_residual = 1;
      out->next_token = inverse_cdf(r, V, (double)u_smp, &out->cdf_margin);
      free(p); free(r);
      return 0;
    }
  }
  out->next_token = inverse_cdf(p, V, (double)u_smp, &out->cdf_margin);
  free(p); free(r);
  return 0;
}

int orc_sample_warp(const double *logits, int V, int gamma, const int32_t *draft, const float *q,
                    const float *u_acc, float u_smp, double T, double top_p, orc_sample_out *out, double *a_out) {
  return orc_sample_cut(logits, V, gamma, draft, q, u_acc, u_smp, T, 0, top_p, out, a_out);
}

int orc_sample(const double *logits, int V, int gamma, const int32_t *draft, const float *q,
               const float *u_acc, float u_smp, double T, orc_sample_out *out, double *a_out) {
  return orc_sample_cut(logits, V, gamma, draft, q, u_acc, u_smp, T, 0, 1.0, out, a_out);
}

/*
 * KV rollback: after tau of gamma drafts were accepted on top of L cached
 * positions, positions [0, L+1+tau) stay valid (context, the pending token and
 * the accepted drafts); everything from the first rejected draft onward is
 * discarded.  pages_released counts the pages (page_size positions each) that
 * covered the appended block but hold no valid position any more.
 */
int orc_rollback(int L, int gamma, int tau, int page_size, int32_t *new_len, int32_t *pages_released) {
  if (L < 0 || gamma < 0 || tau < 0 || tau > gamma || page_size <= 0) return -1;
  int keep = L + 1 + tau, written = L + 1 + gamma;
  *new_len = keep;
  *pages_released = (written + page_size - 1) / page_size - (keep + page_size - 1) / page_size;
  return 0;
}
