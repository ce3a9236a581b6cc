/*
 * flexverify — the cloud-side verification step of FlexSpec (Alg. 2 step 2, Sec. IV-C)
 * for one AMD MI355X (gfx950).
 *
 * One call of fsv_verify() does, for a whole batch of edge requests, what Alg. 2 does
 * between "receive x_draft and restore KV cache" and "transmit x_verified": the target
 * model scores the pending token and the gamma_b received draft tokens of every request in
 * one pass on top of that user's persistent KV session (Sec. IV-C: KV pairs are computed
 * only for the newly received tokens), the drafts are accepted or rejected, the correction
 * (or bonus) token is chosen, and the KV pairs of rejected positions are rolled back.
 *
 * Conventions
 *   - Plain C ABI.  Every pointer is marked HOST or DEVICE.  Device memory is owned by the
 *     caller unless stated otherwise; the library owns only what fsv_create() allocates
 *     (re-tiled weights and a workspace sized from fsv_model_desc).
 *   - Calls that take a stream enqueue their work on that HIP stream (hipStream_t passed as
 *     void*, NULL = the null stream) and return without waiting for the GPU; results are
 *     valid once the stream has been synchronised.  No call reads device memory back to the
 *     host; where the host needs values to size launches it takes HOST copies from the caller.
 *   - Every function that can fail returns 0 (FSV_OK) or a negative fsv_status.  On failure
 *     nothing has been launched.  No exceptions cross the boundary.
 *   - Random numbers are inputs (uniforms in [0,1)), never drawn inside the library.
 *   - A context is not thread safe: calls on one context must not overlap (they share its
 *     workspace), neither on the host nor on different streams.
 */
#ifndef FLEXVERIFY_H
#define FLEXVERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fsv_ctx fsv_ctx;

typedef enum { FSV_F32 = 0, FSV_BF16 = 1 } fsv_dtype;

typedef enum {
  FSV_OK = 0,
  FSV_E_INVALID_ARG = -1, /* NULL pointer, negative size, inconsistent CSR ... (token and page ids
                             live on the device and are clamped into range there, not reported)        */
  FSV_E_CAPACITY = -2,    /* batch, gamma, pages or rows beyond what the context was created for        */
  FSV_E_UNSUPPORTED = -3, /* shape the kernels do not cover (see fsv_create)                            */
  FSV_E_HIP = -4,         /* a HIP runtime call failed (allocation, launch)                             */
  FSV_E_NO_MODEL = -5     /* a model call on a sampler-only context                                     */
} fsv_status;

/*
 * Target model M_t' (Llama-style pre-norm decoder: RMSNorm, rotary embedding with half-split
 * pairing (i, i + head_dim/2), grouped-query attention, SwiGLU MLP, untied LM head, no biases)
 * and the capacity of the context.
 */
typedef struct {
  int32_t n_layers;          /* 0 = sampler-only context (fsv_sample / fsv_rollback only)            */
  int32_t d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t dtype;             /* fsv_dtype of weights, activations and KV cache                        */
  float rms_eps, rope_theta;
  int32_t page_size;         /* positions per KV page; must be 16                                     */
  int32_t max_batch;         /* requests per call                                                     */
  int32_t max_gamma;         /* drafts per request, <= 16                                             */
  int32_t max_pages_per_req; /* columns of the page table                                             */
  int32_t max_rows;          /* sum over requests of (gamma_b + 1); 0 = max_batch * (max_gamma + 1)   */
} fsv_model_desc;

/*
 * Weights.  DEVICE pointers to row-major [out_features][in_features] matrices of the model's
 * dtype; the per-layer members are HOST arrays of n_layers DEVICE pointers.  fsv_create() reads
 * them once (it copies fp32 weights and re-tiles bf16 matrices into the operand order of the
 * matrix cores); the caller may free all of them when fsv_create() has returned.
 * FSV_BF16: the four projections whose input is bounded whatever the model (q|k|v, gate|up and the LM head
 * take a normalised activation, the output projection a convex combination of cached values) run on fp16
 * operands, which have three more significant bits than bf16 at the same size and rate; their matrices are
 * converted once, times a power of two per matrix that puts its largest weight near 2^13, so that every
 * weight down to 2^-31 of the largest converts exactly (smaller ones round on the fp16 subnormal grid of the
 * scaled matrix), and the fp32 sums are multiplied by the inverse power.  The down projection (its input,
 * the SwiGLU output, has no bound) and the KV cache stay bf16.  The conversion of the two fp16 tensors
 * saturates: a normalised activation or an attention output beyond +-65504 (gains in the thousands, or cached
 * values of that size) is held there instead of becoming an infinity; NaN stays NaN.
 */
typedef struct {
  const void *embed;             /* [vocab][d_model]                                          */
  const void *final_norm;        /* [d_model]                                                 */
  const void *lm_head;           /* [vocab][d_model]                                          */
  const void *const *attn_norm;  /* [d_model]                                                 */
  const void *const *w_qkv;      /* [(n_heads + 2 n_kv_heads) head_dim][d_model]: Wq | Wk | Wv */
  const void *const *w_o;        /* [d_model][n_heads head_dim]                               */
  const void *const *mlp_norm;   /* [d_model]                                                 */
  const void *const *w_gate_up;  /* [2 d_ffn][d_model]: gate | up                             */
  const void *const *w_down;     /* [d_model][d_ffn]                                          */
} fsv_weights;

/*
 * One batch of requests.  B = batch, G = total drafts, M = G + B rows.  Request b has
 * gamma_b = draft_offsets[b+1] - draft_offsets[b] drafts; its input rows are the pending token
 * last_token[b] at position seq_lens[b] followed by its drafts at the next positions.
 *
 * KV pools: k_pool and v_pool each hold n_layers * num_pages * n_kv_heads page tiles of
 * page_size * head_dim elements, indexed [layer][physical page][kv head].  Inside a tile
 *   FSV_F32 : [position in page][head_dim] for both pools;
 *   FSV_BF16: the order in which the matrix cores consume it, see fsv_kv_import().
 * Use fsv_kv_import()/fsv_kv_export() to move sessions in and out; do not index tiles directly.
 * Slots that hold no valid position (never written, or left behind by a rollback) may hold any bit pattern,
 * NaN and Inf included: they are masked out of the softmax and cleared before they reach the matrix cores.
 * The call appends the KV pairs of all M rows (positions seq_lens[b] .. seq_lens[b]+gamma_b).
 */
typedef struct {
  int32_t batch;
  int32_t num_pages;                 /* physical pages per layer in each pool                         */
  const int32_t *seq_lens;           /* DEVICE [B]   L_b, cached positions before the call            */
  const int32_t *seq_lens_host;      /* HOST   [B]   same values                                      */
  const int32_t *last_token;         /* DEVICE [B]                                                    */
  const int32_t *draft_offsets;      /* DEVICE [B+1] CSR over drafts                                  */
  const int32_t *draft_offsets_host; /* HOST   [B+1] same values                                      */
  const int32_t *draft_tokens;       /* DEVICE [G]                                                    */
  const float *draft_probs;          /* DEVICE [G][vocab] q_{b,i}(.), the law draft i was drawn from;
                                        may be NULL when every temperature is 0                       */
  const float *u_accept;             /* DEVICE [G]   uniforms in [0,1) for the acceptance tests       */
  const float *u_sample;             /* DEVICE [B]   uniform for the correction / bonus token         */
  const float *temperature;          /* DEVICE [B]   T_b > 0: speculative sampling on softmax(l/T_b);
                                                     T_b = 0: greedy (argmax match, Alg. 2)          */
  const float *temperature_host;     /* HOST   [B]   same values (NULL = all positive)                */
  const int32_t *page_table;         /* DEVICE [B][max_pages_per_req] physical page of each logical
                                        page; must cover positions < seq_lens[b] + gamma_b + 1        */
  void *k_pool, *v_pool;             /* DEVICE, read and written                                      */
  const float *top_p;                /* DEVICE [B]   nucleus mass in (0,1] (1 = no cut), or NULL: the target law
                                                     of every row is cut to its nucleus before the acceptance test
                                                     (Regime B of Sec. V samples with top-p): the most probable
                                                     tokens whose mass first reaches top_p, with every token tied
                                                     with the last one kept; ignored where T_b = 0                */
  const float *top_p_host;           /* HOST   [B]   same values (NULL with top_p NULL)                           */
  const int32_t *top_k;              /* DEVICE [B]   top-k cut of the target law (0 or >= vocab = off), or NULL: the k most
                                                     probable tokens with every token tied with the last of them; applied
                                                     before top_p, which then works on the renormalised rest (the other
                                                     common form of Regime B's cut target law); ignored where T_b = 0     */
  const int32_t *top_k_host;         /* HOST   [B]   same values (NULL with top_k NULL)                           */
  const int32_t *adapter;            /* DEVICE [B]   which adapter of fsv_lora_load() the request's target version uses
                                                     (the evolved target of Sec. IV-A); any value outside 0 .. n_adapters-1
                                                     (say -1) = the base target; NULL = base target for everyone         */
} fsv_batch;

typedef struct {
  int32_t *accepted_len;   /* DEVICE [B] tau_b in [0, gamma_b]                                        */
  int32_t *next_token;     /* DEVICE [B] correction token (tau_b < gamma_b) or bonus token            */
  int32_t *new_seq_lens;   /* DEVICE [B] seq_lens[b] + 1 + tau_b: valid KV positions after rollback   */
  int32_t *pages_released; /* DEVICE [B] tail pages that hold no valid position any more              */
  uint32_t *flags;         /* DEVICE [B] bit0: some tested draft had |u - min(1,p/q)| < 1e-4;
                                         bit1: the emitted token's CDF edge is within 1e-6 of u_sample;
                                         bit2: the token was drawn from the residual max(0, p - q);
                                         bit3: on a row the outcome rests on, the nucleus cut lies within 1e-6
                                               (of the row's mass) of top_p                                   */
  float *logits_out;       /* DEVICE [M][vocab] fp32 target logits, or NULL                           */
} fsv_result;

/*
 * Create a context for one target model M_t' (the "Require: target model" of Alg. 2; Sec. IV-A: the cloud holds the
 * evolving target, the edge only a frozen draft): validate the description, copy / re-tile the weights, allocate the
 * workspace.
 * Supported shapes: page_size 16; head_dim 64 or 128 for FSV_BF16 (any even head_dim for FSV_F32);
 * n_heads a multiple of n_kv_heads with n_heads / n_kv_heads * (max_gamma + 1) <= 96;
 * d_model, d_ffn and n_heads*head_dim multiples of 256 for FSV_BF16; every weight matrix below 4 GiB.
 * For FSV_BF16 one layer of a KV pool (num_pages * n_kv_heads * 16 * head_dim * 2 bytes) must stay below
 * 4 GiB: fsv_verify / fsv_attention return FSV_E_UNSUPPORTED otherwise.
 * weights may be NULL only when n_layers == 0.
 */
int fsv_create(const fsv_model_desc *desc, const fsv_weights *weights, fsv_ctx **out);
/* Release everything fsv_create allocated (no passage of the paper: lifetime plumbing of the boundary).  The caller's
 * pools, page tables and sessions are untouched: a session outlives the context that served it (Sec. IV-C). */
void fsv_destroy(fsv_ctx *ctx);

/*
 * Adapters of the evolving target (Sec. IV-A: the target's parameters are the frozen backbone plus PEFT adapters injected
 * into the transformer layers; the last transformer block and the LM head stay invariant, which is what keeps a frozen
 * edge draft compatible).  An adapter is a LoRA pair per layer l < n_layers - 1 on the fused q|k|v projection and on the
 * output projection:  qkv = W_qkv a + scale B_qkv (A_qkv a),  o = W_o att + scale B_o (A_o att),  with the low-rank
 * products kept in fp32.  One batch may mix requests of different target versions (fsv_batch.adapter).
 * All matrices are DEVICE, row-major [out][in], bf16: A_qkv [rank][d_model], B_qkv [(n_heads + 2 n_kv_heads) head_dim][rank],
 * A_o [rank][n_heads head_dim], B_o [d_model][rank]; the four tables are HOST arrays of (n_layers - 1) * n_adapters DEVICE
 * pointers, entry l * n_adapters + a.  fsv_lora_load copies everything (the caller may free its matrices afterwards) and
 * replaces any set loaded before; lora NULL or n_adapters 0 removes the adapters.  FSV_BF16 models, rank 8 / 16 / 32 / 64.
 * Not to be called while a call on the context is in flight.
 */
typedef struct {
  int32_t n_adapters, rank;
  const float *scale;                 /* HOST [n_adapters]: the factor s (alpha / rank of the LoRA literature) */
  const void *const *a_qkv, *const *b_qkv, *const *a_o, *const *b_o;
} fsv_lora;
int fsv_lora_load(fsv_ctx *ctx, const fsv_lora *lora);

/*
 * The edge draft model on the cloud (Sec. IV-A, structural definition): M_d(x) = H_small(B_shared(x)), where B_shared is
 * a frozen copy of the anchor block -- the base target's LAST transformer block, which the context already holds -- and
 * H_small is a two-layer MLP followed by a vocabulary projection, z = W_v (W_2 silu(W_1 h)) on the block's output h.
 * The uplink carries token ids only (Sec. IV-B); with the draft model the cloud recomputes the law q_i(.) each received
 * draft was drawn from, which the acceptance test of fsv_verify needs when T_b > 0, instead of receiving it.
 *
 * fsv_draft_attach: give the context the head (DEVICE, bf16, row-major [out][in]: w1 [d_hidden][d_model],
 *   w2 [d_proj][d_hidden], w_vocab [vocab][d_proj]; d_hidden and d_proj multiples of 256).  The matrices are re-tiled
 *   and may be freed afterwards; NULL removes the head.  FSV_BF16 models only.
 * fsv_draft_probs: run the draft model over the same rows a verification call scores (pending token + drafts of every
 *   request) on the DRAFT's KV session -- batch->k_pool / v_pool are pools of ONE layer here, same page tables and
 *   lengths as the target's session, appended to in place -- and write q = softmax(z / T_b), fp32:
 *     FSV_DRAFT_Q_VERIFY: q_out [G][vocab], row draft_offsets[b] + i = the law of draft i+1 of request b (from its
 *                         input row i): exactly fsv_batch.draft_probs of the verification call that follows;
 *     FSV_DRAFT_Q_ALL:    q_out [M][vocab], one law per input row (what an edge device samples its next draft from).
 *   Rows of requests with T_b = 0 are left untouched.  logits_out (DEVICE [M][vocab] fp32) may be NULL.
 *   Uses from batch: batch, num_pages, seq_lens(+_host), last_token, draft_offsets(+_host), draft_tokens, temperature,
 *   page_table, k_pool, v_pool.  After the verification call both sessions hold new_seq_lens valid positions.
 */
typedef struct {
  int32_t d_hidden, d_proj;
  const void *w1, *w2, *w_vocab;
} fsv_draft_head;
enum { FSV_DRAFT_Q_VERIFY = 0, FSV_DRAFT_Q_ALL = 1 };
int fsv_draft_attach(fsv_ctx *ctx, const fsv_draft_head *head);
/* fsv_kv_import / fsv_kv_export for the draft's one-layer session: src / dst are [n_pos][n_kv_heads][head_dim]. */
int fsv_draft_kv_import(fsv_ctx *ctx, void *k_pool, void *v_pool, int32_t num_pages, const int32_t *page_table_row,
                        int32_t pos0, int32_t n_pos, const void *src_k, const void *src_v, void *stream);
int fsv_draft_kv_export(fsv_ctx *ctx, const void *k_pool, const void *v_pool, int32_t num_pages,
                        const int32_t *page_table_row, int32_t pos0, int32_t n_pos, void *dst_k, void *dst_v, void *stream);
int fsv_draft_probs(fsv_ctx *ctx, const fsv_batch *batch, int32_t rows_mode, float *q_out, float *logits_out, void *stream);

/*
 * The verification step (Alg. 2 step 2 with the KV append / rollback of Sec. IV-C) for a batch.
 * For T_b > 0 the acceptance rule is speculative sampling, which keeps the law of the emitted
 * tokens equal to the target model's (Sec. II; Regime B of Sec. V): draft i is accepted iff
 * u_i < min(1, p_{i-1}(d_i) / q_i(d_i)) with p = softmax(logits / T_b); after the first rejection
 * at i = tau+1 the token is drawn by inverse CDF (ascending token id, first id whose inclusive
 * running mass exceeds u_sample * total) from max(0, p_tau - q_{tau+1}); when all drafts pass,
 * from p_gamma.  For T_b = 0: accept while d_i == argmax, emit the argmax (lowest id on ties).
 */
int fsv_verify(fsv_ctx *ctx, const fsv_batch *batch, const fsv_result *result, void *stream);

/*
 * The target forward alone: extend KV sessions by rows that need no accept / reject decision -- restoring a user's
 * context from tokens instead of from a saved cache (Alg. 2 "restore KV cache"; Sec. IV-C: the cloud computes the KV
 * pairs of the tokens it receives), e.g. a prompt taken in chunks.  Request b contributes the rows last_token[b],
 * draft_tokens[draft_offsets[b] ..) at positions seq_lens[b] ... exactly as in fsv_verify, their K / V rows are
 * appended, and the call stops after the LM head.  A chunk longer than max_gamma + 1 rows is passed as several
 * requests that share ONE page-table row content and continue each other (seq_lens of the next = seq_lens + rows of
 * the one before): within a layer all rows are appended before any row attends, so a later piece sees the earlier
 * pieces' keys.  Uses from batch: batch, seq_lens(+_host), last_token, draft_offsets(+_host), draft_tokens,
 * page_table, k_pool, v_pool, num_pages (and adapter).  logits_out: DEVICE [M][vocab] fp32, row order as in
 * fsv_verify, or NULL when only the cache is wanted (the logits then stay in the context's own buffer).
 * Nothing is rolled back: the caller's new length of request b is seq_lens[b] + its rows.
 */
int fsv_prefill(fsv_ctx *ctx, const fsv_batch *batch, float *logits_out, void *stream);

/*
 * The accept / resample step alone -- the acceptance loop of Alg. 2 step 2 and its "sample correction token" line, with
 * the speculative-sampling rule of fsv_verify for T_b > 0 -- on caller-provided target logits (DEVICE [M][vocab], row
 * draft_offsets[b] + b + i scores the token after input row i of request b; dtype FSV_BF16 or
 * FSV_F32).  Uses from batch: batch, draft_offsets(+_host), draft_tokens, draft_probs, u_accept,
 * u_sample, temperature(+_host).  Writes accepted_len, next_token, flags.
 */
int fsv_sample(fsv_ctx *ctx, const void *logits, int32_t logits_dtype, const fsv_batch *batch,
               const fsv_result *result, void *stream);

/*
 * fsv_sample for callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same inputs, outputs and arithmetic as fsv_sample, but no context: the sampler's
 * workspace is a fixed 1 MiB device array inside the library (one copy per GPU, held until the process ends), so the
 * call allocates and frees nothing, on the device or through any library.  Limits: batch <= 128, at most 16 drafts per
 * request, at most 1024 rows (drafts + requests), vocab <= 327680; beyond them the call returns FSV_E_CAPACITY and
 * launches nothing.  Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (different streams
 * or threads) race on it; calls on one stream are ordered and safe.  The array keeps the last call's contents; nothing
 * in it needs clearing between calls (every entry a call reads it has written first).  No per-call error text
 * (fsv_last_error needs a context).
 */
int fsv_sample_static(int32_t vocab, const void *logits, int32_t logits_dtype, const fsv_batch *batch,
                      const fsv_result *result, void *stream);

/*
 * KV rollback alone (Sec. IV-C): from seq_lens, draft_offsets and accepted_len (DEVICE [B])
 * compute new_seq_lens and pages_released.  Discarded positions keep stale bytes that no later
 * call reads; the caller returns released pages to its allocator.
 */
int fsv_rollback(fsv_ctx *ctx, const fsv_batch *batch, const int32_t *accepted_len,
                 const fsv_result *result, void *stream);

/*
 * Restore / save a user's KV session (Alg. 2 "restore KV cache").  src_k / src_v (dst for
 * export) are DEVICE arrays [n_layers][n_pos][n_kv_heads][head_dim] of the model's dtype holding
 * positions pos0 .. pos0+n_pos-1; page_table_row is the DEVICE page-table row of the request.
 * For FSV_BF16 a K tile stores element (t, e) (position t in page, feature e) at
 * ((e/16*2 + (e%16)/8)*16 + t)*8 + e%8 and a V tile at ((e/32*2 + (t%8)/4)*32 + e%32)*8 + 4*(t/8) + t%4.
 */
int fsv_kv_import(fsv_ctx *ctx, void *k_pool, void *v_pool, int32_t num_pages, const int32_t *page_table_row,
                  int32_t pos0, int32_t n_pos, const void *src_k, const void *src_v, void *stream);
int fsv_kv_export(fsv_ctx *ctx, const void *k_pool, const void *v_pool, int32_t num_pages,
                  const int32_t *page_table_row, int32_t pos0, int32_t n_pos, void *dst_k, void *dst_v,
                  void *stream);

/*
 * Single kernels of the step, exposed for parity tests and roofline measurements.
 * fsv_linear: y[M][N] (fp32, DEVICE) = x[M][K] (model dtype, row-major, DEVICE) times the re-tiled
 *   weight matrix `which` of `layer` (FSV_W_* below; layer ignored for FSV_W_LM_HEAD), through the
 *   same weight-streaming GEMM kernel fsv_verify uses.  M <= max_rows.
 * fsv_attention: out[M][n_heads*head_dim] (fp32, DEVICE) for queries q[M][n_heads][head_dim] (model
 *   dtype, already rotated) over the paged KV of `layer`; row i of request b attends to positions
 *   0 .. seq_lens[b] + i.  Uses from batch: batch, num_pages, seq_lens(+_host), draft_offsets(+_host),
 *   page_table, k_pool, v_pool.
 */
enum { FSV_W_QKV = 0, FSV_W_O = 1, FSV_W_GATE_UP = 2, FSV_W_DOWN = 3, FSV_W_LM_HEAD = 4 };
int fsv_linear(fsv_ctx *ctx, int32_t which, int32_t layer, const void *x, int32_t M, float *y, void *stream);
int fsv_attention(fsv_ctx *ctx, int32_t layer, const void *q, const fsv_batch *batch, float *out, void *stream);

/*
 * Per-kernel timing with HIP events on the call's stream.  fsv_profile_enable(ctx, mask) makes every
 * later fsv_verify / fsv_sample / fsv_linear / fsv_attention record an event pair around each launch
 * of the kernel classes whose bit (1u << FSV_K_*) is set in mask (0 = off, 0xffffffff = all; at most
 * 8192 launches are kept, later ones are not recorded).  For the GEMM and attention classes the pair
 * rides on the dispatch itself (start and stop of the kernel); for the other classes it is recorded on
 * the stream before and after the launches and so includes the dispatch gaps.  FSV_K_SAMPLE_NUCLEUS brackets
 * all the cut passes of one call (one per key digit and per kind of cut) as one record.  fsv_profile_read() waits for the recorded
 * events and returns, per class, the number of launches, their summed duration and the algorithmic
 * bytes the host computed for them (weights for a GEMM, K and V for attention, logits and draft law
 * for the sampling kernels), then clears the records.  Returns the number of classes written (<= cap).
 */
enum { FSV_K_GEMM_QKV = 0, FSV_K_GEMM_O, FSV_K_GEMM_GATE_UP, FSV_K_GEMM_DOWN, FSV_K_GEMM_LM_HEAD,
       FSV_K_ATTENTION, FSV_K_ATTN_COMBINE, FSV_K_SAMPLE_STATS, FSV_K_SAMPLE_DECIDE, FSV_K_SAMPLE_NUCLEUS,
       FSV_K_NORM, FSV_K_ROPE_APPEND, FSV_K_OTHER, FSV_K_COUNT };
typedef struct {
  int32_t kernel_class; /* FSV_K_*                       */
  int32_t launches;
  double total_ms;      /* sum of event-to-event times   */
  double bytes;         /* algorithmic bytes of those launches as the host computed them at launch  */
} fsv_kernel_time;
int fsv_profile_enable(fsv_ctx *ctx, uint32_t class_mask);
/* Record only every every_n-th launch of each enabled class (1 = all, the default): the event pairs cost a few
 * microseconds of host and dispatch time each, which a timed region with hundreds of launches need not pay in full. */
int fsv_profile_sample(fsv_ctx *ctx, int32_t every_n);
int fsv_profile_read(fsv_ctx *ctx, fsv_kernel_time *out, int32_t cap);
const char *fsv_kernel_class_name(int32_t kernel_class);

/*
 * State around the verification step (host only; no device memory, no stream).
 *
 * Stride selection (Sec. IV-B, refined latency model and throughput objective; Alg. 2 step 1): with
 *   T_fixed    = t_prop + t_base + t_down + header_bits / rate + beta
 *   T_marginal = alpha_edge + bits_per_token / rate + delta_cloud                  (times in seconds, rate in bit/s)
 * fsv_policy_stride returns K* = argmax over K in 1..k_max of E[tokens | K] / (T_fixed + K T_marginal), ties to the
 * smallest K, where E[tokens | K] = 1 + gamma_hat K (FSV_TAU_LINEAR, the numerator Alg. 2 prints) or
 * 1 + gamma_hat + ... + gamma_hat^K (FSV_TAU_GEOMETRIC, the geometric decay model Sec. IV-B names).  The linear
 * numerator makes the objective monotone in K, so its optimum is always 1 or k_max.  *objective_out (may be NULL)
 * receives the objective at K* in tokens per second.  Returns K* >= 1, or a negative fsv_status on a bad argument.
 *
 * fsv_policy_ema is the acceptance-rate average of Alg. 2 step 3: (1 - mu) gamma_hat + mu tau / k (started at 0.8
 * by the algorithm); k <= 0 leaves gamma_hat unchanged.
 */
typedef struct {
  double alpha_edge, beta;             /* edge drafting time: alpha_edge K + beta                        */
  double bits_per_token, header_bits;  /* uplink payload: K b + O_header bits                             */
  double t_prop, t_base, delta_cloud, t_down; /* propagation, cloud base cost, cloud cost per token, downlink */
} fsv_latency_model;
enum { FSV_TAU_LINEAR = 0, FSV_TAU_GEOMETRIC = 1 };
int fsv_policy_stride(const fsv_latency_model *model, double rate, double gamma_hat, int32_t k_max, int32_t tau_model,
                      double *objective_out);
double fsv_policy_ema(double gamma_hat, int32_t tau, int32_t k, double mu);
/* T_step(K, R) = T_edge + T_up + T_cloud + T_down of the same model (Sec. III, step latency; Sec. IV-B for the terms),
 * in seconds; cloud_seconds >= 0 replaces the modelled T_cloud = t_base + K delta_cloud by a measured verification
 * time.  Returns -1 on a bad argument. */
double fsv_policy_step_time(const fsv_latency_model *model, double rate, int32_t k, double cloud_seconds);

/*
 * Page bookkeeping of the persistent per-user KV sessions (Sec. IV-C): which physical pages of the pools a session
 * owns.  HOST only; the caller uploads the page-table rows it passes to fsv_verify.  Not thread safe.
 *   fsv_pager_reserve: make session own ceil(n_positions / 16) pages (it keeps what it has, takes the lowest free
 *     ids for the rest) and write its pages, in logical order, to page_table_row (HOST, at least that many entries;
 *     may be NULL).  FSV_E_CAPACITY when the pool or max_pages_per_session cannot cover it: nothing is taken then.
 *     Call it with seq_len + gamma + 1 before a verification call.
 *   fsv_pager_trim: give back the tail pages beyond ceil(n_positions / 16) (the rollback of rejected positions: pass
 *     new_seq_lens[b]); returns the number of pages released, which equals pages_released[b] of that call.
 *     n_positions = 0 ends the session.
 */
typedef struct fsv_pager fsv_pager;
int fsv_pager_create(int32_t num_pages, int32_t max_sessions, int32_t max_pages_per_session, fsv_pager **out);
void fsv_pager_destroy(fsv_pager *pager);
int fsv_pager_reserve(fsv_pager *pager, int32_t session, int32_t n_positions, int32_t *page_table_row);
int fsv_pager_trim(fsv_pager *pager, int32_t session, int32_t n_positions);
int32_t fsv_pager_free_pages(const fsv_pager *pager);
int32_t fsv_pager_session_pages(const fsv_pager *pager, int32_t session);

/* Text of a status code (no passage of the paper: error convention of the boundary). */
const char *fsv_strerror(int status);
/* Last failure's detail message for this context (HOST string owned by the context). */
const char *fsv_last_error(const fsv_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* FLEXVERIFY_H */
