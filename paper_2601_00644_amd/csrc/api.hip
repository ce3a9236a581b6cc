// C-ABI entry points of libflexverify: argument validation, workspace, launch order of the
// verification step (Alg. 2 step 2 and the KV session handling of Sec. IV-C).
#include <math.h>
#include <new>

#include "fsv_internal.h"

namespace {

const char *kClassNames[FSV_K_COUNT] = {"gemm_qkv",     "gemm_o",        "gemm_gate_up",  "gemm_down",  "gemm_lm_head",
                                        "attention",    "attn_combine",  "sample_stats",  "sample_decide",
                                        "sample_nucleus", "norm",         "rope_append",   "other"};

template <typename T>
int dev_alloc(fsv_ctx *c, T **p, size_t n) {
  FSV_HIP(c, hipMalloc((void **)p, sizeof(T) * (n ? n : 1)));
  return FSV_OK;
}

}  // namespace

// Checks shared by verify / sample / attention: CSR shape and capacity.  Returns M (rows) or < 0.
int fsv_check_batch(fsv_ctx *c, const fsv_batch *b, bool need_kv, bool need_sampling) {
  if (!b) FSV_FAIL(c, FSV_E_INVALID_ARG, "batch is NULL");
  if (b->batch < 0) FSV_FAIL(c, FSV_E_INVALID_ARG, "negative batch");
  if (b->batch > c->d.max_batch) FSV_FAIL(c, FSV_E_CAPACITY, "batch %d > max_batch %d", b->batch, c->d.max_batch);
  if (b->batch == 0) return 0;
  if (!b->draft_offsets || !b->draft_offsets_host) FSV_FAIL(c, FSV_E_INVALID_ARG, "draft_offsets (device and host) required");
  const int32_t *off = b->draft_offsets_host;
  if (off[0] != 0) FSV_FAIL(c, FSV_E_INVALID_ARG, "draft_offsets[0] must be 0");
  for (int i = 0; i < b->batch; ++i) {
    int g = off[i + 1] - off[i];
    if (g < 0) FSV_FAIL(c, FSV_E_INVALID_ARG, "draft_offsets not monotone at request %d", i);
    if (g > c->d.max_gamma) FSV_FAIL(c, FSV_E_CAPACITY, "request %d has %d drafts > max_gamma %d", i, g, c->d.max_gamma);
  }
  const int G = off[b->batch], M = G + b->batch;
  if (M > c->max_rows) FSV_FAIL(c, FSV_E_CAPACITY, "%d rows > max_rows %d", M, c->max_rows);
  if (need_sampling) {
    if (!b->u_sample || !b->temperature) FSV_FAIL(c, FSV_E_INVALID_ARG, "u_sample and temperature required");
    if (G > 0 && !b->draft_tokens) FSV_FAIL(c, FSV_E_INVALID_ARG, "draft_tokens required");
    bool any_pos = true;
    if (b->temperature_host) {
      any_pos = false;
      for (int i = 0; i < b->batch; ++i) {
        float t = b->temperature_host[i];
        if (!(t >= 0.f) || isinf(t)) FSV_FAIL(c, FSV_E_INVALID_ARG, "temperature of request %d is not finite and >= 0", i);
        any_pos |= t > 0.f;
      }
    }
    if (any_pos && G > 0 && (!b->draft_probs || !b->u_accept))
      FSV_FAIL(c, FSV_E_INVALID_ARG, "draft_probs and u_accept required when a temperature is positive");
    if ((b->top_p != nullptr) != (b->top_p_host != nullptr))
      FSV_FAIL(c, FSV_E_INVALID_ARG, "top_p needs both its device and its host copy (or neither)");
    if (b->top_p_host)
      for (int i = 0; i < b->batch; ++i)
        if (!(b->top_p_host[i] > 0.f) || !(b->top_p_host[i] <= 1.f))
          FSV_FAIL(c, FSV_E_INVALID_ARG, "top_p of request %d is not in (0, 1]", i);
    if ((b->top_k != nullptr) != (b->top_k_host != nullptr))
      FSV_FAIL(c, FSV_E_INVALID_ARG, "top_k needs both its device and its host copy (or neither)");
    if (b->top_k_host)
      for (int i = 0; i < b->batch; ++i)
        if (b->top_k_host[i] < 0) FSV_FAIL(c, FSV_E_INVALID_ARG, "top_k of request %d is negative", i);
  }
  if (need_kv) {
    if (!b->seq_lens || !b->seq_lens_host || !b->page_table || !b->k_pool || !b->v_pool)
      FSV_FAIL(c, FSV_E_INVALID_ARG, "seq_lens (device and host), page_table, k_pool, v_pool required");
    if (b->num_pages <= 0) FSV_FAIL(c, FSV_E_INVALID_ARG, "num_pages must be positive");
    for (int i = 0; i < b->batch; ++i) {
      int L = b->seq_lens_host[i], g = off[i + 1] - off[i];
      if (L < 0) FSV_FAIL(c, FSV_E_INVALID_ARG, "seq_lens[%d] negative", i);
      if (fsv_ceil_div(L + g + 1, c->d.page_size) > c->d.max_pages_per_req)
        FSV_FAIL(c, FSV_E_CAPACITY, "request %d needs %d pages > max_pages_per_req %d", i,
                 fsv_ceil_div(L + g + 1, c->d.page_size), c->d.max_pages_per_req);
    }
  }
  return M;
}

extern "C" {

const char *fsv_strerror(int status) {
  switch (status) {
    case FSV_OK: return "ok";
    case FSV_E_INVALID_ARG: return "invalid argument";
    case FSV_E_CAPACITY: return "beyond the capacity the context was created with";
    case FSV_E_UNSUPPORTED: return "shape not supported by the kernels";
    case FSV_E_HIP: return "HIP runtime error";
    case FSV_E_NO_MODEL: return "context holds no model";
    default: return "unknown status";
  }
}

const char *fsv_last_error(const fsv_ctx *ctx) { return ctx ? ctx->err.c_str() : ""; }

const char *fsv_kernel_class_name(int32_t k) { return (k >= 0 && k < FSV_K_COUNT) ? kClassNames[k] : "?"; }

void fsv_destroy(fsv_ctx *c) {
  if (!c) return;
  for (auto &r : c->prof) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  for (hipEvent_t e : c->prof_pool) (void)hipEventDestroy(e);
  void *ptrs[] = {c->embed, c->final_norm, c->lm_head, c->inv_freq, c->rope_tab, c->row_req, c->row_idx, c->row_pos, c->row_tok,
                  c->pmax, c->psum, c->parg, c->bsum, c->acc_scratch, c->sel_ticket, c->nuc_prefix,
                  c->nuc_key, c->nuc_above, c->nuc_total, c->nuc_S, c->nuc_near, c->nuc_done, c->nuc_cabove, c->nuc_kkey, c->nuc_kmass, c->x, c->logits,
                  c->absmax, c->buf_a, c->buf_qkv, c->buf_q, c->buf_att, c->buf_gu, c->buf_act, c->buf_part, c->attn_part, c->attn_part_prefix, c->attn_part_map,
                  c->lora_aq, c->lora_bq, c->lora_ao, c->lora_bo, c->lora_scale, c->lora_t,
                  c->draft_w1, c->draft_w2, c->draft_wv, c->draft_h1, c->draft_h2};
  for (void *p : ptrs)
    if (p) (void)hipFree(p);
  for (auto &L : c->layers) {
    void *lp[] = {L.attn_norm, L.w_qkv, L.w_o, L.mlp_norm, L.w_gate_up, L.w_down};
    for (void *p : lp)
      if (p) (void)hipFree(p);
  }
  delete c;
}

int fsv_create(const fsv_model_desc *desc, const fsv_weights *w, fsv_ctx **out) {
  if (!desc || !out) return FSV_E_INVALID_ARG;
  *out = nullptr;
  const fsv_model_desc &d = *desc;
  if (d.vocab <= 0 || d.max_batch <= 0 || d.max_gamma < 0 || d.n_layers < 0) return FSV_E_INVALID_ARG;
  if (d.max_gamma > 16) return FSV_E_UNSUPPORTED;
  if (fsv_ceil_div(d.vocab, FSV_SBK) > 160) return FSV_E_UNSUPPORTED;
  if (d.n_layers > 0) {
    if (!w) return FSV_E_INVALID_ARG;
    if (d.dtype != FSV_F32 && d.dtype != FSV_BF16) return FSV_E_INVALID_ARG;
    if (d.d_model <= 0 || d.n_heads <= 0 || d.n_kv_heads <= 0 || d.head_dim <= 0 || d.d_ffn <= 0) return FSV_E_INVALID_ARG;
    if (d.page_size != 16 || d.n_heads % d.n_kv_heads != 0 || d.head_dim % 2 != 0) return FSV_E_UNSUPPORTED;
    if (d.max_pages_per_req <= 0) return FSV_E_INVALID_ARG;
    if (d.n_heads / d.n_kv_heads * (d.max_gamma + 1) > 96) return FSV_E_UNSUPPORTED;
    if (d.dtype == FSV_BF16) {
      if (d.head_dim != 64 && d.head_dim != 128) return FSV_E_UNSUPPORTED;
      if (d.d_model % 256 || d.d_ffn % 256 || (d.n_heads * d.head_dim) % 256) return FSV_E_UNSUPPORTED;
    }
    if (!w->embed || !w->final_norm || !w->lm_head || !w->attn_norm || !w->w_qkv || !w->w_o || !w->mlp_norm ||
        !w->w_gate_up || !w->w_down)
      return FSV_E_INVALID_ARG;
  }
  fsv_ctx *c = new (std::nothrow) fsv_ctx();
  if (!c) return FSV_E_HIP;
  c->d = d;
  c->max_rows = d.max_rows > 0 ? d.max_rows : d.max_batch * (d.max_gamma + 1);
  c->group = d.n_layers > 0 ? d.n_heads / d.n_kv_heads : 1;
  c->nsb = fsv_ceil_div(d.vocab, FSV_SBK);
  c->nc = fsv_ceil_div(d.vocab, FSV_CHUNK);
  const size_t R = c->max_rows, B = d.max_batch;
  int rc = FSV_OK;
  auto A = [&](int r) { if (rc == FSV_OK) rc = r; };
  A(dev_alloc(c, &c->row_req, R)); A(dev_alloc(c, &c->row_idx, R)); A(dev_alloc(c, &c->row_pos, R));
  A(dev_alloc(c, &c->row_tok, R));
  A(dev_alloc(c, &c->pmax, R * c->nc)); A(dev_alloc(c, &c->psum, R * c->nc)); A(dev_alloc(c, &c->parg, R * c->nc));
  A(dev_alloc(c, &c->bsum, B * c->nsb));
  A(dev_alloc(c, &c->acc_scratch, B));
  A(dev_alloc(c, &c->sel_ticket, B));
  if (rc == FSV_OK && hipMemset(c->sel_ticket, 0, sizeof(int32_t) * B) != hipSuccess) rc = FSV_E_HIP;
  A(dev_alloc(c, &c->nuc_prefix, R)); A(dev_alloc(c, &c->nuc_key, R)); A(dev_alloc(c, &c->nuc_above, R));
  A(dev_alloc(c, &c->nuc_total, R)); A(dev_alloc(c, &c->nuc_S, R)); A(dev_alloc(c, &c->nuc_near, R));
  A(dev_alloc(c, &c->nuc_cabove, R)); A(dev_alloc(c, &c->nuc_kkey, R)); A(dev_alloc(c, &c->nuc_kmass, R));
  A(dev_alloc(c, &c->nuc_done, R));
  if (rc == FSV_OK && d.n_layers > 0) {
    const size_t rows_pad = (R + 31) / 32 * 32;
    A(dev_alloc(c, &c->x, rows_pad * d.d_model));
    A(dev_alloc(c, &c->logits, R * (size_t)d.vocab));
    if (rc == FSV_OK) rc = (d.dtype == FSV_F32) ? fsv_f32_create(c, w) : fsv_bf16_create(c, w);
    if (rc == FSV_OK && hipDeviceSynchronize() != hipSuccess) rc = FSV_E_HIP;
  }
  if (rc != FSV_OK) {
    fprintf(stderr, "fsv_create: %s (%s)\n", fsv_strerror(rc), c->err.c_str());
    fsv_destroy(c);
    return rc;
  }
  *out = c;
  return FSV_OK;
}

int fsv_verify(fsv_ctx *c, const fsv_batch *b, const fsv_result *r, void *stream) {
  if (!c) return FSV_E_INVALID_ARG;
  if (c->d.n_layers == 0) FSV_FAIL(c, FSV_E_NO_MODEL, "fsv_verify on a sampler-only context");
  if (!r || !r->next_token || !r->flags || !r->new_seq_lens) FSV_FAIL(c, FSV_E_INVALID_ARG, "result pointers missing");
  const int M = fsv_check_batch(c, b, true, true);
  if (M <= 0) return M;
  if (!b->last_token) FSV_FAIL(c, FSV_E_INVALID_ARG, "last_token required");
  hipStream_t s = (hipStream_t)stream;
  float *logits = r->logits_out ? r->logits_out : c->logits;
  // everything that can still fail is decided on the host before the first launch
  fsv_attn_plan pl;
  int rc = (c->d.dtype == FSV_F32) ? fsv_f32_check(c, b) : fsv_bf16_attn_plan_host(c, b, &pl);
  if (rc) return rc;
  if ((rc = fsv_launch_build_rows(c, b, M, s))) return rc;
  rc = (c->d.dtype == FSV_F32) ? fsv_f32_forward(c, b, M, logits, s) : fsv_bf16_forward(c, b, &pl, M, logits, 0, s);
  if (rc) return rc;
  return fsv_launch_sampler(c, logits, FSV_F32, b, r, M, true, s);
}

int fsv_prefill(fsv_ctx *c, const fsv_batch *b, float *logits_out, void *stream) {
  if (!c) return FSV_E_INVALID_ARG;
  if (c->d.n_layers == 0) FSV_FAIL(c, FSV_E_NO_MODEL, "fsv_prefill on a sampler-only context");
  const int M = fsv_check_batch(c, b, true, false);
  if (M <= 0) return M;
  if (!b->last_token) FSV_FAIL(c, FSV_E_INVALID_ARG, "last_token required");
  if (b->draft_offsets_host[b->batch] > 0 && !b->draft_tokens) FSV_FAIL(c, FSV_E_INVALID_ARG, "draft_tokens required");
  hipStream_t s = (hipStream_t)stream;
  float *logits = logits_out ? logits_out : c->logits;
  fsv_attn_plan pl;
  int rc = (c->d.dtype == FSV_F32) ? fsv_f32_check(c, b) : fsv_bf16_attn_plan_host(c, b, &pl);
  if (rc) return rc;
  if ((rc = fsv_launch_build_rows(c, b, M, s))) return rc;
  return (c->d.dtype == FSV_F32) ? fsv_f32_forward(c, b, M, logits, s) : fsv_bf16_forward(c, b, &pl, M, logits, 0, s);
}

int fsv_sample(fsv_ctx *c, const void *logits, int32_t logits_dtype, const fsv_batch *b, const fsv_result *r,
               void *stream) {
  if (!c) return FSV_E_INVALID_ARG;
  if (!logits || !r || !r->next_token || !r->flags) FSV_FAIL(c, FSV_E_INVALID_ARG, "logits / result pointers missing");
  if (logits_dtype != FSV_F32 && logits_dtype != FSV_BF16) FSV_FAIL(c, FSV_E_INVALID_ARG, "bad logits dtype");
  const int M = fsv_check_batch(c, b, false, true);
  if (M <= 0) return M;
  return fsv_launch_sampler(c, logits, logits_dtype, b, r, M, false, (hipStream_t)stream);
}

int fsv_rollback(fsv_ctx *c, const fsv_batch *b, const int32_t *accepted_len, const fsv_result *r, void *stream) {
  if (!c) return FSV_E_INVALID_ARG;
  if (!b || !accepted_len || !r || !r->new_seq_lens) FSV_FAIL(c, FSV_E_INVALID_ARG, "NULL argument");
  if (b->batch < 0 || !b->seq_lens || !b->draft_offsets) FSV_FAIL(c, FSV_E_INVALID_ARG, "seq_lens / draft_offsets missing");
  if (b->batch > c->d.max_batch) FSV_FAIL(c, FSV_E_CAPACITY, "batch %d > max_batch %d", b->batch, c->d.max_batch);
  if (b->batch == 0) return FSV_OK;
  return fsv_launch_rollback(c, b, accepted_len, r, (hipStream_t)stream);
}

static int kv_copy(fsv_ctx *c, void *k_pool, void *v_pool, int32_t num_pages, const int32_t *pt, int32_t pos0,
                   int32_t n, void *kl, void *vl, bool import, void *stream, bool draft = false) {
  if (!c) return FSV_E_INVALID_ARG;
  if (c->d.n_layers == 0) FSV_FAIL(c, FSV_E_NO_MODEL, "KV copy on a sampler-only context");
  if (!k_pool || !v_pool || !pt || !kl || !vl || num_pages <= 0 || pos0 < 0 || n < 0)
    FSV_FAIL(c, FSV_E_INVALID_ARG, "NULL pointer or negative size");
  if (fsv_ceil_div(pos0 + n, c->d.page_size) > c->d.max_pages_per_req)
    FSV_FAIL(c, FSV_E_CAPACITY, "positions up to %d exceed the page table", pos0 + n);
  if (n == 0) return FSV_OK;
  hipStream_t s = (hipStream_t)stream;
  if (draft) {
    if (c->d.dtype != FSV_BF16) FSV_FAIL(c, FSV_E_UNSUPPORTED, "the draft model is implemented for FSV_BF16 models");
    return fsv_bf16_kv_copy(c, k_pool, v_pool, num_pages, pt, pos0, n, kl, vl, import, 1, s);
  }
  return (c->d.dtype == FSV_F32) ? fsv_f32_kv_copy(c, k_pool, v_pool, num_pages, pt, pos0, n, kl, vl, import, s)
                                 : fsv_bf16_kv_copy(c, k_pool, v_pool, num_pages, pt, pos0, n, kl, vl, import, c->d.n_layers, s);
}

int fsv_draft_kv_import(fsv_ctx *c, void *k_pool, void *v_pool, int32_t num_pages, const int32_t *pt, int32_t pos0,
                        int32_t n_pos, const void *src_k, const void *src_v, void *stream) {
  return kv_copy(c, k_pool, v_pool, num_pages, pt, pos0, n_pos, (void *)src_k, (void *)src_v, true, stream, true);
}

int fsv_draft_kv_export(fsv_ctx *c, const void *k_pool, const void *v_pool, int32_t num_pages, const int32_t *pt,
                        int32_t pos0, int32_t n_pos, void *dst_k, void *dst_v, void *stream) {
  return kv_copy(c, (void *)k_pool, (void *)v_pool, num_pages, pt, pos0, n_pos, dst_k, dst_v, false, stream, true);
}

int fsv_kv_import(fsv_ctx *c, void *k_pool, void *v_pool, int32_t num_pages, const int32_t *pt, int32_t pos0,
                  int32_t n_pos, const void *src_k, const void *src_v, void *stream) {
  return kv_copy(c, k_pool, v_pool, num_pages, pt, pos0, n_pos, (void *)src_k, (void *)src_v, true, stream);
}

int fsv_kv_export(fsv_ctx *c, const void *k_pool, const void *v_pool, int32_t num_pages, const int32_t *pt,
                  int32_t pos0, int32_t n_pos, void *dst_k, void *dst_v, void *stream) {
  return kv_copy(c, (void *)k_pool, (void *)v_pool, num_pages, pt, pos0, n_pos, dst_k, dst_v, false, stream);
}

int fsv_lora_load(fsv_ctx *c, const fsv_lora *lo) {
  if (!c) return FSV_E_INVALID_ARG;
  if (c->d.n_layers == 0) FSV_FAIL(c, FSV_E_NO_MODEL, "fsv_lora_load on a sampler-only context");
  if (c->d.dtype != FSV_BF16) FSV_FAIL(c, FSV_E_UNSUPPORTED, "adapters are implemented for FSV_BF16 models");
  if (lo && lo->n_adapters != 0) {
    if (lo->n_adapters < 0 || lo->n_adapters > 1024) FSV_FAIL(c, FSV_E_INVALID_ARG, "n_adapters must be in 0..1024");
    if (lo->rank != 8 && lo->rank != 16 && lo->rank != 32 && lo->rank != 64)
      FSV_FAIL(c, FSV_E_UNSUPPORTED, "adapter rank %d: 8, 16, 32 and 64 are implemented", lo->rank);
    if (c->d.d_model > 8192) FSV_FAIL(c, FSV_E_UNSUPPORTED, "adapters need d_model <= 8192");
    if (!lo->scale || !lo->a_qkv || !lo->b_qkv || !lo->a_o || !lo->b_o) FSV_FAIL(c, FSV_E_INVALID_ARG, "NULL adapter table");
    const int cnt = (c->d.n_layers - 1) * lo->n_adapters;
    for (int i = 0; i < cnt; ++i)
      if (!lo->a_qkv[i] || !lo->b_qkv[i] || !lo->a_o[i] || !lo->b_o[i]) FSV_FAIL(c, FSV_E_INVALID_ARG, "NULL adapter matrix %d", i);
  }
  return fsv_bf16_lora_load(c, lo);
}

int fsv_draft_attach(fsv_ctx *c, const fsv_draft_head *h) {
  if (!c) return FSV_E_INVALID_ARG;
  if (c->d.n_layers == 0) FSV_FAIL(c, FSV_E_NO_MODEL, "fsv_draft_attach on a sampler-only context");
  if (c->d.dtype != FSV_BF16) FSV_FAIL(c, FSV_E_UNSUPPORTED, "the draft model is implemented for FSV_BF16 models");
  if (h) {
    if (!h->w1 || !h->w2 || !h->w_vocab) FSV_FAIL(c, FSV_E_INVALID_ARG, "NULL head matrix");
    if (h->d_hidden <= 0 || h->d_proj <= 0 || h->d_hidden % 256 || h->d_proj % 256)
      FSV_FAIL(c, FSV_E_UNSUPPORTED, "d_hidden and d_proj must be positive multiples of 256");
    if (c->d.d_model > 8192) FSV_FAIL(c, FSV_E_UNSUPPORTED, "the draft head needs d_model <= 8192");
  }
  return fsv_bf16_draft_attach(c, h);
}

int fsv_draft_probs(fsv_ctx *c, const fsv_batch *b, int32_t rows_mode, float *q_out, float *logits_out, void *stream) {
  if (!c) return FSV_E_INVALID_ARG;
  if (c->d.n_layers == 0) FSV_FAIL(c, FSV_E_NO_MODEL, "fsv_draft_probs on a sampler-only context");
  if (!c->draft_wv) FSV_FAIL(c, FSV_E_INVALID_ARG, "no draft head attached (fsv_draft_attach)");
  if (!q_out || (rows_mode != FSV_DRAFT_Q_VERIFY && rows_mode != FSV_DRAFT_Q_ALL)) FSV_FAIL(c, FSV_E_INVALID_ARG, "bad argument");
  const int M = fsv_check_batch(c, b, true, false);
  if (M <= 0) return M;
  if (!b->last_token || !b->temperature) FSV_FAIL(c, FSV_E_INVALID_ARG, "last_token and temperature required");
  if (b->draft_offsets_host[b->batch] > 0 && !b->draft_tokens) FSV_FAIL(c, FSV_E_INVALID_ARG, "draft_tokens required");
  fsv_attn_plan pl;
  int rc = fsv_bf16_attn_plan_host(c, b, &pl);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  if ((rc = fsv_launch_build_rows(c, b, M, s))) return rc;
  return fsv_bf16_draft_probs(c, b, &pl, M, rows_mode == FSV_DRAFT_Q_ALL, q_out, logits_out ? logits_out : c->logits, s);
}

int fsv_linear(fsv_ctx *c, int32_t which, int32_t layer, const void *x, int32_t M, float *y, void *stream) {
  if (!c) return FSV_E_INVALID_ARG;
  if (c->d.n_layers == 0) FSV_FAIL(c, FSV_E_NO_MODEL, "fsv_linear on a sampler-only context");
  if (!x || !y || M <= 0 || which < FSV_W_QKV || which > FSV_W_LM_HEAD) FSV_FAIL(c, FSV_E_INVALID_ARG, "bad argument");
  if (which != FSV_W_LM_HEAD && (layer < 0 || layer >= c->d.n_layers)) FSV_FAIL(c, FSV_E_INVALID_ARG, "bad layer");
  if (M > c->max_rows) FSV_FAIL(c, FSV_E_CAPACITY, "%d rows > max_rows %d", M, c->max_rows);
  hipStream_t s = (hipStream_t)stream;
  return (c->d.dtype == FSV_F32) ? fsv_f32_linear(c, which, layer, x, M, y, s) : fsv_bf16_linear(c, which, layer, x, M, y, s);
}

int fsv_attention(fsv_ctx *c, int32_t layer, const void *q, const fsv_batch *b, float *out, void *stream) {
  if (!c) return FSV_E_INVALID_ARG;
  if (c->d.n_layers == 0) FSV_FAIL(c, FSV_E_NO_MODEL, "fsv_attention on a sampler-only context");
  if (!q || !out || layer < 0 || layer >= c->d.n_layers) FSV_FAIL(c, FSV_E_INVALID_ARG, "bad argument");
  const int M = fsv_check_batch(c, b, true, false);
  if (M <= 0) return M;
  hipStream_t s = (hipStream_t)stream;
  fsv_attn_plan pl;
  int rc = (c->d.dtype == FSV_F32) ? fsv_f32_check(c, b) : fsv_bf16_attn_plan_host(c, b, &pl);
  if (rc) return rc;
  fsv_batch bb = *b;
  bb.last_token = nullptr;
  bb.draft_tokens = nullptr;
  if ((rc = fsv_launch_build_rows(c, &bb, M, s))) return rc;
  return (c->d.dtype == FSV_F32) ? fsv_f32_attention(c, layer, q, b, M, out, s)
                                 : fsv_bf16_attention(c, layer, q, b, &pl, M, out, s);
}

int fsv_profile_enable(fsv_ctx *c, uint32_t class_mask) {
  if (!c) return FSV_E_INVALID_ARG;
  c->prof_mask = class_mask;
  for (int &n : c->prof_seen) n = 0;
  return FSV_OK;
}

int fsv_profile_sample(fsv_ctx *c, int32_t every_n) {
  if (!c || every_n < 1) return FSV_E_INVALID_ARG;
  c->prof_every = every_n;
  return FSV_OK;
}

int fsv_profile_read(fsv_ctx *c, fsv_kernel_time *out, int32_t cap) {
  if (!c || !out || cap <= 0) return FSV_E_INVALID_ARG;
  fsv_kernel_time acc[FSV_K_COUNT];
  for (int i = 0; i < FSV_K_COUNT; ++i) acc[i] = fsv_kernel_time{i, 0, 0.0, 0.0};
  for (auto &r : c->prof) {
    float ms = 0.f;
    if (hipEventSynchronize(r.e1) == hipSuccess && hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
      acc[r.cls].launches += 1;
      acc[r.cls].total_ms += ms;
      acc[r.cls].bytes += r.bytes;
    }
    c->prof_pool.push_back(r.e0);   // kept for the records to come
    c->prof_pool.push_back(r.e1);
  }
  c->prof.clear();
  int n = 0;
  for (int i = 0; i < FSV_K_COUNT && n < cap; ++i)
    if (acc[i].launches > 0) out[n++] = acc[i];
  return n;
}

}  // extern "C"
