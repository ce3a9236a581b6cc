// Internal declarations shared by the translation units of libflexverify (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stdio.h>
#include <string>
#include <vector>

#include "flexverify.h"

#define FSV_WAVE 64

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;   // one MFMA A/B operand (8 bf16 per lane)
typedef __attribute__((ext_vector_type(16))) float f32x16_t;   // one 32x32 MFMA accumulator
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// ---- sampler geometry -------------------------------------------------------------------------
// A vocabulary row is cut into sub-blocks of SBK ids and chunks of SPC sub-blocks; the statistics
// kernel keeps one (max, sum, argmax) triple per chunk (one wave per chunk), the mass kernel one sum
// per sub-block (one wave per sub-block); the selection kernel scans one sub-block with 256 threads
// x 8 consecutive ids.
#define FSV_SBK 2048
#define FSV_SPC 4
#define FSV_CHUNK (FSV_SBK * FSV_SPC)

struct fsv_prof_rec {
  int cls;
  double bytes;
  hipEvent_t e0, e1;
};

struct fsv_layer_w {
  // fp32 path: plain copies [out][in]; bf16 path: re-tiled matrices, plain gains
  void *attn_norm = nullptr, *w_qkv = nullptr, *w_o = nullptr, *mlp_norm = nullptr, *w_gate_up = nullptr,
       *w_down = nullptr;
  // bf16 path: the matrices stored in fp16 carry a power of two; the projection's sums are multiplied by its inverse
  float os_qkv = 1.0f, os_o = 1.0f, os_gate_up = 1.0f;
};

struct fsv_ctx {
  fsv_model_desc d{};
  int max_rows = 0;
  int group = 1;          // query heads per KV head
  int nc = 0;             // vocabulary chunks per row
  int nsb = 0;            // vocabulary sub-blocks per row
  std::string err;

  // weights (library-owned)
  void *embed = nullptr, *final_norm = nullptr, *lm_head = nullptr;
  std::vector<fsv_layer_w> layers;
  float *inv_freq = nullptr;        // [head_dim/2] rotary frequencies (bf16 path; fp64 values)
  float *rope_tab = nullptr;        // [max_rows][head_dim/2][2] cos, sin of the rows of the current call

  // row map, built per call on the device
  int32_t *row_req = nullptr, *row_idx = nullptr, *row_pos = nullptr, *row_tok = nullptr;

  // sampler workspace
  float *pmax = nullptr;    // [max_rows][nc]
  double *psum = nullptr;   // [max_rows][nc]
  int32_t *parg = nullptr;  // [max_rows][nc]
  double *bsum = nullptr;   // [max_batch][nsb]
  int32_t *sel_ticket = nullptr;   // [max_batch] blocks of a request that have left their masses; zero between calls
  int32_t *acc_scratch = nullptr;  // [max_batch] accepted_len when the caller passes none
  // nucleus (top-p) selection, per logits row: digit-by-digit state, then the cut key, the kept mass, the near flag
  uint32_t *nuc_prefix = nullptr, *nuc_key = nullptr, *nuc_cabove = nullptr, *nuc_kkey = nullptr;
  unsigned long long *nuc_above = nullptr, *nuc_total = nullptr, *nuc_kmass = nullptr;
  double *nuc_S = nullptr;
  int32_t *nuc_near = nullptr, *nuc_done = nullptr;   // nuc_done[row]: the windowed pass has settled the row's cut

  // model workspace (both paths)
  float *x = nullptr;       // [rows_pad][d_model] residual stream, fp32
  float *logits = nullptr;  // [max_rows][vocab] fp32 when the caller passes no logits_out
  int strip_pad_bytes = 8192;   // bf16 path: padding between the weight strips of a re-tiled matrix (FSV_STRIP_PAD_KIB overrides)
  int gemm_ncw_force = 0;       // bf16 path: 2..4 = weight strips per GEMM block fixed (FSV_GEMM_NCW, a measurement and test knob)
  float os_lm_head = 1.0f;      // bf16 path: inverse of the power of two the fp16 LM-head matrix carries
  uint32_t *absmax = nullptr;   // bf16 path: one word for the largest weight magnitude of the matrix being converted
  void *buf_a = nullptr, *buf_qkv = nullptr, *buf_q = nullptr, *buf_att = nullptr, *buf_gu = nullptr,
       *buf_act = nullptr, *buf_part = nullptr;
  size_t part_bytes = 0;
  size_t q_plane_units = 0;     // 16-byte units of one plane of buf_q (bf16 path: plane 0 = hi, plane 1 = lo of the queries)
  void *attn_part = nullptr;    // per-part attention results (O, then (m, l)) of requests with several parts
  size_t attn_part_bytes = 0;
  int n_cus = 0;                // compute units of the device the context was created on
  int attn_wave_target = 0;     // waves the attention schedule aims at (resident waves of the device)
  int attn_wave_cap = 0;        // waves the partial buffers hold
  int attn_depth = 2;           // K/V tiles in flight per attention wave
  int attn_min_tpw = 5;         // fewest key tiles a part is given: with a single 2048-position request, parts of 5 tiles
                                // (13 per kv head, merged from one batch of loads) beat parts of 2 (33 per head) by 4 % of the call
  int attn_w2 = 26, attn_w3 = 36;  // cost of a key tile for a request with two / three query-row tiles, in 1/16 of one with one
  int32_t *attn_part_prefix = nullptr, *attn_part_map = nullptr;   // parts before each request; 8-int record per part

  // LoRA adapters of the evolved target (bf16 path): tables [layer < n_layers - 1][adapter][...], library-owned
  int lora_n = 0, lora_rank = 0;
  uint16_t *lora_aq = nullptr, *lora_bq = nullptr, *lora_ao = nullptr, *lora_bo = nullptr;
  float *lora_scale = nullptr;   // [lora_n]
  float *lora_t = nullptr;       // [max_rows][64] A_qkv x of the rows of the current call

  // head of the edge draft model (bf16 path): re-tiled W_1, W_2, W_v and the operands between them
  int draft_dh = 0, draft_dp = 0;
  void *draft_w1 = nullptr, *draft_w2 = nullptr, *draft_wv = nullptr, *draft_h1 = nullptr, *draft_h2 = nullptr;

  // profiling
  uint32_t prof_mask = 0;
  int prof_every = 1;                     // record every n-th launch of an enabled class (fsv_profile_sample)
  int prof_seen[16] = {0};                // launches of each class seen since profiling was enabled
  std::vector<fsv_prof_rec> prof;
  std::vector<hipEvent_t> prof_pool;      // events of records already read, reused by later records
};

#define FSV_FAIL(ctx, code, ...)                                   \
  do {                                                             \
    char _b[512];                                                  \
    snprintf(_b, sizeof _b, __VA_ARGS__);                          \
    if (ctx) (ctx)->err = _b;                                      \
    return (code);                                                 \
  } while (0)

#define FSV_HIP(ctx, call)                                                                  \
  do {                                                                                      \
    hipError_t _e = (call);                                                                 \
    if (_e != hipSuccess) FSV_FAIL(ctx, FSV_E_HIP, "%s: %s", #call, hipGetErrorString(_e)); \
  } while (0)

// scoped event pair around one kernel class (no-op unless profiling is on).  By default the pair is recorded on the
// stream before and after whatever is launched inside the scope; a launch that can carry its own start / stop events
// (hipExtLaunchKernelGGL) takes them with ext() instead, which times the kernel itself without the dispatch gaps.
struct fsv_prof_scope {
  fsv_ctx *c;
  hipStream_t s;
  fsv_prof_rec r{};
  bool on, external;
  fsv_prof_scope(fsv_ctx *ctx, hipStream_t st, int cls, double bytes, bool ext_mode = false)
      : c(ctx), s(st), on(ctx && ((ctx->prof_mask >> cls) & 1u)), external(ext_mode) {
    if (!on) return;
    if (c->prof_every > 1 && (c->prof_seen[cls]++ % c->prof_every) != 0) { on = false; return; }
    if (c->prof.size() >= 8192) { on = false; return; }
    r.cls = cls;
    r.bytes = bytes;
    auto get = [&](hipEvent_t *e) {
      if (!c->prof_pool.empty()) { *e = c->prof_pool.back(); c->prof_pool.pop_back(); return true; }
      return hipEventCreate(e) == hipSuccess;
    };
    if (!get(&r.e0)) { on = false; return; }
    if (!get(&r.e1)) { c->prof_pool.push_back(r.e0); on = false; return; }
    if (!external) (void)hipEventRecord(r.e0, s);
  }
  hipEvent_t start() const { return (on && external) ? r.e0 : nullptr; }
  hipEvent_t stop() const { return (on && external) ? r.e1 : nullptr; }
  ~fsv_prof_scope() {
    if (!on) return;
    if (!external) (void)hipEventRecord(r.e1, s);
    c->prof.push_back(r);
  }
};

static inline int fsv_ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- entry points of the other translation units ----------------------------------------------
// api.hip: CSR shape, capacity and pointer checks shared by the entry points.  Returns the number of rows or a status < 0.
int fsv_check_batch(fsv_ctx *c, const fsv_batch *b, bool need_kv, bool need_sampling);
// sampler.hip
int fsv_launch_build_rows(fsv_ctx *c, const fsv_batch *b, int M, hipStream_t s);
int fsv_launch_sampler(fsv_ctx *c, const void *logits, int logits_dtype, const fsv_batch *b, const fsv_result *r,
                       int M, bool with_rollback, hipStream_t s);
int fsv_launch_rollback(fsv_ctx *c, const fsv_batch *b, const int32_t *accepted, const fsv_result *r, hipStream_t s);
// path_f32.hip
int fsv_f32_create(fsv_ctx *c, const fsv_weights *w);
int fsv_f32_check(fsv_ctx *c, const fsv_batch *b);   // host only: what the launches of a forward / attention need
int fsv_f32_forward(fsv_ctx *c, const fsv_batch *b, int M, float *logits, hipStream_t s);
int fsv_f32_linear(fsv_ctx *c, int which, int layer, const void *x, int M, float *y, hipStream_t s);
int fsv_f32_attention(fsv_ctx *c, int layer, const void *q, const fsv_batch *b, int M, float *out, hipStream_t s);
int fsv_f32_kv_copy(fsv_ctx *c, void *k_pool, void *v_pool, int num_pages, const int32_t *pt_row, int pos0, int n,
                    void *k_lin, void *v_lin, bool import, hipStream_t s);
// attn_bf16.hip
struct fsv_attn_plan {
  int tpw = 0;          // target key tiles per part
  int waves = 0;        // parts x kv heads
  int rt = 1;           // query-row tiles of the widest request
  bool split = false;   // some request has several parts
  double kv_tokens = 0;
};
int fsv_bf16_attn_create(fsv_ctx *c);
int fsv_bf16_attn_plan_host(fsv_ctx *c, const fsv_batch *b, fsv_attn_plan *pl);          // host only; may fail
int fsv_bf16_attn_plan_launch(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan *pl, hipStream_t s);
int fsv_bf16_attn_launch(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan *pl, size_t layer_off, hipStream_t s);
// gemm_bf16.hip: y = x W^T through the weight-streaming kernel; epi 0 = fp32 split partials [splits][Mpad][N],
// 1 = SwiGLU to the bf16 operand order, 2 = fp32 rows [M][N]
int fsv_bf16_gemm_init(fsv_ctx *c);
int fsv_bf16_gemm(fsv_ctx *c, int cls, int epi, const void *Wp, const void *Ap, void *out, int N, int K, int NTpad, int M,
                  int splits, int KBo, int f16, float oscale, int ncw, hipStream_t st);
// path_bf16.hip
int fsv_bf16_create(fsv_ctx *c, const fsv_weights *w);
int fsv_bf16_forward(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan *pl, int M, float *logits, int draft, hipStream_t s);
int fsv_bf16_draft_attach(fsv_ctx *c, const fsv_draft_head *h);
int fsv_bf16_draft_probs(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan *pl, int M, int all_rows, float *q_out, float *logits,
                         hipStream_t s);
int fsv_bf16_linear(fsv_ctx *c, int which, int layer, const void *x, int M, float *y, hipStream_t s);
int fsv_bf16_lora_load(fsv_ctx *c, const fsv_lora *lo);
int fsv_bf16_attention(fsv_ctx *c, int layer, const void *q, const fsv_batch *b, const fsv_attn_plan *pl, int M, float *out,
                       hipStream_t s);
int fsv_bf16_kv_copy(fsv_ctx *c, void *k_pool, void *v_pool, int num_pages, const int32_t *pt_row, int pos0, int n,
                     void *k_lin, void *v_lin, bool import, int layers, hipStream_t s);
void fsv_free_weights(fsv_ctx *c);
