// FSV_F32 instantiation of the target forward (Alg. 2 step 2: the target model scores the pending
// token and the draft block on top of the restored KV session, Sec. IV-C).  This is the
// correctness configuration (a tiny fp32 decoder): plain fp32 kernels, one launch per operation,
// no matrix cores.  The bf16 path in path_bf16.hip is the one built for throughput.
#include <math.h>

#include "fsv_internal.h"

namespace {

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__global__ void k_embed(int d, const float *__restrict__ E, const int32_t *__restrict__ row_tok, float *__restrict__ x) {
  const int r = blockIdx.x;
  const float *src = E + (size_t)row_tok[r] * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) x[(size_t)r * d + k] = src[k];
}

// y = x * g / sqrt(mean(x^2) + eps), one block per row
__global__ __launch_bounds__(256) void k_rmsnorm(int d, float eps, const float *__restrict__ x,
                                                 const float *__restrict__ g, float *__restrict__ y) {
  const int r = blockIdx.x, tid = threadIdx.x;
  const float *xr = x + (size_t)r * d;
  float ss = 0.f;
  for (int k = tid; k < d; k += 256) ss += xr[k] * xr[k];
  ss = wave_sum(ss);
  __shared__ float s[4];
  if ((tid & 63) == 0) s[tid >> 6] = ss;
  __syncthreads();
  const float rinv = 1.0f / sqrtf(((s[0] + s[1]) + (s[2] + s[3])) / (float)d + eps);
  for (int k = tid; k < d; k += 256) y[(size_t)r * d + k] = xr[k] * rinv * g[k];
}

// y[m][n] (+)= sum_k a[m][k] * w[n][k]; one wave per output column, lanes stride over k
__global__ __launch_bounds__(256) void k_linear(int M, int N, int K, const float *__restrict__ a,
                                                const float *__restrict__ w, float *__restrict__ y, int accumulate) {
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (n >= N) return;
  const float *wr = w + (size_t)n * K;
  for (int m = 0; m < M; ++m) {
    const float *ar = a + (size_t)m * K;
    float acc = 0.f;
    for (int k = lane; k < K; k += 64) acc = fmaf(ar[k], wr[k], acc);
    acc = wave_sum(acc);
    if (lane == 0) {
      size_t o = (size_t)m * N + n;
      y[o] = accumulate ? y[o] + acc : acc;
    }
  }
}

// Rotate q and k by their position (half-split pairing), write q to qbuf and k, v into the paged pools.
__global__ void k_rope_append(int H, int Hkv, int hd, double theta, int num_pages, int max_pages,
                              const float *__restrict__ qkv, const int32_t *__restrict__ row_req,
                              const int32_t *__restrict__ row_pos, const int32_t *__restrict__ page_table,
                              float *__restrict__ qbuf, float *__restrict__ kpool, float *__restrict__ vpool,
                              size_t layer_off, int page_size) {
  const int r = blockIdx.x, half = hd / 2, heads = H + 2 * Hkv;
  const int pos = row_pos[r], b = row_req[r];
  const float *src = qkv + (size_t)r * heads * hd;
  // page ids live on the device: an id outside the pool is clamped into it (wrong data, never a wild write)
  const int page = min(max(page_table[(size_t)b * max_pages + pos / page_size], 0), num_pages - 1), slot = pos % page_size;
  for (int t = threadIdx.x; t < heads * half; t += blockDim.x) {
    const int h = t / half, i = t % half;
    const float a = src[h * hd + i], bb = src[h * hd + i + half];
    if (h < H + Hkv) {
      const double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
      const float cs = (float)cos(ang), sn = (float)sin(ang);
      const float ra = a * cs - bb * sn, rb = a * sn + bb * cs;
      if (h < H) {
        qbuf[(size_t)r * H * hd + h * hd + i] = ra;
        qbuf[(size_t)r * H * hd + h * hd + i + half] = rb;
      } else {
        float *dst = kpool + layer_off + (((size_t)page * Hkv + (h - H)) * page_size + slot) * hd;
        dst[i] = ra;
        dst[i + half] = rb;
      }
    } else {
      float *dst = vpool + layer_off + (((size_t)page * Hkv + (h - H - Hkv)) * page_size + slot) * hd;
      dst[i] = a;
      dst[i + half] = bb;
    }
  }
}

// One wave per (row, query head): scores into LDS, softmax, weighted sum of values.
__global__ __launch_bounds__(64) void k_attention(int H, int Hkv, int hd, int max_pages, int num_pages, int page_size,
                                                  const float *__restrict__ qbuf, const int32_t *__restrict__ row_req,
                                                  const int32_t *__restrict__ row_pos,
                                                  const int32_t *__restrict__ page_table,
                                                  const float *__restrict__ kpool, const float *__restrict__ vpool,
                                                  size_t layer_off, float *__restrict__ out) {
  extern __shared__ float sc[];
  const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  const int b = row_req[r], nkeys = row_pos[r] + 1, kvh = h / (H / Hkv);
  const float *q = qbuf + ((size_t)r * H + h) * hd;
  const int32_t *pt = page_table + (size_t)b * max_pages;
  const float scale = 1.0f / sqrtf((float)hd);
  float mx = -INFINITY;
  for (int j = lane; j < nkeys; j += 64) {
    const int page = min(max(pt[j / page_size], 0), num_pages - 1);
    const float *kr = kpool + layer_off + (((size_t)page * Hkv + kvh) * page_size + j % page_size) * hd;
    float s = 0.f;
    for (int e = 0; e < hd; ++e) s = fmaf(q[e], kr[e], s);
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float den = 0.f;
  for (int j = lane; j < nkeys; j += 64) {
    float p = expf(sc[j] - mx);
    sc[j] = p;
    den += p;
  }
  den = wave_sum(den);
  __syncthreads();
  for (int e = lane; e < hd; e += 64) {
    float acc = 0.f;
    for (int j = 0; j < nkeys; ++j) {
      const int page = min(max(pt[j / page_size], 0), num_pages - 1);
      const float *vr = vpool + layer_off + (((size_t)page * Hkv + kvh) * page_size + j % page_size) * hd;
      acc = fmaf(sc[j], vr[e], acc);
    }
    out[((size_t)r * H + h) * hd + e] = acc / den;
  }
}

__global__ void k_swiglu(int M, int F, const float *__restrict__ gu, float *__restrict__ act) {
  size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (size_t)M * F) return;
  size_t m = t / F, f = t % F;
  float g = gu[m * 2 * F + f], u = gu[m * 2 * F + F + f];
  act[t] = g / (1.0f + expf(-g)) * u;
}

__global__ void k_kv_copy(int Hkv, int hd, int page_size, int n_layers, int num_pages, const int32_t *__restrict__ pt,
                          int pos0, int n, float *__restrict__ kpool, float *__restrict__ vpool, float *__restrict__ klin,
                          float *__restrict__ vlin, int import) {
  // one block per (position, layer)
  const int p = blockIdx.x, l = blockIdx.y, pos = pos0 + p;
  const size_t layer_off = (size_t)l * num_pages * Hkv * page_size * hd;
  const int page = min(max(pt[pos / page_size], 0), num_pages - 1), slot = pos % page_size;
  for (int t = threadIdx.x; t < Hkv * hd; t += blockDim.x) {
    const int h = t / hd, e = t % hd;
    const size_t pi = layer_off + (((size_t)page * Hkv + h) * page_size + slot) * hd + e;
    const size_t li = (((size_t)l * n + p) * Hkv + h) * hd + e;
    if (import) { kpool[pi] = klin[li]; vpool[pi] = vlin[li]; }
    else { klin[li] = kpool[pi]; vlin[li] = vpool[pi]; }
  }
}

int dev_copy(fsv_ctx *c, void **dst, const void *src, size_t bytes) {
  FSV_HIP(c, hipMalloc(dst, bytes));
  FSV_HIP(c, hipMemcpy(*dst, src, bytes, hipMemcpyDeviceToDevice));
  return FSV_OK;
}

size_t layer_stride(const fsv_ctx *c, int num_pages) {
  return (size_t)num_pages * c->d.n_kv_heads * c->d.page_size * c->d.head_dim;
}

void launch_linear(int M, int N, int K, const float *a, const float *w, float *y, int acc, hipStream_t s) {
  hipLaunchKernelGGL(k_linear, dim3(fsv_ceil_div(N, 4)), dim3(256), 0, s, M, N, K, a, w, y, acc);
}

}  // namespace

int fsv_f32_create(fsv_ctx *c, const fsv_weights *w) {
  const fsv_model_desc &d = c->d;
  const size_t f = sizeof(float);
  const int qd = d.n_heads * d.head_dim, qkvd = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  int rc;
  if ((rc = dev_copy(c, &c->embed, w->embed, f * d.vocab * d.d_model))) return rc;
  if ((rc = dev_copy(c, &c->final_norm, w->final_norm, f * d.d_model))) return rc;
  if ((rc = dev_copy(c, &c->lm_head, w->lm_head, f * d.vocab * d.d_model))) return rc;
  c->layers.resize(d.n_layers);
  for (int l = 0; l < d.n_layers; ++l) {
    fsv_layer_w &L = c->layers[l];
    if ((rc = dev_copy(c, &L.attn_norm, w->attn_norm[l], f * d.d_model))) return rc;
    if ((rc = dev_copy(c, &L.w_qkv, w->w_qkv[l], f * qkvd * d.d_model))) return rc;
    if ((rc = dev_copy(c, &L.w_o, w->w_o[l], f * d.d_model * qd))) return rc;
    if ((rc = dev_copy(c, &L.mlp_norm, w->mlp_norm[l], f * d.d_model))) return rc;
    if ((rc = dev_copy(c, &L.w_gate_up, w->w_gate_up[l], f * 2 * d.d_ffn * d.d_model))) return rc;
    if ((rc = dev_copy(c, &L.w_down, w->w_down[l], f * d.d_model * d.d_ffn))) return rc;
  }
  const size_t R = c->max_rows;
  FSV_HIP(c, hipMalloc(&c->buf_a, f * R * d.d_model));
  FSV_HIP(c, hipMalloc(&c->buf_qkv, f * R * qkvd));
  FSV_HIP(c, hipMalloc(&c->buf_q, f * R * qd));
  FSV_HIP(c, hipMalloc(&c->buf_att, f * R * qd));
  FSV_HIP(c, hipMalloc(&c->buf_gu, f * R * 2 * d.d_ffn));
  FSV_HIP(c, hipMalloc(&c->buf_act, f * R * d.d_ffn));
  return FSV_OK;
}

static int max_keys_of(const fsv_batch *b) {
  int max_keys = 0;
  for (int i = 0; i < b->batch; ++i) {
    int g = b->draft_offsets_host[i + 1] - b->draft_offsets_host[i];
    max_keys = max(max_keys, b->seq_lens_host[i] + g + 1);
  }
  return max_keys;
}

int fsv_f32_check(fsv_ctx *c, const fsv_batch *b) {
  const int max_keys = max_keys_of(b);
  if (sizeof(float) * (size_t)max_keys > 64 * 1024)
    FSV_FAIL(c, FSV_E_UNSUPPORTED, "fp32 path: %d keys exceed the 16384 it keeps in LDS", max_keys);
  return FSV_OK;
}

int fsv_f32_forward(fsv_ctx *c, const fsv_batch *b, int M, float *logits, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  const int qd = d.n_heads * d.head_dim, qkvd = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  float *x = c->x, *a = (float *)c->buf_a, *qkv = (float *)c->buf_qkv, *qb = (float *)c->buf_q;
  float *att = (float *)c->buf_att, *gu = (float *)c->buf_gu, *act = (float *)c->buf_act;
  const size_t lds = sizeof(float) * max_keys_of(b);   // fsv_f32_check has bounded it
  hipLaunchKernelGGL(k_embed, dim3(M), dim3(256), 0, s, d.d_model, (const float *)c->embed, c->row_tok, x);
  for (int l = 0; l < d.n_layers; ++l) {
    const fsv_layer_w &L = c->layers[l];
    const size_t lo = (size_t)l * layer_stride(c, b->num_pages);
    hipLaunchKernelGGL(k_rmsnorm, dim3(M), dim3(256), 0, s, d.d_model, d.rms_eps, x, (const float *)L.attn_norm, a);
    launch_linear(M, qkvd, d.d_model, a, (const float *)L.w_qkv, qkv, 0, s);
    hipLaunchKernelGGL(k_rope_append, dim3(M), dim3(256), 0, s, d.n_heads, d.n_kv_heads, d.head_dim,
                       (double)d.rope_theta, b->num_pages, d.max_pages_per_req, qkv, c->row_req, c->row_pos,
                       b->page_table, qb, (float *)b->k_pool, (float *)b->v_pool, lo, d.page_size);
    hipLaunchKernelGGL(k_attention, dim3(M, d.n_heads), dim3(64), lds, s, d.n_heads, d.n_kv_heads, d.head_dim,
                       d.max_pages_per_req, b->num_pages, d.page_size, qb, c->row_req, c->row_pos, b->page_table,
                       (const float *)b->k_pool, (const float *)b->v_pool, lo, att);
    launch_linear(M, d.d_model, qd, att, (const float *)L.w_o, x, 1, s);
    hipLaunchKernelGGL(k_rmsnorm, dim3(M), dim3(256), 0, s, d.d_model, d.rms_eps, x, (const float *)L.mlp_norm, a);
    launch_linear(M, 2 * d.d_ffn, d.d_model, a, (const float *)L.w_gate_up, gu, 0, s);
    hipLaunchKernelGGL(k_swiglu, dim3(fsv_ceil_div(M * d.d_ffn, 256)), dim3(256), 0, s, M, d.d_ffn, gu, act);
    launch_linear(M, d.d_model, d.d_ffn, act, (const float *)L.w_down, x, 1, s);
  }
  hipLaunchKernelGGL(k_rmsnorm, dim3(M), dim3(256), 0, s, d.d_model, d.rms_eps, x, (const float *)c->final_norm, a);
  launch_linear(M, d.vocab, d.d_model, a, (const float *)c->lm_head, logits, 0, s);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_f32_linear(fsv_ctx *c, int which, int layer, const void *x, int M, float *y, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  const int qd = d.n_heads * d.head_dim, qkvd = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  const float *w;
  int N, K;
  switch (which) {
    case FSV_W_QKV: w = (const float *)c->layers[layer].w_qkv; N = qkvd; K = d.d_model; break;
    case FSV_W_O: w = (const float *)c->layers[layer].w_o; N = d.d_model; K = qd; break;
    case FSV_W_GATE_UP: w = (const float *)c->layers[layer].w_gate_up; N = 2 * d.d_ffn; K = d.d_model; break;
    case FSV_W_DOWN: w = (const float *)c->layers[layer].w_down; N = d.d_model; K = d.d_ffn; break;
    default: w = (const float *)c->lm_head; N = d.vocab; K = d.d_model; break;
  }
  launch_linear(M, N, K, (const float *)x, w, y, 0, s);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_f32_attention(fsv_ctx *c, int layer, const void *q, const fsv_batch *b, int M, float *out, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  const size_t lds = sizeof(float) * max_keys_of(b);   // fsv_f32_check has bounded it
  const size_t lo = (size_t)layer * layer_stride(c, b->num_pages);
  hipLaunchKernelGGL(k_attention, dim3(M, d.n_heads), dim3(64), lds, s, d.n_heads, d.n_kv_heads, d.head_dim,
                     d.max_pages_per_req, b->num_pages, d.page_size, (const float *)q, c->row_req, c->row_pos, b->page_table,
                     (const float *)b->k_pool, (const float *)b->v_pool, lo, out);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_f32_kv_copy(fsv_ctx *c, void *k_pool, void *v_pool, int num_pages, const int32_t *pt_row, int pos0, int n,
                    void *k_lin, void *v_lin, bool import, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  hipLaunchKernelGGL(k_kv_copy, dim3(n, d.n_layers), dim3(256), 0, s, d.n_kv_heads, d.head_dim, d.page_size,
                     d.n_layers, num_pages, pt_row, pos0, n, (float *)k_pool, (float *)v_pool, (float *)k_lin,
                     (float *)v_lin, import ? 1 : 0);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}
