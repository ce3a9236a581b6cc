// Vocabulary-wide softmax statistics, acceptance tests, residual / bonus token selection and KV
// rollback: the accept / reject part of Alg. 2 step 2 (greedy form as printed there; for
// temperature > 0 the speculative-sampling rule that keeps the output law equal to the target's,
// Sec. II and Regime B of Sec. V) and the rollback of Sec. IV-C.
//
// Three launches, all bound by streaming logits from HBM:
//   k_row_stats   grid (chunks, rows)      one pass over every logits row: per chunk (max, sum e^{(l-max)/T}, argmax)
//   k_accept_mass grid (slices, requests)  acceptance tests from gathered scalars, then one pass over the
//                                          single row the emitted token is drawn from (and its draft-law row)
//                                          producing the mass of every 2048-id sub-block
//   k_select      grid (requests)          locate the sub-block and the id by inverse CDF, emit flags, roll back
// Every floating-point sum is taken in a fixed order (no atomics), so results are reproducible.
#include <limits.h>
#include <math.h>

#include "fsv_internal.h"

namespace {

constexpr double kLog2e = 1.4426950408889634074;

// e^{d * k / log2e} for d <= 0 (k = log2(e) / T), product formed in fp64, 2^frac on the transcendental unit.
__device__ inline float exp_scaled(float d, double k) {
  double z = (double)d * k;
  if (!(z > -1000.0)) return 0.f;  // also catches -inf and NaN (all -inf chunk)
  double n = rint(z);
  float f = (float)(z - n);
  return ldexpf(__builtin_amdgcn_exp2f(f), (int)n);
}

template <typename LT>
struct loader;

template <>
struct loader<uint16_t> {  // bf16 bit patterns
  static __device__ inline void load8(const uint16_t *row, int i0, int V, bool vec, float fill, float (&v)[8]) {
    if (vec && i0 + 8 <= V) {
      uint4 raw = *reinterpret_cast<const uint4 *>(row + i0);
      uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[2 * j] = __uint_as_float(w[j] << 16);
        v[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (i0 + j < V) ? __uint_as_float((uint32_t)row[i0 + j] << 16) : fill;
    }
  }
};

template <>
struct loader<float> {
  static __device__ inline void load8(const float *row, int i0, int V, bool vec, float fill, float (&v)[8]) {
    if (vec && i0 + 8 <= V) {
      float4 a = *reinterpret_cast<const float4 *>(row + i0);
      float4 b = *reinterpret_cast<const float4 *>(row + i0 + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
      v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (i0 + j < V) ? row[i0 + j] : fill;
    }
  }
};

// Inclusive scan of one double per thread over a 256-thread block, fixed order.  s_w: 4 doubles of LDS.
__device__ inline double block_incl_scan(double v, double *s_w, double *total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    double t = __shfl_up(v, off, 64);
    if (lane >= off) v += t;
  }
  __syncthreads();  // protect s_w from a previous use
  if (lane == 63) s_w[w] = v;
  __syncthreads();
  double pre = 0.0, tot = 0.0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i < w) pre += s_w[i];
    tot += s_w[i];
  }
  if (total) *total = tot;
  return v + pre;
}

__global__ void k_build_rows(int B, int V, const int32_t *seq_lens, const int32_t *last_token, const int32_t *off,
                             const int32_t *draft, int32_t *row_req, int32_t *row_idx, int32_t *row_pos,
                             int32_t *row_tok) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int o = off[b], g = off[b + 1] - o, rs = o + b;
  int L = seq_lens ? seq_lens[b] : 0;
  for (int i = 0; i <= g; ++i) {
    row_req[rs + i] = b;
    row_idx[rs + i] = i;
    row_pos[rs + i] = L + i;
    if (row_tok) {
      int t = (i == 0) ? (last_token ? last_token[b] : 0) : (draft ? draft[o + i - 1] : 0);
      row_tok[rs + i] = min(max(t, 0), V - 1);
    }
  }
}

template <typename LT>
__global__ __launch_bounds__(256) void k_row_stats(const LT *__restrict__ logits, int V, int nc,
                                                   const int32_t *__restrict__ row_req,
                                                   const float *__restrict__ temperature, float *__restrict__ pmax,
                                                   double *__restrict__ psum, int32_t *__restrict__ parg, int vec) {
  const int c = blockIdx.x, r = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const LT *row = logits + (size_t)r * V;
  const float T = temperature[row_req[r]];
  float v[FSV_SPC][8];
  const int base = c * FSV_CHUNK + tid * 8;
#pragma unroll
  for (int s = 0; s < FSV_SPC; ++s) loader<LT>::load8(row, base + s * FSV_SBK, V, vec != 0, -INFINITY, v[s]);
  float mx = -INFINITY;
  int ai = INT_MAX;
#pragma unroll
  for (int s = 0; s < FSV_SPC; ++s)
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (v[s][j] > mx) { mx = v[s][j]; ai = base + s * FSV_SBK + j; }
  // block (max, lowest id attaining it)
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    float om = __shfl_xor(mx, off, 64);
    int oi = __shfl_xor(ai, off, 64);
    if (om > mx || (om == mx && oi < ai)) { mx = om; ai = oi; }
  }
  __shared__ float s_m[4];
  __shared__ int s_i[4];
  __shared__ double s_d[4];
  if (lane == 0) { s_m[w] = mx; s_i[w] = ai; }
  __syncthreads();
  mx = s_m[0]; ai = s_i[0];
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (s_m[i] > mx || (s_m[i] == mx && s_i[i] < ai)) { mx = s_m[i]; ai = s_i[i]; }
  double sum = 0.0;
  if (T > 0.f) {
    const double k = kLog2e / (double)T;
#pragma unroll
    for (int s = 0; s < FSV_SPC; ++s)
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += (double)exp_scaled(v[s][j] - mx, k);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) s_d[w] = sum;
    __syncthreads();
    sum = (s_d[0] + s_d[1]) + (s_d[2] + s_d[3]);
  }
  if (tid == 0) {
    pmax[(size_t)r * nc + c] = mx;
    psum[(size_t)r * nc + c] = sum;
    parg[(size_t)r * nc + c] = ai;
  }
}

// Combine the per-chunk statistics of one row in chunk order: row max, sum of e^{(l-max)/T}, argmax id.
__device__ inline void combine_row(const float *pmax, const double *psum, const int32_t *parg, int nc, double invT,
                                   double *m_out, double *S_out, int *arg_out) {
  float m = pmax[0];
  int a = parg[0];
  for (int c = 1; c < nc; ++c)
    if (pmax[c] > m) { m = pmax[c]; a = parg[c]; }   // strict: the earliest chunk wins ties
  double S = 0.0;
  if (invT > 0.0)
    for (int c = 0; c < nc; ++c) {
      double sc = (pmax[c] == m) ? 1.0 : exp(((double)pmax[c] - (double)m) * invT);
      S += psum[c] * sc;
    }
  *m_out = (double)m;
  *S_out = S;
  *arg_out = a;
}

#define FSV_MAX_GAMMA 16

template <typename LT>
__device__ inline double thread_masses(const LT *lrow, const float *qrow, int i0, int V, bool lvec, bool qvec,
                                       float m, double k, double invS, bool residual, double (&mass)[8]) {
  float lv[8], qv[8];
  loader<LT>::load8(lrow, i0, V, lvec, -INFINITY, lv);
  if (residual) loader<float>::load8(qrow, i0, V, qvec, 0.f, qv);
  double t = 0.0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    double p = (double)exp_scaled(lv[j] - m, k) * invS;
    if (residual) {
      p -= (double)qv[j];
      p = p > 0.0 ? p : 0.0;
    }
    mass[j] = p;
    t += p;
  }
  return t;
}

template <typename LT>
__global__ __launch_bounds__(256) void k_accept_mass(
    const LT *__restrict__ logits, int V, int nc, int nsb, const int32_t *__restrict__ off,
    const int32_t *__restrict__ draft, const float *__restrict__ q, const float *__restrict__ u_acc,
    const float *__restrict__ temperature, const float *__restrict__ pmax, const double *__restrict__ psum,
    const int32_t *__restrict__ parg, double *__restrict__ bsum, int32_t *__restrict__ tau_ws,
    double *__restrict__ rowstat, int32_t *__restrict__ accepted_len, int32_t *__restrict__ next_token,
    uint32_t *__restrict__ flags, int lvec, int qvec) {
  const int b = blockIdx.y, tid = threadIdx.x;
  const int o = off[b], gamma = min(off[b + 1] - o, FSV_MAX_GAMMA), rs = o + b;
  const float T = temperature[b];
  if (T <= 0.f) {  // greedy (Alg. 2): accept while the draft equals the argmax, emit the argmax
    if (blockIdx.x == 0 && tid == 0) {
      int tau = 0, am = 0;
      for (;;) {
        double m_, S_;
        combine_row(pmax + (size_t)(rs + tau) * nc, psum, parg + (size_t)(rs + tau) * nc, nc, 0.0, &m_, &S_, &am);
        if (tau < gamma && draft[o + tau] == am) ++tau; else break;
      }
      tau_ws[b] = tau;
      accepted_len[b] = tau;
      next_token[b] = am;
      flags[b] = 0u;
    }
    return;
  }
  const double invT = 1.0 / (double)T, k = kLog2e * invT;
  __shared__ double s_m[FSV_MAX_GAMMA + 1], s_S[FSV_MAX_GAMMA + 1];
  __shared__ int s_acc[FSV_MAX_GAMMA], s_near[FSV_MAX_GAMMA];
  __shared__ int s_tau;
  __shared__ double s_w[4];
  if (tid <= gamma) {
    const int r = rs + tid;
    double m, S;
    int am;
    combine_row(pmax + (size_t)r * nc, psum + (size_t)r * nc, parg + (size_t)r * nc, nc, invT, &m, &S, &am);
    s_m[tid] = m;
    s_S[tid] = S;
    if (tid < gamma) {  // row r scores draft tid+1
      int d = min(max(draft[o + tid], 0), V - 1);
      float lv;
      if constexpr (sizeof(LT) == 2) lv = __uint_as_float((uint32_t)logits[(size_t)r * V + d] << 16);
      else lv = logits[(size_t)r * V + d];
      double p = exp(((double)lv - m) * invT) / S;
      double qd = (double)q[(size_t)(o + tid) * V + d];
      double ratio = p / qd;
      double a = (ratio >= 1.0) ? 1.0 : ratio;
      if (!(a == a)) a = 0.0;
      double u = (double)u_acc[o + tid];
      s_acc[tid] = (u < a) ? 1 : 0;
      s_near[tid] = (fabs(u - a) < 1e-4) ? 1 : 0;
    }
  }
  __syncthreads();
  if (tid == 0) {
    int tau = 0;
    while (tau < gamma && s_acc[tau]) ++tau;
    s_tau = tau;
  }
  __syncthreads();
  const int tau = s_tau;
  const bool residual = tau < gamma;
  const double m = s_m[tau], invS = 1.0 / s_S[tau];
  if (blockIdx.x == 0 && tid == 0) {
    uint32_t f = residual ? 4u : 0u;
    for (int i = 0; i < gamma && i <= tau; ++i) f |= s_near[i] ? 1u : 0u;
    tau_ws[b] = tau;
    accepted_len[b] = tau;
    flags[b] = f;
    rowstat[2 * b] = m;
    rowstat[2 * b + 1] = invS;
  }
  const LT *lrow = logits + (size_t)(rs + tau) * V;
  const float *qrow = residual ? q + (size_t)(o + tau) * V : nullptr;
  for (int sb = blockIdx.x; sb < nsb; sb += gridDim.x) {
    double mass[8], tot;
    double t = thread_masses<LT>(lrow, qrow, sb * FSV_SBK + tid * 8, V, lvec != 0, qvec != 0, (float)m, k, invS,
                                 residual, mass);
    block_incl_scan(t, s_w, &tot);
    if (tid == 0) bsum[(size_t)b * nsb + sb] = tot;
  }
}

#define FSV_MAX_NSB 160

template <typename LT>
__global__ __launch_bounds__(256) void k_select(
    const LT *__restrict__ logits, int V, int nsb, const int32_t *__restrict__ off, const float *__restrict__ q,
    const float *__restrict__ u_smp, const float *__restrict__ temperature, const double *__restrict__ bsum,
    const int32_t *__restrict__ tau_ws, const double *__restrict__ rowstat, int32_t *__restrict__ next_token,
    uint32_t *__restrict__ flags, const int32_t *__restrict__ seq_lens, int32_t *__restrict__ new_seq_lens,
    int32_t *__restrict__ pages_released, int page_size, int lvec, int qvec) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int o = off[b], gamma = min(off[b + 1] - o, FSV_MAX_GAMMA), rs = o + b;
  const int tau = tau_ws[b];
  if (tid == 0 && seq_lens && new_seq_lens) {  // KV rollback: keep [0, L+1+tau)
    int L = seq_lens[b], keep = L + 1 + tau, written = L + 1 + (off[b + 1] - o);
    new_seq_lens[b] = keep;
    if (pages_released)
      pages_released[b] = (written + page_size - 1) / page_size - (keep + page_size - 1) / page_size;
  }
  const float T = temperature[b];
  if (T <= 0.f) return;
  __shared__ double s_sb[FSV_MAX_NSB];
  __shared__ double s_w[4];
  __shared__ double s_Z, s_lo;
  __shared__ int s_pick, s_first, s_lastpos;
  bool residual = tau < gamma;
  const double m = rowstat[2 * b], invS = rowstat[2 * b + 1];
  const double k = kLog2e / (double)T;
  const LT *lrow = logits + (size_t)(rs + tau) * V;
  const float *qrow = residual ? q + (size_t)(o + tau) * V : nullptr;
  for (int sb = tid; sb < nsb; sb += 256) s_sb[sb] = bsum[(size_t)b * nsb + sb];
  __syncthreads();
  if (tid == 0) {
    double Z = 0.0;
    for (int sb = 0; sb < nsb; ++sb) Z += s_sb[sb];
    s_Z = Z;
  }
  __syncthreads();
  if (residual && !(s_Z > 0.0)) {
    // p <= q everywhere after rounding: the residual carries no mass, draw from p itself
    __syncthreads();
    residual = false;
    qrow = nullptr;
    for (int sb = 0; sb < nsb; ++sb) {
      double mass[8], tot;
      double t = thread_masses<LT>(lrow, qrow, sb * FSV_SBK + tid * 8, V, lvec != 0, qvec != 0, (float)m, k, invS,
                                   false, mass);
      block_incl_scan(t, s_w, &tot);
      if (tid == 0) s_sb[sb] = tot;
    }
    __syncthreads();
    if (tid == 0) {
      double Z = 0.0;
      for (int sb = 0; sb < nsb; ++sb) Z += s_sb[sb];
      s_Z = Z;
    }
    __syncthreads();
  }
  const double Z = s_Z, target = (double)u_smp[b] * Z;
  if (tid == 0) {
    double run = 0.0, lo = 0.0;
    int pick = -1, lastpos = 0;
    for (int sb = 0; sb < nsb; ++sb) {
      double prev = run;
      run += s_sb[sb];
      if (s_sb[sb] > 0.0) lastpos = sb;
      if (pick < 0 && run > target) { pick = sb; lo = prev; }
    }
    if (pick < 0) { pick = lastpos; lo = INFINITY; }  // rounding left no crossing: last id with mass
    s_pick = pick;
    s_lo = lo;
    s_first = INT_MAX;
    s_lastpos = -1;
  }
  __syncthreads();
  const int sb = s_pick;
  const double lo = s_lo;
  double mass[8];
  const int i0 = sb * FSV_SBK + tid * 8;
  double t = thread_masses<LT>(lrow, qrow, i0, V, lvec != 0, qvec != 0, (float)m, k, invS, residual, mass);
  double incl = block_incl_scan(t, s_w, nullptr);
  const bool crosses = (lo + incl) > target;  // false for every thread when lo == inf
  if (crosses) atomicMin(&s_first, tid);
  int lp = -1;
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (mass[j] > 0.0) lp = i0 + j;
  if (lp >= 0) atomicMax(&s_lastpos, lp);
  __syncthreads();
  if (s_first == INT_MAX) {
    if (tid == 0) {
      next_token[b] = max(s_lastpos, 0);
      flags[b] = (flags[b] & (residual ? ~0u : ~4u)) | 2u;
    }
    return;
  }
  if (tid == s_first) {
    double run = lo + (incl - t), margin = 0.0;
    int pick = -1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      double prev = run;
      run += mass[j];
      if (pick < 0 && run > target) {
        pick = i0 + j;
        margin = fmin(target - prev, run - target) / Z;
      }
    }
    if (pick < 0) { pick = lp >= 0 ? lp : i0; margin = 0.0; }
    next_token[b] = pick;
    uint32_t f = flags[b];
    if (!residual) f &= ~4u;
    if (margin < 1e-6) f |= 2u;
    flags[b] = f;
  }
}

__global__ void k_rollback(int B, const int32_t *seq_lens, const int32_t *off, const int32_t *accepted,
                           int32_t *new_seq_lens, int32_t *pages_released, int page_size) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int g = off[b + 1] - off[b], tau = min(max(accepted[b], 0), g);
  int L = seq_lens[b], keep = L + 1 + tau, written = L + 1 + g;
  new_seq_lens[b] = keep;
  if (pages_released) pages_released[b] = (written + page_size - 1) / page_size - (keep + page_size - 1) / page_size;
}

template <typename LT>
int launch_sampler_t(fsv_ctx *c, const LT *logits, const fsv_batch *b, const fsv_result *r, int M, bool with_rollback,
                     hipStream_t s) {
  const int V = c->d.vocab, B = b->batch, nc = c->nc, nsb = c->nsb;
  const int lalign = (sizeof(LT) == 2) ? 8 : 4;
  const int lvec = (V % lalign == 0 && ((uintptr_t)logits % 16) == 0) ? 1 : 0;
  const int qvec = (V % 4 == 0 && ((uintptr_t)b->draft_probs % 16) == 0) ? 1 : 0;
  int32_t *acc = r->accepted_len ? r->accepted_len : c->acc_scratch;
  {
    fsv_prof_scope ps(c, s, FSV_K_SAMPLE_STATS, (double)M * V * sizeof(LT));
    hipLaunchKernelGGL(k_row_stats<LT>, dim3(nc, M), dim3(256), 0, s, logits, V, nc, c->row_req, b->temperature,
                       c->pmax, c->psum, c->parg, lvec);
  }
  {
    fsv_prof_scope ps(c, s, FSV_K_SAMPLE_ACCEPT, (double)B * V * (sizeof(LT) + 4));
    int slices = nsb < 8 ? nsb : 8;
    hipLaunchKernelGGL(k_accept_mass<LT>, dim3(slices, B), dim3(256), 0, s, logits, V, nc, nsb, b->draft_offsets,
                       b->draft_tokens, b->draft_probs, b->u_accept, b->temperature, c->pmax, c->psum, c->parg,
                       c->bsum, c->tau_ws, c->rowstat, acc, r->next_token, r->flags, lvec, qvec);
  }
  {
    fsv_prof_scope ps(c, s, FSV_K_SAMPLE_SELECT, (double)B * FSV_SBK * (sizeof(LT) + 4));
    hipLaunchKernelGGL(k_select<LT>, dim3(B), dim3(256), 0, s, logits, V, nsb, b->draft_offsets, b->draft_probs,
                       b->u_sample, b->temperature, c->bsum, c->tau_ws, c->rowstat, r->next_token, r->flags,
                       with_rollback ? b->seq_lens : nullptr, with_rollback ? r->new_seq_lens : nullptr,
                       with_rollback ? r->pages_released : nullptr, c->d.page_size, lvec, qvec);
  }
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

}  // namespace

int fsv_launch_build_rows(fsv_ctx *c, const fsv_batch *b, int M, hipStream_t s) {
  (void)M;
  hipLaunchKernelGGL(k_build_rows, dim3(fsv_ceil_div(b->batch, 256)), dim3(256), 0, s, b->batch, c->d.vocab,
                     b->seq_lens, b->last_token, b->draft_offsets, b->draft_tokens, c->row_req, c->row_idx,
                     c->row_pos, c->row_tok);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_launch_sampler(fsv_ctx *c, const void *logits, int logits_dtype, const fsv_batch *b, const fsv_result *r,
                       int M, bool with_rollback, hipStream_t s) {
  if (logits_dtype == FSV_BF16)
    return launch_sampler_t<uint16_t>(c, (const uint16_t *)logits, b, r, M, with_rollback, s);
  return launch_sampler_t<float>(c, (const float *)logits, b, r, M, with_rollback, s);
}

int fsv_launch_rollback(fsv_ctx *c, const fsv_batch *b, const int32_t *accepted, const fsv_result *r, hipStream_t s) {
  hipLaunchKernelGGL(k_rollback, dim3(fsv_ceil_div(b->batch, 256)), dim3(256), 0, s, b->batch, b->seq_lens,
                     b->draft_offsets, accepted, r->new_seq_lens, r->pages_released, c->d.page_size);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}
