// FSV_BF16 instantiation of the target forward (Alg. 2 step 2: the target model scores the pending
// token and the received draft block on top of the user's restored KV session; Sec. IV-C: KV pairs
// are computed only for the new tokens).  Written for gfx950: 64-wide waves, 16-bit matrix cores
// (v_mfma_f32_32x32x16_bf16 / _f16: the activations that are bounded by construction, i.e. the output of
// a normalisation and of the attention, travel in fp16, everything else in bf16), weights and KV pages stored in the order the matrix cores consume
// them so that every global load of the two dominant streams (weights, KV) is one contiguous
// 1 KiB request per wave and needs no LDS round trip.
//
// Operand order ("tile" = what one wave feeds to one MFMA as the 32-row operand):
//   element (row r, k) of a [rows][K] matrix lives at ((r/32 * K/16 + k/16) * 64 + r%32 + 32*((k%16)/8)) * 8 + k%8.
// Weights use it with r = output feature (re-tiled once at create), activations with r = batch row.
// The product is formed transposed, D[n][m] = sum_k W[n][k] X[m][k], so each lane ends up with four
// consecutive output features of one row.
//
// This file: weight re-tiling, the residual / RMSNorm kernel (fused with the split-K reduction), RoPE + KV append,
// session import / export, and the launch order of one forward.  The GEMM kernel is in gemm_bf16.hip, the attention
// kernels in attn_bf16.hip (both are built with their own compiler flags).
#include <math.h>
#include <stdlib.h>

#include "bf16_common.h"

using namespace fsv_bf16;

namespace {

// ---------------------------------------------------------------------------------------------
// one-time weight re-tiling
// ---------------------------------------------------------------------------------------------
// mode 0: packed row n' = source row n'.  mode 1 (gate|up): every 32-row tile holds 16 hidden features,
// gate and up interleaved in groups of 8 (rows 0-7 gate f0-7, 8-15 up f0-7, 16-23 gate f8-15, 24-31 up f8-15),
// so that after the MFMA one lane owns gate and up of the same four features.
__global__ void k_pack_w(const uint16_t *__restrict__ W, int N, int K, int NTpad, int mode, int F, uint4 *__restrict__ out,
                         int f16, float wscale, int strip_units) {
  // strip_units: 16-byte units from one strip of 32 features to the next (K / 16 * 64 of operands, then padding)
  const size_t unit = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int KB = K / 16;
  if (unit >= (size_t)NTpad * strip_units) return;
  const int nt = (int)(unit / strip_units), rem = (int)(unit % strip_units);
  if (rem >= KB * 64) {   // padding between strips
    out[unit] = make_uint4(0, 0, 0, 0);
    return;
  }
  const int lane = rem & 63, kb = rem >> 6;
  const int np = nt * 32 + (lane & 31), k0 = kb * 16 + 8 * (lane >> 5);
  int src = -1;
  if (mode == 0) {
    if (np < N) src = np;
  } else {
    const int nl = np & 31, f = 16 * (np >> 5) + 8 * (nl >> 4) + (nl & 7), up = (nl >> 3) & 1;
    if (f < F) src = up * F + f;
  }
  uint4 v = make_uint4(0, 0, 0, 0);
  if (src >= 0) v = *reinterpret_cast<const uint4 *>(W + (size_t)src * K + k0);
  if (f16) {   // bf16 -> fp16 times a power of two (see pack_weight)
    uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      w4[j] = f2h2(__uint_as_float(w4[j] << 16) * wscale, __uint_as_float(w4[j] & 0xffff0000u) * wscale);
    v = make_uint4(w4[0], w4[1], w4[2], w4[3]);
  }
  out[unit] = v;
}

// largest magnitude (as bf16 bits without the sign) of n bf16 values, n a multiple of 8; *out starts at zero
__global__ void k_absmax_bf16(const uint4 *__restrict__ W, size_t n8, uint32_t *__restrict__ out) {
  uint32_t m = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (size_t)gridDim.x * blockDim.x) {
    const uint4 v = W[i];
    const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) m = max(m, max(w4[j] & 0x7fffu, (w4[j] >> 16) & 0x7fffu));
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
  if ((threadIdx.x & 63) == 0 && m) atomicMax(out, m);
}

// row-major bf16 [M][K] -> operand order (f16: converted to fp16, the operand type of that projection), zero rows up to Mpad
__global__ void k_pack_act(const uint16_t *__restrict__ x, int M, int Mpad, int K, uint4 *__restrict__ out, int f16) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int K8 = K / 8;
  if (t >= (size_t)Mpad * K8) return;
  const int m = t / K8, k0 = (t % K8) * 8;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (m < M) v = *reinterpret_cast<const uint4 *>(x + (size_t)m * K + k0);
  if (f16) {
    uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) w4[j] = f2h2(__uint_as_float(w4[j] << 16), __uint_as_float(w4[j] & 0xffff0000u));
    v = make_uint4(w4[0], w4[1], w4[2], w4[3]);
  }
  out[tile_unit(m, k0, K / 16)] = v;
}

// operand order fp16 (the attention output) -> row-major fp32 [M][K]
__global__ void k_unpack_act(const uint4 *__restrict__ in, int M, int K, float *__restrict__ y) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int K8 = K / 8;
  if (t >= (size_t)M * K8) return;
  const int m = t / K8, k0 = (t % K8) * 8;
  uint4 v = in[tile_unit(m, k0, K / 16)];
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
  float *dst = y + (size_t)m * K + k0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    dst[2 * j] = h2f((uint16_t)(w[j] & 0xffffu));
    dst[2 * j + 1] = h2f((uint16_t)(w[j] >> 16));
  }
}

// y[m][src(n')] = sum_s part[s][m][n']   (fixed order over s)
__global__ void k_reduce_part(const float *__restrict__ part, int S, int Mpad, int M, int N, int mode, int F,
                              float *__restrict__ y) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (size_t)M * N) return;
  const int m = t / N, np = t % N;
  float acc = 0.f;
  for (int s = 0; s < S; ++s) acc += part[((size_t)s * Mpad + m) * N + np];
  int dst = np;
  if (mode == 1) {
    const int nl = np & 31, f = 16 * (np >> 5) + 8 * (nl >> 4) + (nl & 7), up = (nl >> 3) & 1;
    dst = up * F + f;
  }
  y[(size_t)m * N + dst] = acc;
}

enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_F32 = 2 };  // epilogues of fsv_bf16_gemm

// ---------------------------------------------------------------------------------------------
// residual stream: x (+)= sum of split partials (or embedding), RMSNorm, emit the next GEMM's operand
// ---------------------------------------------------------------------------------------------
// LoRA adapters of the evolved target (Sec. IV-A: frozen backbone plus adapters; the last block and the LM head carry
// none): y = W x + s B (A x) on the fused q|k|v projection and on the output projection.  The low-rank side never goes
// through the big GEMM: "shrink" (t = A x, rank numbers per row) and "expand" (+= s B t) run inside the per-row kernels
// that produce and consume the projection's operands, where a row has one adapter and its matrices are read
// contiguously; the products are fp32 and never rounded.
struct lora_args {
  const int32_t *row_req = nullptr, *adapter = nullptr;   // adapter id per request (outside [0, n): none)
  int n = 0, rank = 0;
  const float *scale = nullptr;                           // [n]
  const uint16_t *aq = nullptr;                           // LQ: A_qkv of the layer whose projection follows, [n][rank][d]
  float *t_out = nullptr;                                 // LQ: [rows][64] A_qkv x of every row
  const uint16_t *ao = nullptr, *bo = nullptr;            // LO: A_o [n][rank][qd], B_o [n][d][rank] of this layer
  const uint4 *att = nullptr;                             // LO: the attention output (operand order), qd wide
  int qd = 0;
};

// t[j] = sum_k A[j][k] x[k] over the block: every thread contributes the slices it holds, eight ranks at a time; the
// per-wave sums meet in LDS and are added in wave order.  s_part: [16 waves][64].
template <typename F>
__device__ inline void lora_shrink(const uint16_t *__restrict__ A, int rank, int K, int tid, int nthreads, F &&slice,
                                   float (*s_part)[64], float *s_t) {
  const int w = tid >> 6, nw = nthreads >> 6;
  for (int j0 = 0; j0 < rank; j0 += 8) {
    float part[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int k0 = tid * 8; k0 < K; k0 += nthreads * 8) {
      float xv[8];
      slice(k0, xv);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(A + (size_t)(j0 + j) * K + k0);
        const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int u = 0; u < 4; ++u)
          part[j] += __uint_as_float(w4[u] << 16) * xv[2 * u] + __uint_as_float(w4[u] & 0xffff0000u) * xv[2 * u + 1];
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float t = wave_sum(part[j]);
      if ((tid & 63) == 0) s_part[w][j0 + j] = t;
    }
  }
  __syncthreads();
  if (tid < rank) {
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += s_part[i][tid];  // fixed order
    s_t[tid] = t;
  }
  __syncthreads();
}

template <int EMBED, int LQ, int LO, int RAW = 0>
__global__ __launch_bounds__(1024) void k_resid_norm(int M, int d, float eps, const int32_t *__restrict__ row_tok,
                                                     const uint16_t *__restrict__ E, const float *__restrict__ part,
                                                     int S, int Mpad, float *__restrict__ x,
                                                     const uint16_t *__restrict__ gain, uint4 *__restrict__ a_out,
                                                     lora_args lo) {
  const int r = blockIdx.x, tid = threadIdx.x, KB = d / 16, stride = blockDim.x * 8, nw = blockDim.x >> 6;
  if (r >= M) {
    for (int k0 = tid * 8; k0 < d; k0 += stride) a_out[tile_unit(r, k0, KB)] = make_uint4(0, 0, 0, 0);
    return;
  }
  float *xr = x + (size_t)r * d;
  __shared__ float s_ss[16];
  __shared__ float s_part[(LQ || LO) ? 16 : 1][64], s_t[64];
  int ad = -1;
  if (LQ || LO) {
    ad = lo.adapter[lo.row_req[r]];
    if (ad < 0 || ad >= lo.n) ad = -1;   // block-uniform: the row's request has no adapter
  }
  // sum of the split slices (in slice order) on top of the residual, or the embedding row
  auto gather = [&](int k0, float(&v)[8]) {
    if (EMBED) {
      uint4 raw = *reinterpret_cast<const uint4 *>(E + (size_t)row_tok[r] * d + k0);
      uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[2 * j] = __uint_as_float(w4[j] << 16);
        v[2 * j + 1] = __uint_as_float(w4[j] & 0xffff0000u);
      }
    } else {
      float4 a = *reinterpret_cast<const float4 *>(xr + k0), b = *reinterpret_cast<const float4 *>(xr + k0 + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
      const float *p = part + (size_t)r * d + k0;
      const size_t sstr = (size_t)Mpad * d;
      int s = 0;
      for (; s + 4 <= S; s += 4) {  // four slices in flight; summed in slice order
        float4 pa[4], pb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          pa[u] = *reinterpret_cast<const float4 *>(p + (s + u) * sstr);
          pb[u] = *reinterpret_cast<const float4 *>(p + (s + u) * sstr + 4);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          v[0] += pa[u].x; v[1] += pa[u].y; v[2] += pa[u].z; v[3] += pa[u].w;
          v[4] += pb[u].x; v[5] += pb[u].y; v[6] += pb[u].z; v[7] += pb[u].w;
        }
      }
      for (; s < S; ++s) {
        float4 pa = *reinterpret_cast<const float4 *>(p + s * sstr), pb = *reinterpret_cast<const float4 *>(p + s * sstr + 4);
        v[0] += pa.x; v[1] += pa.y; v[2] += pa.z; v[3] += pa.w; v[4] += pb.x; v[5] += pb.y; v[6] += pb.z; v[7] += pb.w;
      }
    }
  };
  auto pack = [&](const float(&v)[8], uint4 graw, float rinv) {
    uint32_t g4[4] = {graw.x, graw.y, graw.z, graw.w};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float g0 = __uint_as_float(g4[j] << 16), g1 = __uint_as_float(g4[j] & 0xffff0000u);
      // a normalised activation is at most sqrt(d) times its gain: fp16; the raw residual stream has no bound: bf16
      if (RAW) o[j] = (uint32_t)f2bf(v[2 * j] * rinv * g0) | ((uint32_t)f2bf(v[2 * j + 1] * rinv * g1) << 16);
      else o[j] = f2h2(v[2 * j] * rinv * g0, v[2 * j + 1] * rinv * g1);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
  };
  if (stride >= d) {
    // At most one 8-wide slice per thread (every shape up to d = 8192): the slice stays in registers across the
    // block-wide sum of squares, and the gains are fetched together with the inputs, so the kernel is one round of
    // loads, one reduction and one round of stores.  Threads beyond the row width only take part in the reductions.
    const int k0 = tid * 8;
    const bool live = k0 < d;
    uint4 graw = make_uint4(0, 0, 0, 0);
    float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (live) {
      graw = *reinterpret_cast<const uint4 *>(gain + k0);
      gather(k0, v);
    }
    if (LO && ad >= 0) {
      // output projection of an adapted request: v += s B_o (A_o att), att = this row of the attention output
      const int KBa = lo.qd / 16;
      auto att_slice = [&](int kk, float(&xv)[8]) {
        const uint4 raw = lo.att[tile_unit(r, kk, KBa)];   // fp16
        const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          xv[2 * u] = h2f((uint16_t)(w4[u] & 0xffffu));
          xv[2 * u + 1] = h2f((uint16_t)(w4[u] >> 16));
        }
      };
      lora_shrink(lo.ao + (size_t)ad * lo.rank * lo.qd, lo.rank, lo.qd, tid, (int)blockDim.x, att_slice, s_part, s_t);
      if (live) {
        const float sc = lo.scale[ad];
        const uint16_t *B = lo.bo + ((size_t)ad * d + k0) * lo.rank;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          float acc = 0.f;
          for (int j = 0; j < lo.rank; j += 8) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(B + (size_t)i * lo.rank + j);
            const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int u = 0; u < 4; ++u)
              acc += __uint_as_float(w4[u] << 16) * s_t[j + 2 * u] + __uint_as_float(w4[u] & 0xffff0000u) * s_t[j + 2 * u + 1];
          }
          v[i] += sc * acc;
        }
      }
    }
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
    ss = wave_sum(ss);
    if ((tid & 63) == 0) s_ss[tid >> 6] = ss;
    if (live) {
      *reinterpret_cast<float4 *>(xr + k0) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4 *>(xr + k0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
    __syncthreads();
    float tot = 0.f;
    for (int i = 0; i < nw; ++i) tot += s_ss[i];  // fixed order
    // RAW: the operand is the residual stream itself (input of the draft model's head), no normalisation and no gains
    const uint4 packed = RAW ? pack(v, make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u), 1.0f)
                             : pack(v, graw, 1.0f / sqrtf(tot / (float)d + eps));
    if (live) a_out[tile_unit(r, k0, KB)] = packed;
    if (LQ && ad >= 0) {
      // the q|k|v projection that follows is adapted for this row: leave t = A_qkv a (a = the operand just stored)
      auto own_slice = [&](int kk, float(&xv)[8]) {   // kk == k0: one slice per thread
        const uint32_t w4[4] = {packed.x, packed.y, packed.z, packed.w};   // fp16 (never the RAW form)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          xv[2 * u] = h2f((uint16_t)(w4[u] & 0xffffu));
          xv[2 * u + 1] = h2f((uint16_t)(w4[u] >> 16));
        }
      };
      lora_shrink(lo.aq + (size_t)ad * lo.rank * d, lo.rank, d, tid, (int)blockDim.x, own_slice, s_part, s_t);
      if (tid < lo.rank) lo.t_out[(size_t)r * 64 + tid] = s_t[tid];
    }
    return;
  }
  // rows wider than 8192 (no adapters there: fsv_lora_load refuses such a model)
  float ss = 0.f;
  for (int k0 = tid * 8; k0 < d; k0 += stride) {
    float v[8];
    gather(k0, v);
    *reinterpret_cast<float4 *>(xr + k0) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(xr + k0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
#pragma unroll
    for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) s_ss[tid >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
  for (int i = 0; i < nw; ++i) tot += s_ss[i];  // fixed order
  const float rinv = 1.0f / sqrtf(tot / (float)d + eps);
  for (int k0 = tid * 8; k0 < d; k0 += stride) {  // each thread re-reads exactly what it wrote
    float4 a = *reinterpret_cast<const float4 *>(xr + k0), b = *reinterpret_cast<const float4 *>(xr + k0 + 4);
    float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    a_out[tile_unit(r, k0, KB)] = pack(v, *reinterpret_cast<const uint4 *>(gain + k0), rinv);
  }
}

// ---------------------------------------------------------------------------------------------
// KV page tiles (16 positions x head_dim per kv head)
// ---------------------------------------------------------------------------------------------
__global__ void k_kv_copy(int Hkv, int hd, int num_pages, const int32_t *__restrict__ pt, int pos0, int n,
                          uint16_t *__restrict__ kpool, uint16_t *__restrict__ vpool, uint16_t *__restrict__ klin,
                          uint16_t *__restrict__ vlin, int import) {
  const int p = blockIdx.x, l = blockIdx.y, pos = pos0 + p;
  const int page = min(max(pt[pos >> 4], 0), num_pages - 1), t = pos & 15;
  for (int i = threadIdx.x; i < Hkv * hd; i += blockDim.x) {
    const int hh = i / hd, e = i % hd;
    const size_t tile = (((size_t)l * num_pages + page) * Hkv + hh) * (16 * hd);
    const size_t li = (((size_t)l * n + p) * Hkv + hh) * hd + e;
    if (import) {
      kpool[tile + k_tile_off(t, e)] = klin[li];
      vpool[tile + v_tile_off(t, e)] = vlin[li];
    } else {
      klin[li] = kpool[tile + k_tile_off(t, e)];
      vlin[li] = vpool[tile + v_tile_off(t, e)];
    }
  }
}

// ---------------------------------------------------------------------------------------------
// rotary embedding + KV append; consumes the split partials of the QKV projection
// ---------------------------------------------------------------------------------------------
// cos / sin of every row's rotation angles, once per call (the angles depend on the row's position only, not on the
// layer): tab[(row * hd/2 + i) * 2 + {0, 1}].  The angle is formed and reduced in fp64.
__global__ void k_rope_table(int M, int half, const double *__restrict__ inv_freq, const int32_t *__restrict__ row_pos,
                             float *__restrict__ tab) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= M * half) return;
  double sn, cs;
  sincos((double)row_pos[t / half] * inv_freq[t % half], &sn, &cs);
  reinterpret_cast<float2 *>(tab)[t] = make_float2((float)cs, (float)sn);
}

template <int LORA>
__global__ __launch_bounds__(256) void k_rope_append(int H, int Hkv, int hd, const float *__restrict__ rope_tab,
                                                     const float *__restrict__ part, int S, int Mpad,
                                                     const int32_t *__restrict__ row_req,
                                                     const int32_t *__restrict__ row_idx,
                                                     const int32_t *__restrict__ row_pos,
                                                     const int32_t *__restrict__ page_table, int max_pages,
                                                     int num_pages, size_t layer_off, uint16_t *__restrict__ qp,
                                                     size_t q_plane, uint16_t *__restrict__ kpool,
                                                     uint16_t *__restrict__ vpool, const int32_t *__restrict__ adapter,
                                                     int n_adapters, int rank, const float *__restrict__ lscale,
                                                     const uint16_t *__restrict__ bq, const float *__restrict__ tq) {
  // grid = (rows, blocks of 256 threads over the heads of the q|k|v projection); a thread owns four consecutive
  // rotation pairs (i .. i+3, i+half .. i+half+3) of one head.  The partial sums and the rotation table only need the
  // row index, so their loads are issued first, next to the row's request / position / page lookups.
  const int r = blockIdx.x, half = hd / 2, qpt = half / 4, heads = H + 2 * Hkv, qkvd = heads * hd, group = H / Hkv;
  const int item = blockIdx.y * blockDim.x + threadIdx.x;
  if (item >= heads * qpt) return;
  const int hh = item / qpt, i = (item % qpt) * 4;
  const float *p = part + (size_t)r * qkvd + hh * hd + i;
  const size_t sstr = (size_t)Mpad * qkvd;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f), c = a;
  {
    int s = 0;
    for (; s + 4 <= S; s += 4) {  // four slices in flight; summed in slice order
      float4 pa[4], pc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        pa[u] = *reinterpret_cast<const float4 *>(p + (s + u) * sstr);
        pc[u] = *reinterpret_cast<const float4 *>(p + (s + u) * sstr + half);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        a.x += pa[u].x; a.y += pa[u].y; a.z += pa[u].z; a.w += pa[u].w;
        c.x += pc[u].x; c.y += pc[u].y; c.z += pc[u].z; c.w += pc[u].w;
      }
    }
    for (; s < S; ++s) {
      const float4 pa = *reinterpret_cast<const float4 *>(p + s * sstr), pc = *reinterpret_cast<const float4 *>(p + s * sstr + half);
      a.x += pa.x; a.y += pa.y; a.z += pa.z; a.w += pa.w;
      c.x += pc.x; c.y += pc.y; c.z += pc.z; c.w += pc.w;
    }
  }
  const int b = row_req[r], i_row = row_idx[r], pos = row_pos[r];
  float av[4] = {a.x, a.y, a.z, a.w}, cv[4] = {c.x, c.y, c.z, c.w};
  if (LORA) {
    // adapted request: qkv += s B_qkv t, t = A_qkv a left by the norm kernel (before the rotation: it is part of the
    // projection); bq: [n][qkvd][rank], tq: [rows][64]
    const int ad = adapter[b];
    if (ad >= 0 && ad < n_adapters) {
      const float sc = lscale[ad];
      const uint16_t *B = bq + ((size_t)ad * qkvd + hh * hd + i) * rank;
      const float *t = tq + (size_t)r * 64;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint16_t *brow = B + (size_t)((e < 4) ? e : (half + e - 4)) * rank;
        float acc = 0.f;
        for (int j = 0; j < rank; j += 8) {
          const uint4 raw = *reinterpret_cast<const uint4 *>(brow + j);
          const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
          for (int u = 0; u < 4; ++u)
            acc += __uint_as_float(w4[u] << 16) * t[j + 2 * u] + __uint_as_float(w4[u] & 0xffff0000u) * t[j + 2 * u + 1];
        }
        if (e < 4) av[e] += sc * acc; else cv[e - 4] += sc * acc;
      }
    }
  }
  if (hh < H + Hkv) {
    const float4 t0 = *reinterpret_cast<const float4 *>(rope_tab + ((size_t)r * half + i) * 2);      // cos, sin, cos, sin
    const float4 t1 = *reinterpret_cast<const float4 *>(rope_tab + ((size_t)r * half + i) * 2 + 4);
    const float cs[4] = {t0.x, t0.z, t1.x, t1.z}, sn[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float ra = av[j] * cs[j] - cv[j] * sn[j], rb = av[j] * sn[j] + cv[j] * cs[j];
      av[j] = ra;
      cv[j] = rb;
    }
  }
  auto pack4 = [](const uint16_t(&h)[4]) { return make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)); };
  if (hh < H) {
    // the query operand keeps 16 significant bits: plane 0 the nearest bf16, plane 1 the nearest bf16 of the rest
    const int kvh = hh / group, rr = i_row * group + hh % group;
    const size_t o0 = q_elem_off(b, kvh, rr, i, Hkv, hd), o1 = q_elem_off(b, kvh, rr, i + half, Hkv, hd);
    uint16_t ah[4], ch[4], al[4], cl[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      ah[j] = f2bf(av[j]);
      ch[j] = f2bf(cv[j]);
      al[j] = f2bf(av[j] - bf2f(ah[j]));
      cl[j] = f2bf(cv[j] - bf2f(ch[j]));
    }
    *reinterpret_cast<uint2 *>(qp + o0) = pack4(ah);
    *reinterpret_cast<uint2 *>(qp + o1) = pack4(ch);
    *reinterpret_cast<uint2 *>(qp + q_plane + o0) = pack4(al);
    *reinterpret_cast<uint2 *>(qp + q_plane + o1) = pack4(cl);
    return;
  }
  const int page = min(max(page_table[(size_t)b * max_pages + (pos >> 4)], 0), num_pages - 1), t = pos & 15;
  uint16_t ab[4], cb[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    ab[j] = f2bf(av[j]);
    cb[j] = f2bf(cv[j]);
  }
  if (hh < H + Hkv) {
    uint16_t *tile = kpool + layer_off + ((size_t)page * Hkv + (hh - H)) * (16 * hd);
    *reinterpret_cast<uint2 *>(tile + k_tile_off(t, i)) = pack4(ab);          // four consecutive features sit together
    *reinterpret_cast<uint2 *>(tile + k_tile_off(t, i + half)) = pack4(cb);
  } else {
    uint16_t *tile = vpool + layer_off + ((size_t)page * Hkv + (hh - H - Hkv)) * (16 * hd);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      tile[v_tile_off(t, i + j)] = ab[j];
      tile[v_tile_off(t, i + half + j)] = cb[j];
    }
  }
}

// row-major rotated queries [M][H][hd] -> query operand (stand-alone attention entry point)
__global__ void k_pack_q(int H, int Hkv, int hd, const uint16_t *__restrict__ q, const int32_t *__restrict__ row_req,
                         const int32_t *__restrict__ row_idx, uint16_t *__restrict__ qp, size_t q_plane) {
  const int r = blockIdx.x, group = H / Hkv;
  const int b = row_req[r], i_row = row_idx[r];
  for (int idx = threadIdx.x; idx < H * hd; idx += blockDim.x) {
    const int hh = idx / hd, e = idx % hd;
    const size_t o = q_elem_off(b, hh / group, i_row * group + hh % group, e, Hkv, hd);
    qp[o] = q[(size_t)r * H * hd + idx];
    qp[q_plane + o] = 0;  // the caller's queries are bf16 already
  }
}

// ---------------------------------------------------------------------------------------------
// head of the draft model (Sec. IV-A: two-layer MLP + vocabulary projection) and its law
// ---------------------------------------------------------------------------------------------
// sum of the split partials of a head projection (slice order), optional silu, stored as the next projection's operand
template <int SILU>
__global__ void k_head_act(const float *__restrict__ part, int S, int Mpad, int M, int N, uint4 *__restrict__ out) {
  const int r = blockIdx.x, KB = N / 16;
  for (int k0 = threadIdx.x * 8; k0 < N; k0 += blockDim.x * 8) {
    uint32_t o[4] = {0, 0, 0, 0};
    if (r < M) {
      float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      const float *p = part + (size_t)r * N + k0;
      for (int s = 0; s < S; ++s) {
        const float4 a = *reinterpret_cast<const float4 *>(p + (size_t)s * Mpad * N), b = *reinterpret_cast<const float4 *>(p + (size_t)s * Mpad * N + 4);
        v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w; v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float x0 = v[2 * j], x1 = v[2 * j + 1];
        if (SILU) { x0 = x0 / (1.0f + __expf(-x0)); x1 = x1 / (1.0f + __expf(-x1)); }
        o[j] = (uint32_t)f2bf(x0) | ((uint32_t)f2bf(x1) << 16);
      }
    }
    out[tile_unit(r, k0, KB)] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// q = softmax(z / T_b) of the draft's logits rows, fp32: one block per logits row.  all_rows 0: the laws the verification
// call takes (draft i+1 of request b from row i < gamma_b, written to q row draft_offsets[b] + i); 1: every row.
__global__ __launch_bounds__(256) void k_softmax_q(const float *__restrict__ z, int V, const int32_t *__restrict__ row_req,
                                                   const int32_t *__restrict__ row_idx, const int32_t *__restrict__ off,
                                                   const float *__restrict__ temperature, int all_rows, float *__restrict__ q) {
  const int m = blockIdx.x, tid = threadIdx.x, b = row_req[m], i = row_idx[m];
  const float T = temperature[b];
  if (!(T > 0.f)) return;                                   // greedy requests need no law
  if (!all_rows && i >= off[b + 1] - off[b]) return;        // the last row of a request scores no draft
  const float *zr = z + (size_t)m * V;
  float *qr = q + (size_t)(all_rows ? m : m - b) * V;
  __shared__ float s_f[4];
  __shared__ double s_d[4];
  float mx = -INFINITY;
  for (int k = tid; k < V; k += 256) mx = fmaxf(mx, zr[k]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  if ((tid & 63) == 0) s_f[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(s_f[0], s_f[1]), fmaxf(s_f[2], s_f[3]));
  const float k2 = kLog2eF / T;
  double sum = 0.0;
  for (int k0 = tid; k0 < V; k0 += 256 * 8) {   // eight terms in fp32, the groups in fp64
    float g = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (k0 + j * 256 < V) g += __builtin_amdgcn_exp2f((zr[k0 + j * 256] - mx) * k2);
    sum += (double)g;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
  if ((tid & 63) == 0) s_d[tid >> 6] = sum;
  __syncthreads();
  const float inv = (float)(1.0 / ((s_d[0] + s_d[1]) + (s_d[2] + s_d[3])));
  for (int k = tid; k < V; k += 256) qr[k] = __builtin_amdgcn_exp2f((zr[k] - mx) * k2) * inv;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
enum { W_DRAFT1 = 5, W_DRAFT2 = 6, W_DRAFTV = 7 };   // the three projections of the draft model's head (after FSV_W_*)

struct gemm_shape {
  int N, K, NTpad, mode;  // mode 1 = gate|up interleave
  int f16;                // operands in fp16: the projections fed by a normalisation or by the attention output
};

gemm_shape shape_of(const fsv_ctx *c, int which) {
  const fsv_model_desc &d = c->d;
  const int qd = d.n_heads * d.head_dim, qkvd = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  gemm_shape s{};
  switch (which) {
    case FSV_W_QKV: s.N = qkvd; s.K = d.d_model; s.f16 = 1; break;
    case FSV_W_O: s.N = d.d_model; s.K = qd; s.f16 = 1; break;
    case FSV_W_GATE_UP: s.N = 2 * d.d_ffn; s.K = d.d_model; s.mode = 1; s.f16 = 1; break;
    case FSV_W_DOWN: s.N = d.d_model; s.K = d.d_ffn; break;
    case W_DRAFT1: s.N = c->draft_dh; s.K = d.d_model; break;
    case W_DRAFT2: s.N = c->draft_dp; s.K = c->draft_dh; break;
    case W_DRAFTV: s.N = d.vocab; s.K = c->draft_dp; break;
    default: s.N = d.vocab; s.K = d.d_model; s.f16 = 1; break;   // LM head
  }
  s.NTpad = fsv_ceil_div(fsv_ceil_div(s.N, 32), 4) * 4;
  return s;
}

// How a projection is cut into blocks: compute waves (weight strips of 32 features) per block and K splits.
struct gemm_launch {
  int ncw, splits;
};

// K splits so that feature blocks x splits x row blocks comes to about one block per compute unit (a block fills
// the unit's LDS with its activation ring; more splits only add partial sums to write and read back)
int pick_splits(const fsv_ctx *c, const gemm_shape &s, int Mt, bool allow, int ncw) {
  if (!allow) return 1;
  const int nchunks = s.K / KCHUNK, base = fsv_ceil_div(s.NTpad, ncw) * fsv_ceil_div(Mt, 4);
  int sp = c->n_cus / base;
  sp = max(1, min(sp, nchunks));
  if (sp >= 8) sp &= ~7;  // a multiple of eight keeps each split on one XCD (see k_gemm); the K cut is balanced, not equal
  else {
    // the longest block sets the time: the fewest splits whose longest block is no longer than with sp (five splits of
    // sixteen granules give blocks of 3 and 4, four give blocks of 4: same time, a fifth fewer partial sums)
    const int longest = fsv_ceil_div(nchunks, sp);
    while (sp > 1 && fsv_ceil_div(nchunks, sp - 1) == longest) --sp;
  }
  return sp;
}

// With one row block (up to 128 rows) a projection is bound by streaming its weights, every wave streams its own strip
// and what counts is that all compute units take part: among four, three and two strips per block take the one with
// the least serial work per compute unit, rounds of blocks x strips per block x granules per split (8B shapes: q|k|v
// goes from 48 x 4 = 192 blocks of four strips to 64 x 4 = 256 blocks of three; 1B shapes: gate|up from 128 blocks to
// 256 of two strips).  Ties keep the larger block.  With several row blocks the matrix cores are the bound and a
// block keeps one compute wave per SIMD.
gemm_launch pick_launch(const fsv_ctx *c, const gemm_shape &s, int Mt, bool allow) {
  if (c->gemm_ncw_force) return gemm_launch{c->gemm_ncw_force, pick_splits(c, s, Mt, allow, c->gemm_ncw_force)};
  gemm_launch best{4, pick_splits(c, s, Mt, allow, 4)};
  if (Mt > 4) return best;
  const int nchunks = s.K / KCHUNK;
  long best_cost = -1;
  for (int ncw = 4; ncw >= 2; --ncw) {
    const int sp = pick_splits(c, s, Mt, allow, ncw);
    const long blocks = (long)fsv_ceil_div(s.NTpad, ncw) * sp;
    const long cost = (long)fsv_ceil_div((int)blocks, c->n_cus) * ncw * fsv_ceil_div(nchunks, sp);
    if (best_cost < 0 || cost < best_cost) {
      best = gemm_launch{ncw, sp};
      best_cost = cost;
    }
  }
  return best;
}

// Re-tile one weight matrix into the operand order of the matrix cores.  A matrix of an fp16 projection (shape_of().f16)
// is converted from bf16 on the way, times 2^s with s chosen so that its largest weight lands in [2^13, 2^14): every
// weight down to 2^-31 of the largest is then an exact fp16 number (smaller ones round on the 2^-24 grid of the scaled
// matrix), and nothing overflows.  *oscale receives 2^-s, which the projection multiplies its fp32 sums by.
int pack_weight(fsv_ctx *c, const void *src, int which, void **dst, float *oscale = nullptr) {
  gemm_shape s = shape_of(c, which);
  const int strip_units = (s.K / 16) * 64 + c->strip_pad_bytes / 16;
  const size_t units = (size_t)s.NTpad * strip_units;
  if (units * 16 > 0xFFFF0000ull) FSV_FAIL(c, FSV_E_UNSUPPORTED, "a weight matrix must stay below 4 GiB");
  float wscale = 1.0f;
  if (s.f16) {
    if (!oscale) FSV_FAIL(c, FSV_E_INVALID_ARG, "internal: an fp16 projection needs a place for its scale");
    if (!c->absmax) FSV_HIP(c, hipMalloc((void **)&c->absmax, sizeof(uint32_t)));
    FSV_HIP(c, hipMemset(c->absmax, 0, sizeof(uint32_t)));
    const size_t n8 = (size_t)s.N * s.K / 8;
    hipLaunchKernelGGL(k_absmax_bf16, dim3((unsigned)min((size_t)4096, (n8 + 255) / 256)), dim3(256), 0, 0, (const uint4 *)src, n8,
                       c->absmax);
    uint32_t bits = 0;
    FSV_HIP(c, hipMemcpy(&bits, c->absmax, sizeof bits, hipMemcpyDeviceToHost));
    int sh = 0;
    if (bits >= 0x0080u && bits < 0x7f80u) sh = 13 - ((int)(bits >> 7) - 127);   // a finite, normal largest weight
    sh = max(-100, min(100, sh));
    wscale = ldexpf(1.0f, sh);
    *oscale = ldexpf(1.0f, -sh);
  }
  FSV_HIP(c, hipMalloc(dst, units * 16));
  hipLaunchKernelGGL(k_pack_w, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, 0, (const uint16_t *)src, s.N, s.K,
                     s.NTpad, s.mode, c->d.d_ffn, (uint4 *)*dst, s.f16, wscale, strip_units);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int copy_dev(fsv_ctx *c, void **dst, const void *src, size_t bytes) {
  FSV_HIP(c, hipMalloc(dst, bytes));
  FSV_HIP(c, hipMemcpy(*dst, src, bytes, hipMemcpyDeviceToDevice));
  return FSV_OK;
}

template <int EPI>
int launch_gemm(fsv_ctx *c, int cls, const void *Wp, const void *Ap, void *out, const gemm_shape &s, int M, gemm_launch gl,
                hipStream_t st, float oscale = 1.0f) {
  return fsv_bf16_gemm(c, cls, EPI, Wp, Ap, out, s.N, s.K, s.NTpad, M, gl.splits, (EPI == EPI_SWIGLU) ? c->d.d_ffn / 16 : 0,
                       s.f16, oscale, gl.ncw, st);
}

size_t layer_stride(const fsv_ctx *c, int num_pages) {
  return (size_t)num_pages * c->d.n_kv_heads * 16 * c->d.head_dim;
}

}  // namespace

int fsv_bf16_create(fsv_ctx *c, const fsv_weights *w) {
  const fsv_model_desc &d = c->d;
  const int qd = d.n_heads * d.head_dim, qkvd = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  int rc;
  {
    int dev = 0;
    FSV_HIP(c, hipGetDevice(&dev));
    FSV_HIP(c, hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (c->n_cus < 1) c->n_cus = 1;
  }
  if (const char *e = getenv("FSV_STRIP_PAD_KIB")) {   // measurement knob; read before any matrix is re-tiled
    const int v = atoi(e);
    if (v >= 0 && v <= 64) c->strip_pad_bytes = v * 1024;
  }
  if (const char *e = getenv("FSV_GEMM_NCW")) {   // read before anything is sized by pick_launch
    const int v = atoi(e);
    if (v >= 2 && v <= 4) c->gemm_ncw_force = v;
  }
  if ((rc = copy_dev(c, &c->embed, w->embed, (size_t)2 * d.vocab * d.d_model))) return rc;
  if ((rc = copy_dev(c, &c->final_norm, w->final_norm, (size_t)2 * d.d_model))) return rc;
  if ((rc = pack_weight(c, w->lm_head, FSV_W_LM_HEAD, &c->lm_head, &c->os_lm_head))) return rc;
  c->layers.resize(d.n_layers);
  for (int l = 0; l < d.n_layers; ++l) {
    fsv_layer_w &L = c->layers[l];
    if ((rc = copy_dev(c, &L.attn_norm, w->attn_norm[l], (size_t)2 * d.d_model))) return rc;
    if ((rc = copy_dev(c, &L.mlp_norm, w->mlp_norm[l], (size_t)2 * d.d_model))) return rc;
    if ((rc = pack_weight(c, w->w_qkv[l], FSV_W_QKV, &L.w_qkv, &L.os_qkv))) return rc;
    if ((rc = pack_weight(c, w->w_o[l], FSV_W_O, &L.w_o, &L.os_o))) return rc;
    if ((rc = pack_weight(c, w->w_gate_up[l], FSV_W_GATE_UP, &L.w_gate_up, &L.os_gate_up))) return rc;
    if ((rc = pack_weight(c, w->w_down[l], FSV_W_DOWN, &L.w_down))) return rc;
  }
  // rotary frequencies theta^(-2i/hd) in fp64
  {
    std::vector<double> f(d.head_dim / 2);
    for (int i = 0; i < d.head_dim / 2; ++i) f[i] = pow((double)d.rope_theta, -2.0 * i / d.head_dim);
    FSV_HIP(c, hipMalloc((void **)&c->inv_freq, sizeof(double) * f.size()));
    FSV_HIP(c, hipMemcpy(c->inv_freq, f.data(), sizeof(double) * f.size(), hipMemcpyHostToDevice));
  }
  FSV_HIP(c, hipMalloc((void **)&c->rope_tab, sizeof(float) * (size_t)c->max_rows * d.head_dim));
  const int MtMax = fsv_ceil_div(c->max_rows, 32);
  const size_t rows_pad = (size_t)MtMax * 32;
  auto zalloc = [&](void **p, size_t bytes) -> int {
    FSV_HIP(c, hipMalloc(p, bytes));
    FSV_HIP(c, hipMemset(*p, 0, bytes));
    return FSV_OK;
  };
  const int widest = max(max(d.d_model, qd), d.d_ffn);
  if ((rc = zalloc(&c->buf_a, rows_pad * widest * 2))) return rc;       // operand-order activations (also x packing)
  if ((rc = zalloc(&c->buf_att, rows_pad * qd * 2))) return rc;
  if ((rc = zalloc(&c->buf_act, rows_pad * d.d_ffn * 2))) return rc;
  c->q_plane_units = (size_t)d.max_batch * RTMAX * d.n_kv_heads * d.head_dim * 32 / 8;
  if ((rc = zalloc(&c->buf_q, 2 * c->q_plane_units * 16))) return rc;   // two planes: hi and lo
  // split-K partials: worst case over row counts
  size_t part = 0;
  for (int which = FSV_W_QKV; which <= FSV_W_LM_HEAD; ++which) {
    gemm_shape s = shape_of(c, which);
    if (which == FSV_W_LM_HEAD) continue;  // written straight to the logits
    for (int Mt = 1; Mt <= MtMax; ++Mt)
      part = max(part, (size_t)pick_launch(c, s, Mt, which != FSV_W_GATE_UP).splits * Mt * 32 * s.N * 4);
  }
  c->part_bytes = part;
  if ((rc = zalloc(&c->buf_part, part))) return rc;
  if ((rc = fsv_bf16_attn_create(c))) return rc;
  if ((rc = fsv_bf16_gemm_init(c))) return rc;
  FSV_HIP(c, hipDeviceSynchronize());
  return FSV_OK;
}

int fsv_bf16_forward(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan *plan, int M, float *logits, int draft, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  const int Mt = fsv_ceil_div(M, 32), Mpad = Mt * 32;
  const gemm_shape sq = shape_of(c, FSV_W_QKV), so = shape_of(c, FSV_W_O), sg = shape_of(c, FSV_W_GATE_UP),
                   sd = shape_of(c, FSV_W_DOWN), sl = shape_of(c, FSV_W_LM_HEAD);
  const gemm_launch glq = pick_launch(c, sq, Mt, true), glo = pick_launch(c, so, Mt, true), gld = pick_launch(c, sd, Mt, true),
                    glg = pick_launch(c, sg, Mt, false), gll = pick_launch(c, sl, Mt, false);
  const int spq = glq.splits, spo = glo.splits, spd = gld.splits;
  float *part = (float *)c->buf_part;
  const int nthr = min(1024, max(64, fsv_ceil_div(d.d_model / 8, 64) * 64));  // one 8-wide slice per thread
  int rc;
  const fsv_attn_plan &pl = *plan;
  if ((rc = fsv_bf16_attn_plan_launch(c, b, plan, s))) return rc;
  {
    const int n = M * (d.head_dim / 2);
    hipLaunchKernelGGL(k_rope_table, dim3(fsv_ceil_div(n, 256)), dim3(256), 0, s, M, d.head_dim / 2,
                       (const double *)c->inv_freq, c->row_pos, (float *)c->rope_tab);
  }
  // draft model (Sec. IV-A): only the anchor block (the last layer) on the draft's one-layer KV pools, then its own head
  const int l_first = draft ? d.n_layers - 1 : 0;
  // adapters of the evolved target: per-request LoRA pairs on q|k|v and o of every layer but the last
  const bool lora = !draft && c->lora_n > 0 && b->adapter != nullptr;
  const size_t qd = (size_t)d.n_heads * d.head_dim, qkvd = qd + 2 * (size_t)d.n_kv_heads * d.head_dim;
  auto lora_for = [&](int layer, bool lq, bool lo_) {
    lora_args la;
    la.row_req = c->row_req; la.adapter = b->adapter; la.n = c->lora_n; la.rank = c->lora_rank; la.scale = c->lora_scale;
    if (lq) { la.aq = c->lora_aq + (size_t)layer * c->lora_n * c->lora_rank * d.d_model; la.t_out = c->lora_t; }
    if (lo_) {
      la.ao = c->lora_ao + (size_t)layer * c->lora_n * c->lora_rank * qd;
      la.bo = c->lora_bo + (size_t)layer * c->lora_n * d.d_model * c->lora_rank;
      la.att = (const uint4 *)c->buf_att; la.qd = (int)qd;
    }
    return la;
  };
  const bool lq0 = lora && d.n_layers > 1;
  {
    fsv_prof_scope ps(c, s, FSV_K_NORM, 0.0);
    if (lq0)
      hipLaunchKernelGGL((k_resid_norm<1, 1, 0>), dim3(Mpad), dim3(nthr), 0, s, M, d.d_model, d.rms_eps, c->row_tok,
                         (const uint16_t *)c->embed, nullptr, 0, Mpad, c->x, (const uint16_t *)c->layers[l_first].attn_norm,
                         (uint4 *)c->buf_a, lora_for(0, true, false));
    else
      hipLaunchKernelGGL((k_resid_norm<1, 0, 0>), dim3(Mpad), dim3(nthr), 0, s, M, d.d_model, d.rms_eps, c->row_tok,
                         (const uint16_t *)c->embed, nullptr, 0, Mpad, c->x, (const uint16_t *)c->layers[l_first].attn_norm,
                         (uint4 *)c->buf_a, lora_args{});
  }
  for (int l = l_first; l < d.n_layers; ++l) {
    const fsv_layer_w &L = c->layers[l];
    const size_t lo = (size_t)(draft ? 0 : l) * layer_stride(c, b->num_pages);
    const bool adapted = lora && l < d.n_layers - 1;         // the last block belongs to the invariant head
    const bool next_adapted = lora && l + 1 < d.n_layers - 1;
    if ((rc = launch_gemm<EPI_PARTIAL>(c, FSV_K_GEMM_QKV, L.w_qkv, c->buf_a, part, sq, M, glq, s, L.os_qkv))) return rc;
    {
      fsv_prof_scope ps(c, s, FSV_K_ROPE_APPEND, 0.0);
      const dim3 rg(M, fsv_ceil_div((d.n_heads + 2 * d.n_kv_heads) * (d.head_dim / 8), 256));
#define FSV_ROPE_ARGS d.n_heads, d.n_kv_heads, d.head_dim, (const float *)c->rope_tab, part, spq, Mpad, c->row_req, c->row_idx, \
                      c->row_pos, b->page_table, d.max_pages_per_req, b->num_pages, lo, (uint16_t *)c->buf_q,                  \
                      c->q_plane_units * 8, (uint16_t *)b->k_pool, (uint16_t *)b->v_pool
      if (adapted)
        hipLaunchKernelGGL(k_rope_append<1>, rg, dim3(256), 0, s, FSV_ROPE_ARGS, b->adapter, c->lora_n, c->lora_rank,
                           (const float *)c->lora_scale, c->lora_bq + (size_t)l * c->lora_n * qkvd * c->lora_rank,
                           (const float *)c->lora_t);
      else
        hipLaunchKernelGGL(k_rope_append<0>, rg, dim3(256), 0, s, FSV_ROPE_ARGS, nullptr, 0, 0, nullptr, nullptr, nullptr);
#undef FSV_ROPE_ARGS
    }
    if ((rc = fsv_bf16_attn_launch(c, b, &pl, lo, s))) return rc;
    if ((rc = launch_gemm<EPI_PARTIAL>(c, FSV_K_GEMM_O, L.w_o, c->buf_att, part, so, M, glo, s, L.os_o))) return rc;
    {
      fsv_prof_scope ps(c, s, FSV_K_NORM, 0.0);
      if (adapted)
        hipLaunchKernelGGL((k_resid_norm<0, 0, 1>), dim3(Mpad), dim3(nthr), 0, s, M, d.d_model, d.rms_eps, c->row_tok, nullptr,
                           part, spo, Mpad, c->x, (const uint16_t *)L.mlp_norm, (uint4 *)c->buf_a, lora_for(l, false, true));
      else
        hipLaunchKernelGGL((k_resid_norm<0, 0, 0>), dim3(Mpad), dim3(nthr), 0, s, M, d.d_model, d.rms_eps, c->row_tok, nullptr,
                           part, spo, Mpad, c->x, (const uint16_t *)L.mlp_norm, (uint4 *)c->buf_a, lora_args{});
    }
    if ((rc = launch_gemm<EPI_SWIGLU>(c, FSV_K_GEMM_GATE_UP, L.w_gate_up, c->buf_a, c->buf_act, sg, M, glg, s, L.os_gate_up))) return rc;
    if ((rc = launch_gemm<EPI_PARTIAL>(c, FSV_K_GEMM_DOWN, L.w_down, c->buf_act, part, sd, M, gld, s))) return rc;
    {
      fsv_prof_scope ps(c, s, FSV_K_NORM, 0.0);
      const void *gain = (l + 1 < d.n_layers) ? c->layers[l + 1].attn_norm : c->final_norm;
      if (draft)
        hipLaunchKernelGGL((k_resid_norm<0, 0, 0, 1>), dim3(Mpad), dim3(nthr), 0, s, M, d.d_model, d.rms_eps, c->row_tok, nullptr,
                           part, spd, Mpad, c->x, (const uint16_t *)gain, (uint4 *)c->buf_a, lora_args{});
      else if (next_adapted)
        hipLaunchKernelGGL((k_resid_norm<0, 1, 0>), dim3(Mpad), dim3(nthr), 0, s, M, d.d_model, d.rms_eps, c->row_tok, nullptr,
                           part, spd, Mpad, c->x, (const uint16_t *)gain, (uint4 *)c->buf_a, lora_for(l + 1, true, false));
      else
        hipLaunchKernelGGL((k_resid_norm<0, 0, 0>), dim3(Mpad), dim3(nthr), 0, s, M, d.d_model, d.rms_eps, c->row_tok, nullptr,
                           part, spd, Mpad, c->x, (const uint16_t *)gain, (uint4 *)c->buf_a, lora_args{});
    }
  }
  if (draft) {
    // H_small: z = W_v (W_2 silu(W_1 h)), h = the block's output as just stored in buf_a
    const gemm_shape s1 = shape_of(c, W_DRAFT1), s2 = shape_of(c, W_DRAFT2), sv = shape_of(c, W_DRAFTV);
    const gemm_launch gl1 = pick_launch(c, s1, Mt, true), gl2 = pick_launch(c, s2, Mt, true), glv = pick_launch(c, sv, Mt, false);
    const int sp1 = gl1.splits, sp2 = gl2.splits;
    if ((rc = launch_gemm<EPI_PARTIAL>(c, FSV_K_OTHER, c->draft_w1, c->buf_a, part, s1, M, gl1, s))) return rc;
    hipLaunchKernelGGL(k_head_act<1>, dim3(Mpad), dim3(256), 0, s, part, sp1, Mpad, M, s1.N, (uint4 *)c->draft_h1);
    if ((rc = launch_gemm<EPI_PARTIAL>(c, FSV_K_OTHER, c->draft_w2, c->draft_h1, part, s2, M, gl2, s))) return rc;
    hipLaunchKernelGGL(k_head_act<0>, dim3(Mpad), dim3(256), 0, s, part, sp2, Mpad, M, s2.N, (uint4 *)c->draft_h2);
    if ((rc = launch_gemm<EPI_F32>(c, FSV_K_GEMM_LM_HEAD, c->draft_wv, c->draft_h2, logits, sv, M, glv, s))) return rc;
    FSV_HIP(c, hipGetLastError());
    return FSV_OK;
  }
  if ((rc = launch_gemm<EPI_F32>(c, FSV_K_GEMM_LM_HEAD, c->lm_head, c->buf_a, logits, sl, M, gll, s, c->os_lm_head))) return rc;
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

// The head of the draft model: re-tile its three matrices, size the buffers between them.
int fsv_bf16_draft_attach(fsv_ctx *c, const fsv_draft_head *h) {
  void *old[] = {c->draft_w1, c->draft_w2, c->draft_wv, c->draft_h1, c->draft_h2};
  for (void *p : old)
    if (p) (void)hipFree(p);
  c->draft_w1 = c->draft_w2 = c->draft_wv = c->draft_h1 = c->draft_h2 = nullptr;
  c->draft_dh = c->draft_dp = 0;
  if (!h) return FSV_OK;
  c->draft_dh = h->d_hidden;
  c->draft_dp = h->d_proj;
  int rc;
  if ((rc = pack_weight(c, h->w1, W_DRAFT1, &c->draft_w1))) return rc;
  if ((rc = pack_weight(c, h->w2, W_DRAFT2, &c->draft_w2))) return rc;
  if ((rc = pack_weight(c, h->w_vocab, W_DRAFTV, &c->draft_wv))) return rc;
  const int MtMax = fsv_ceil_div(c->max_rows, 32);
  const size_t rows_pad = (size_t)MtMax * 32;
  FSV_HIP(c, hipMalloc(&c->draft_h1, rows_pad * h->d_hidden * 2));
  FSV_HIP(c, hipMemset(c->draft_h1, 0, rows_pad * h->d_hidden * 2));
  FSV_HIP(c, hipMalloc(&c->draft_h2, rows_pad * h->d_proj * 2));
  FSV_HIP(c, hipMemset(c->draft_h2, 0, rows_pad * h->d_proj * 2));
  size_t part = c->part_bytes;   // the split partials of the head's projections share the forward's buffer
  for (int which : {W_DRAFT1, W_DRAFT2}) {
    const gemm_shape sh = shape_of(c, which);
    for (int Mt = 1; Mt <= MtMax; ++Mt) part = max(part, (size_t)pick_launch(c, sh, Mt, true).splits * Mt * 32 * sh.N * 4);
  }
  if (part > c->part_bytes) {
    (void)hipFree(c->buf_part);
    c->buf_part = nullptr;
    FSV_HIP(c, hipMalloc(&c->buf_part, part));
    FSV_HIP(c, hipMemset(c->buf_part, 0, part));
    c->part_bytes = part;
  }
  FSV_HIP(c, hipDeviceSynchronize());
  return FSV_OK;
}

// The draft's law for every received draft token (or every row): anchor block on the draft's KV pools, head, softmax.
int fsv_bf16_draft_probs(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan *plan, int M, int all_rows, float *q_out,
                         float *logits, hipStream_t s) {
  int rc = fsv_bf16_forward(c, b, plan, M, logits, 1, s);
  if (rc) return rc;
  hipLaunchKernelGGL(k_softmax_q, dim3(M), dim3(256), 0, s, logits, c->d.vocab, c->row_req, c->row_idx, b->draft_offsets,
                     b->temperature, all_rows, q_out);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

// Copy a set of adapters into library-owned tables [layer][adapter][...] (replacing any earlier set).
int fsv_bf16_lora_load(fsv_ctx *c, const fsv_lora *lo) {
  const fsv_model_desc &d = c->d;
  void *old[] = {c->lora_aq, c->lora_bq, c->lora_ao, c->lora_bo, c->lora_scale, c->lora_t};
  for (void *p : old)
    if (p) (void)hipFree(p);
  c->lora_aq = c->lora_bq = c->lora_ao = c->lora_bo = nullptr;
  c->lora_scale = nullptr;
  c->lora_t = nullptr;
  c->lora_n = c->lora_rank = 0;
  if (!lo || lo->n_adapters == 0 || d.n_layers < 2) return FSV_OK;
  const int n = lo->n_adapters, r = lo->rank, NLa = d.n_layers - 1;
  const size_t qd = (size_t)d.n_heads * d.head_dim, qkvd = qd + 2 * (size_t)d.n_kv_heads * d.head_dim, dm = d.d_model;
  FSV_HIP(c, hipMalloc((void **)&c->lora_aq, 2 * (size_t)NLa * n * r * dm));
  FSV_HIP(c, hipMalloc((void **)&c->lora_bq, 2 * (size_t)NLa * n * qkvd * r));
  FSV_HIP(c, hipMalloc((void **)&c->lora_ao, 2 * (size_t)NLa * n * r * qd));
  FSV_HIP(c, hipMalloc((void **)&c->lora_bo, 2 * (size_t)NLa * n * dm * r));
  FSV_HIP(c, hipMalloc((void **)&c->lora_scale, sizeof(float) * n));
  FSV_HIP(c, hipMalloc((void **)&c->lora_t, sizeof(float) * 64 * (size_t)c->max_rows));
  FSV_HIP(c, hipMemcpy(c->lora_scale, lo->scale, sizeof(float) * n, hipMemcpyHostToDevice));
  for (int l = 0; l < NLa; ++l)
    for (int a = 0; a < n; ++a) {
      const size_t i = (size_t)l * n + a;
      FSV_HIP(c, hipMemcpy(c->lora_aq + i * r * dm, lo->a_qkv[i], 2 * (size_t)r * dm, hipMemcpyDeviceToDevice));
      FSV_HIP(c, hipMemcpy(c->lora_bq + i * qkvd * r, lo->b_qkv[i], 2 * qkvd * r, hipMemcpyDeviceToDevice));
      FSV_HIP(c, hipMemcpy(c->lora_ao + i * r * qd, lo->a_o[i], 2 * (size_t)r * qd, hipMemcpyDeviceToDevice));
      FSV_HIP(c, hipMemcpy(c->lora_bo + i * dm * r, lo->b_o[i], 2 * dm * r, hipMemcpyDeviceToDevice));
    }
  FSV_HIP(c, hipDeviceSynchronize());
  c->lora_n = n;
  c->lora_rank = r;
  return FSV_OK;
}

int fsv_bf16_linear(fsv_ctx *c, int which, int layer, const void *x, int M, float *y, hipStream_t s) {
  const gemm_shape sh = shape_of(c, which);
  const int Mt = fsv_ceil_div(M, 32), Mpad = Mt * 32;
  const void *Wp;
  int cls;
  float os = 1.0f;
  switch (which) {
    case FSV_W_QKV: Wp = c->layers[layer].w_qkv; cls = FSV_K_GEMM_QKV; os = c->layers[layer].os_qkv; break;
    case FSV_W_O: Wp = c->layers[layer].w_o; cls = FSV_K_GEMM_O; os = c->layers[layer].os_o; break;
    case FSV_W_GATE_UP: Wp = c->layers[layer].w_gate_up; cls = FSV_K_GEMM_GATE_UP; os = c->layers[layer].os_gate_up; break;
    case FSV_W_DOWN: Wp = c->layers[layer].w_down; cls = FSV_K_GEMM_DOWN; break;
    default: Wp = c->lm_head; cls = FSV_K_GEMM_LM_HEAD; os = c->os_lm_head; break;
  }
  const size_t nact = (size_t)Mpad * (sh.K / 8);
  hipLaunchKernelGGL(k_pack_act, dim3((unsigned)((nact + 255) / 256)), dim3(256), 0, s, (const uint16_t *)x, M, Mpad, sh.K,
                     (uint4 *)c->buf_a, sh.f16);
  int rc;
  if (which == FSV_W_LM_HEAD) return launch_gemm<EPI_F32>(c, cls, Wp, c->buf_a, y, sh, M, pick_launch(c, sh, Mt, false), s, os);
  const gemm_launch gl = pick_launch(c, sh, Mt, which != FSV_W_GATE_UP);
  const int sp = gl.splits;
  if ((rc = launch_gemm<EPI_PARTIAL>(c, cls, Wp, c->buf_a, c->buf_part, sh, M, gl, s, os))) return rc;
  const size_t n = (size_t)M * sh.N;
  hipLaunchKernelGGL(k_reduce_part, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float *)c->buf_part, sp, Mpad,
                     M, sh.N, sh.mode, c->d.d_ffn, y);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_bf16_attention(fsv_ctx *c, int layer, const void *q, const fsv_batch *b, const fsv_attn_plan *plan, int M, float *out,
                       hipStream_t s) {
  const fsv_model_desc &d = c->d;
  const fsv_attn_plan &pl = *plan;
  hipLaunchKernelGGL(k_pack_q, dim3(M), dim3(256), 0, s, d.n_heads, d.n_kv_heads, d.head_dim, (const uint16_t *)q,
                     c->row_req, c->row_idx, (uint16_t *)c->buf_q, c->q_plane_units * 8);
  int rc;
  if ((rc = fsv_bf16_attn_plan_launch(c, b, plan, s))) return rc;
  if ((rc = fsv_bf16_attn_launch(c, b, &pl, (size_t)layer * layer_stride(c, b->num_pages), s))) return rc;
  const int qd = d.n_heads * d.head_dim;
  const size_t n = (size_t)M * (qd / 8);
  hipLaunchKernelGGL(k_unpack_act, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const uint4 *)c->buf_att, M, qd, out);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_bf16_kv_copy(fsv_ctx *c, void *k_pool, void *v_pool, int num_pages, const int32_t *pt_row, int pos0, int n,
                     void *k_lin, void *v_lin, bool import, int layers, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  hipLaunchKernelGGL(k_kv_copy, dim3(n, layers), dim3(256), 0, s, d.n_kv_heads, d.head_dim, num_pages, pt_row, pos0, n,
                     (uint16_t *)k_pool, (uint16_t *)v_pool, (uint16_t *)k_lin, (uint16_t *)v_lin, import ? 1 : 0);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}
