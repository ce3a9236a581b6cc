// FSV_BF16 instantiation of the target forward (Alg. 2 step 2: the target model scores the pending
// token and the received draft block on top of the user's restored KV session; Sec. IV-C: KV pairs
// are computed only for the new tokens).  Written for gfx950: 64-wide waves, bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16), weights and KV pages stored in the order the matrix cores consume
// them so that every global load of the two dominant streams (weights, KV) is one contiguous
// 1 KiB request per wave and needs no LDS round trip.
//
// Operand order ("tile" = what one wave feeds to one MFMA as the 32-row operand):
//   element (row r, k) of a [rows][K] matrix lives at ((r/32 * K/16 + k/16) * 64 + r%32 + 32*((k%16)/8)) * 8 + k%8.
// Weights use it with r = output feature (re-tiled once at create), activations with r = batch row.
// The product is formed transposed, D[n][m] = sum_k W[n][k] X[m][k], so each lane ends up with four
// consecutive output features of one row.
#include <math.h>
#include <stdlib.h>

#include "fsv_internal.h"

namespace {

typedef __hip_bfloat16 bf16;

constexpr int KCB = 8;           // k-blocks (of 16) staged per LDS chunk: 128 contraction elements
constexpr int KCHUNK = KCB * 16;
constexpr int RTMAX = 3;         // query-row tiles of 32 per (request, kv head): group * (gamma+1) <= 96
constexpr float kLog2eF = 1.4426950408889634f;

__device__ inline float bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline uint16_t f2bf(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// offset, in 16-byte units, of the operand unit holding (row r, k .. k+7), k a multiple of 8
__device__ __host__ inline size_t tile_unit(int r, int k, int KB) {
  return ((size_t)(r >> 5) * KB + (k >> 4)) * 64 + (r & 31) + 32 * ((k >> 3) & 1);
}

// ---------------------------------------------------------------------------------------------
// one-time weight re-tiling
// ---------------------------------------------------------------------------------------------
// mode 0: packed row n' = source row n'.  mode 1 (gate|up): every 32-row tile holds 16 hidden features,
// gate and up interleaved in groups of 8 (rows 0-7 gate f0-7, 8-15 up f0-7, 16-23 gate f8-15, 24-31 up f8-15),
// so that after the MFMA one lane owns gate and up of the same four features.
__global__ void k_pack_w(const uint16_t *__restrict__ W, int N, int K, int NTpad, int mode, int F, uint4 *__restrict__ out) {
  const size_t unit = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int KB = K / 16;
  if (unit >= (size_t)NTpad * KB * 64) return;
  const int lane = unit & 63, kb = (unit >> 6) % KB, nt = (unit >> 6) / KB;
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
  out[unit] = v;
}

// row-major bf16 [M][K] -> operand order, zero rows up to Mpad
__global__ void k_pack_act(const uint16_t *__restrict__ x, int M, int Mpad, int K, uint4 *__restrict__ out) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int K8 = K / 8;
  if (t >= (size_t)Mpad * K8) return;
  const int m = t / K8, k0 = (t % K8) * 8;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (m < M) v = *reinterpret_cast<const uint4 *>(x + (size_t)m * K + k0);
  out[tile_unit(m, k0, K / 16)] = v;
}

// operand order bf16 -> row-major fp32 [M][K]
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
    dst[2 * j] = __uint_as_float(w[j] << 16);
    dst[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
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

// ---------------------------------------------------------------------------------------------
// weight-streaming GEMM
// ---------------------------------------------------------------------------------------------
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_F32 = 2 };

// One wave owns 32 output features (one weight tile row) for up to MT*32 batch rows and streams that
// weight strip straight from HBM into MFMA operand registers; the four waves of a block share the
// activation chunk, staged through LDS in operand order.  grid = (feature tiles / 4, K splits, row blocks).
template <int MT, int EPI>
__global__ __launch_bounds__(256) void k_gemm(const bf16x8_t *__restrict__ Wp, const uint4 *__restrict__ Ap,
                                              void *__restrict__ out, int N, int KB, int Mt_total, int M, int Mpad,
                                              int cps, int nchunks, int KBo) {
  __shared__ uint4 lds[2][MT * KCB * 64];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, h = lane >> 5;
  const int nt = blockIdx.x * 4 + w, split = blockIdx.y, mt0 = blockIdx.z * MT;
  const int mtc = min(MT, Mt_total - mt0);
  const int c0 = split * cps, c1 = min(c0 + cps, nchunks);
  f32x16_t acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

  const bf16x8_t *wrow = Wp + (size_t)nt * KB * 64 + lane;
  constexpr int APT = MT * KCB * 64 / 256;  // 16-byte units of the activation chunk each thread stages
  uint4 areg[APT];
  bf16x8_t wcur[KCB], wnext[KCB];

  auto load_a = [&](int c) {
#pragma unroll
    for (int p = 0; p < APT; ++p) {
      const int i = p * 256 + tid, mt = i / (KCB * 64), rem = i % (KCB * 64);
      areg[p] = (mt < mtc) ? Ap[((size_t)(mt0 + mt) * KB + c * KCB) * 64 + rem] : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int p = 0; p < APT; ++p) lds[buf][p * 256 + tid] = areg[p];
  };
  auto load_w = [&](int c, bf16x8_t(&dst)[KCB]) {
#pragma unroll
    for (int kb = 0; kb < KCB; ++kb) dst[kb] = wrow[(size_t)(c * KCB + kb) * 64];
  };

  if (c0 < c1) {
    load_a(c0);
    load_w(c0, wcur);
    store_a(0);
    __syncthreads();
    for (int c = c0; c < c1; ++c) {
      const int buf = (c - c0) & 1;
      const bool more = c + 1 < c1;
      if (more) {
        load_a(c + 1);
        load_w(c + 1, wnext);
      }
#pragma unroll
      for (int kb = 0; kb < KCB; ++kb) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if (mt < mtc) {
            uint4 raw = lds[buf][(mt * KCB + kb) * 64 + lane];
            bf16x8_t a = *reinterpret_cast<bf16x8_t *>(&raw);
            acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wcur[kb], a, acc[mt], 0, 0, 0);
          }
        }
      }
      if (more) {
        store_a(buf ^ 1);
#pragma unroll
        for (int kb = 0; kb < KCB; ++kb) wcur[kb] = wnext[kb];
      }
      __syncthreads();
    }
  }

  // epilogue: lane holds, for batch row m = tile*32 + lane%32, features nt*32 + 8*(v/4) + 4*h + v%4
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (mt >= mtc) continue;
    const int m = (mt0 + mt) * 32 + (lane & 31);
    if constexpr (EPI == EPI_PARTIAL) {
      float *dst = (float *)out + ((size_t)split * Mpad + m) * N;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n0 = nt * 32 + 8 * g + 4 * h;
        if (n0 + 3 < N) {
          *reinterpret_cast<float4 *>(dst + n0) =
              make_float4(acc[mt][4 * g], acc[mt][4 * g + 1], acc[mt][4 * g + 2], acc[mt][4 * g + 3]);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (n0 + r < N) dst[n0 + r] = acc[mt][4 * g + r];
        }
      }
    } else if constexpr (EPI == EPI_F32) {
      if (m < M) {
        float *dst = (float *)out + (size_t)m * N;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n0 = nt * 32 + 8 * g + 4 * h;
          if (n0 + 3 < N && (N & 3) == 0) {
            *reinterpret_cast<float4 *>(dst + n0) =
                make_float4(acc[mt][4 * g], acc[mt][4 * g + 1], acc[mt][4 * g + 2], acc[mt][4 * g + 3]);
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (n0 + r < N) dst[n0 + r] = acc[mt][4 * g + r];
          }
        }
      }
    } else {  // SwiGLU: regs 0-3 gate / 4-7 up of features 16*nt + 4h + r, regs 8-11 / 12-15 of 16*nt + 8 + 4h + r
      if (nt < KBo) {
        uint16_t *base = (uint16_t *)out;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          uint16_t o4[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float gte = acc[mt][8 * j + r], up = acc[mt][8 * j + 4 + r];
            o4[r] = f2bf(gte / (1.0f + __expf(-gte)) * up);
          }
          const size_t unit = ((size_t)(mt0 + mt) * KBo + nt) * 64 + (lane & 31) + 32 * j;
          uint2 pk = make_uint2((uint32_t)o4[0] | ((uint32_t)o4[1] << 16), (uint32_t)o4[2] | ((uint32_t)o4[3] << 16));
          *reinterpret_cast<uint2 *>(base + unit * 8 + 4 * h) = pk;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// residual stream: x (+)= sum of split partials (or embedding), RMSNorm, emit the next GEMM's operand
// ---------------------------------------------------------------------------------------------
template <int EMBED>
__global__ __launch_bounds__(256) void k_resid_norm(int M, int d, float eps, const int32_t *__restrict__ row_tok,
                                                    const uint16_t *__restrict__ E, const float *__restrict__ part,
                                                    int S, int Mpad, float *__restrict__ x,
                                                    const uint16_t *__restrict__ gain, uint4 *__restrict__ a_out) {
  const int r = blockIdx.x, tid = threadIdx.x, KB = d / 16;
  if (r >= M) {
    for (int k0 = tid * 8; k0 < d; k0 += 2048) a_out[tile_unit(r, k0, KB)] = make_uint4(0, 0, 0, 0);
    return;
  }
  float *xr = x + (size_t)r * d;
  float ss = 0.f;
  for (int k0 = tid * 8; k0 < d; k0 += 2048) {
    float v[8];
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
      for (int s = 0; s < S; ++s) {
        const float *p = part + ((size_t)s * Mpad + r) * d + k0;
        float4 pa = *reinterpret_cast<const float4 *>(p), pb = *reinterpret_cast<const float4 *>(p + 4);
        v[0] += pa.x; v[1] += pa.y; v[2] += pa.z; v[3] += pa.w; v[4] += pb.x; v[5] += pb.y; v[6] += pb.z; v[7] += pb.w;
      }
    }
    *reinterpret_cast<float4 *>(xr + k0) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(xr + k0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
#pragma unroll
    for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
  }
  ss = wave_sum(ss);
  __shared__ float s_ss[4];
  if ((tid & 63) == 0) s_ss[tid >> 6] = ss;
  __syncthreads();
  const float rinv = 1.0f / sqrtf(((s_ss[0] + s_ss[1]) + (s_ss[2] + s_ss[3])) / (float)d + eps);
  for (int k0 = tid * 8; k0 < d; k0 += 2048) {  // each thread re-reads exactly what it wrote
    float4 a = *reinterpret_cast<const float4 *>(xr + k0), b = *reinterpret_cast<const float4 *>(xr + k0 + 4);
    float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint4 graw = *reinterpret_cast<const uint4 *>(gain + k0);
    uint32_t g4[4] = {graw.x, graw.y, graw.z, graw.w};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float g0 = __uint_as_float(g4[j] << 16), g1 = __uint_as_float(g4[j] & 0xffff0000u);
      o[j] = (uint32_t)f2bf(v[2 * j] * rinv * g0) | ((uint32_t)f2bf(v[2 * j + 1] * rinv * g1) << 16);
    }
    a_out[tile_unit(r, k0, KB)] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// ---------------------------------------------------------------------------------------------
// KV page tiles (16 positions x head_dim per kv head)
// ---------------------------------------------------------------------------------------------
// K tile: element (t, e) at ((e/16*2 + (e%16)/8)*16 + t)*8 + e%8       (operand of the score MFMA, rows = keys)
// V tile: element (t, e) at ((e/32*2 + (t%8)/4)*32 + e%32)*8 + 4*(t/8) + t%4   (operand of the P.V MFMA, rows = features,
//         contraction index ordered the way the score accumulators leave the probabilities in registers)
__device__ __host__ inline int k_tile_off(int t, int e) { return (((e >> 4) * 2 + ((e >> 3) & 1)) * 16 + t) * 8 + (e & 7); }
__device__ __host__ inline int v_tile_off(int t, int e) {
  return (((e >> 5) * 2 + ((t >> 2) & 1)) * 32 + (e & 31)) * 8 + 4 * (t >> 3) + (t & 3);
}

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
// query operand: row rr = i*group + g of (request, kv head), feature e:
//   (((b*RTMAX + rr/32)*Hkv + kvh)*(hd/16) + e/16)*64 + rr%32 + 32*((e%16)/8) units of 8, element e%8
__device__ inline size_t q_elem_off(int b, int kvh, int rr, int e, int Hkv, int hd) {
  return (((((size_t)b * RTMAX + (rr >> 5)) * Hkv + kvh) * (hd >> 4) + (e >> 4)) * 64 + (rr & 31) + 32 * ((e >> 3) & 1)) * 8 +
         (e & 7);
}

__global__ __launch_bounds__(256) void k_rope_append(int H, int Hkv, int hd, const double *__restrict__ inv_freq,
                                                     const float *__restrict__ part, int S, int Mpad,
                                                     const int32_t *__restrict__ row_req,
                                                     const int32_t *__restrict__ row_idx,
                                                     const int32_t *__restrict__ row_pos,
                                                     const int32_t *__restrict__ page_table, int max_pages,
                                                     int num_pages, size_t layer_off, uint16_t *__restrict__ qp,
                                                     uint16_t *__restrict__ kpool, uint16_t *__restrict__ vpool) {
  __shared__ float s_cos[64], s_sin[64];
  const int r = blockIdx.x, half = hd / 2, heads = H + 2 * Hkv, qkvd = heads * hd, group = H / Hkv;
  const int b = row_req[r], i_row = row_idx[r], pos = row_pos[r];
  if (threadIdx.x < half) {
    double sn, cs;
    sincos((double)pos * inv_freq[threadIdx.x], &sn, &cs);
    s_cos[threadIdx.x] = (float)cs;
    s_sin[threadIdx.x] = (float)sn;
  }
  __syncthreads();
  const int page = min(max(page_table[(size_t)b * max_pages + (pos >> 4)], 0), num_pages - 1), t = pos & 15;
  for (int idx = threadIdx.x; idx < heads * half; idx += blockDim.x) {
    const int hh = idx / half, i = idx % half;
    float a = 0.f, c = 0.f;
    for (int s = 0; s < S; ++s) {
      const float *p = part + ((size_t)s * Mpad + r) * qkvd + hh * hd;
      a += p[i];
      c += p[i + half];
    }
    if (hh < H + Hkv) {
      const float ra = a * s_cos[i] - c * s_sin[i], rb = a * s_sin[i] + c * s_cos[i];
      a = ra;
      c = rb;
    }
    if (hh < H) {
      const int kvh = hh / group, rr = i_row * group + hh % group;
      qp[q_elem_off(b, kvh, rr, i, Hkv, hd)] = f2bf(a);
      qp[q_elem_off(b, kvh, rr, i + half, Hkv, hd)] = f2bf(c);
    } else if (hh < H + Hkv) {
      uint16_t *tile = kpool + layer_off + ((size_t)page * Hkv + (hh - H)) * (16 * hd);
      tile[k_tile_off(t, i)] = f2bf(a);
      tile[k_tile_off(t, i + half)] = f2bf(c);
    } else {
      uint16_t *tile = vpool + layer_off + ((size_t)page * Hkv + (hh - H - Hkv)) * (16 * hd);
      tile[v_tile_off(t, i)] = f2bf(a);
      tile[v_tile_off(t, i + half)] = f2bf(c);
    }
  }
}

// row-major rotated queries [M][H][hd] -> query operand (stand-alone attention entry point)
__global__ void k_pack_q(int H, int Hkv, int hd, const uint16_t *__restrict__ q, const int32_t *__restrict__ row_req,
                         const int32_t *__restrict__ row_idx, uint16_t *__restrict__ qp) {
  const int r = blockIdx.x, group = H / Hkv;
  const int b = row_req[r], i_row = row_idx[r];
  for (int idx = threadIdx.x; idx < H * hd; idx += blockDim.x) {
    const int hh = idx / hd, e = idx % hd;
    qp[q_elem_off(b, hh / group, i_row * group + hh % group, e, Hkv, hd)] = q[(size_t)r * H * hd + idx];
  }
}

// ---------------------------------------------------------------------------------------------
// multi-query paged attention
// ---------------------------------------------------------------------------------------------
// One block = (key range of CH tokens, kv head, request); its four waves take 32-key tiles round robin.
// Per tile a wave loads K and V page tiles straight into MFMA operand registers (each byte of the KV
// stream is used by exactly one wave, all `group` query heads and all gamma+1 positions share it),
// forms S^T = K Q^T (rows = keys, so a query row's scores sit in two lanes), does the online softmax in
// registers, and feeds the probabilities back as the B operand of O^T += V^T P^T without any shuffle:
// the V tile is stored in the key order the score accumulators produce.
template <int HD, int RT>
__global__ __launch_bounds__(256) void k_attention(
    int Hkv, int group, int CH, int rows_max, int max_splits, const uint4 *__restrict__ qp,
    const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ off, const int32_t *__restrict__ page_table,
    int max_pages, int num_pages, const uint16_t *__restrict__ kpool, const uint16_t *__restrict__ vpool,
    size_t layer_off, float *__restrict__ part_o, float *__restrict__ part_ml, uint16_t *__restrict__ out, int KBq) {
  constexpr int KS = HD / 16, VC = HD / 32, OSTR = HD + 4;
  // the query operand and the wave-merge buffer share LDS: the queries are dead once every wave has left its key loop
  constexpr int QBYTES = RT * KS * 64 * 16, OBYTES = RT * 32 * OSTR * 4;
  __shared__ __attribute__((aligned(16))) unsigned char s_raw[QBYTES > OBYTES ? QBYTES : OBYTES];
  uint4 *s_q = reinterpret_cast<uint4 *>(s_raw);
  float *s_o = reinterpret_cast<float *>(s_raw);
  __shared__ float s_m[4][RT * 32], s_l[4][RT * 32];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, h = lane >> 5, r = lane & 31;
  const int b = blockIdx.z, kvh = blockIdx.y, split = blockIdx.x;
  const int L = seq_lens[b], gamma = off[b + 1] - off[b], rs = off[b] + b;
  const int nk = L + gamma + 1, R = group * (gamma + 1);
  const int nsplit = (nk + CH - 1) / CH;
  if (split >= nsplit) return;
  const int rtc = min(RT, (R + 31) >> 5);
  const int key0 = split * CH, key1 = min(nk, key0 + CH);
  const int ntiles = (key1 - key0 + 31) >> 5;
  // queries -> LDS (zero for rows beyond R)
  for (int i = tid; i < RT * KS * 64; i += 256) {
    const int rt = i / (KS * 64), rem = i % (KS * 64), rr = rt * 32 + (rem & 31);
    s_q[i] = (rr < R) ? qp[(((size_t)b * RTMAX + rt) * Hkv + kvh) * (KS * 64) + rem] : make_uint4(0, 0, 0, 0);
  }
  __syncthreads();

  const float sc = kLog2eF / sqrtf((float)HD);
  f32x16_t o[RT][VC];
  float mrun[RT], lrun[RT];
  int lim[RT];  // last key this lane's query row may see
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
    for (int c = 0; c < VC; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[rt][c][v] = 0.f;
    mrun[rt] = -INFINITY;
    lrun[rt] = 0.f;
    const int rr = rt * 32 + r;
    lim[rt] = (rr < R) ? L + rr / group : -1;
  }
  const int32_t *pt = page_table + (size_t)b * max_pages;
  const int npg = (nk + 15) >> 4;

  auto tile_ptrs = [&](int tl, const uint16_t *&k0, const uint16_t *&k1, const uint16_t *&v0, const uint16_t *&v1) {
    const int p0 = (key0 >> 4) + tl * 2, p1 = min(p0 + 1, npg - 1);
    const int g0 = min(max(pt[p0], 0), num_pages - 1), g1 = min(max(pt[p1], 0), num_pages - 1);
    const size_t t0 = layer_off + ((size_t)g0 * Hkv + kvh) * (16 * HD), t1 = layer_off + ((size_t)g1 * Hkv + kvh) * (16 * HD);
    k0 = kpool + t0; k1 = kpool + t1; v0 = vpool + t0; v1 = vpool + t1;
  };
  bf16x8_t kreg[KS], vreg[VC][2];
  auto load_tile = [&](int tl) {
    const uint16_t *k0, *k1, *v0, *v1;
    tile_ptrs(tl, k0, k1, v0, v1);
    const uint16_t *kp = (r < 16) ? k0 : k1;  // operand row = key r: rows 0-15 first page, 16-31 second page
#pragma unroll
    for (int s = 0; s < KS; ++s)
      kreg[s] = *reinterpret_cast<const bf16x8_t *>(kp + (((s * 2 + h) * 16) + (r & 15)) * 8);
#pragma unroll
    for (int c = 0; c < VC; ++c) {
      vreg[c][0] = *reinterpret_cast<const bf16x8_t *>(v0 + ((c * 2 + h) * 32 + r) * 8);
      vreg[c][1] = *reinterpret_cast<const bf16x8_t *>(v1 + ((c * 2 + h) * 32 + r) * 8);
    }
  };

  for (int tl = w; tl < ntiles; tl += 4) {
    load_tile(tl);
    const int kbase = key0 + tl * 32;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      if (rt >= rtc) continue;
      f32x16_t s;
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 raw = s_q[(rt * KS + ks) * 64 + lane];
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kreg[ks], *reinterpret_cast<bf16x8_t *>(&raw), s, 0, 0, 0);
      }
      // accumulator v of this lane: key kbase + 8*(v/4) + 4h + v%4, query row rt*32 + r
      float tmax = -INFINITY;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = kbase + 8 * (v >> 2) + 4 * h + (v & 3);
        s[v] = (key <= lim[rt]) ? s[v] * sc : -INFINITY;
        tmax = fmaxf(tmax, s[v]);
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float mnew = fmaxf(mrun[rt], tmax);
      const float muse = (mnew == -INFINITY) ? 0.f : mnew;
      const float alpha = __builtin_amdgcn_exp2f(mrun[rt] - muse);
      mrun[rt] = mnew;
      float psum = 0.f;
      bf16x8_t pb[2];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(s[v] - muse);
        psum += p;
        pb[v >> 3][v & 7] = (__bf16)p;
      }
      lrun[rt] = lrun[rt] * alpha + psum;
#pragma unroll
      for (int c = 0; c < VC; ++c) {
#pragma unroll
        for (int v = 0; v < 16; ++v) o[rt][c][v] *= alpha;
        o[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vreg[c][0], pb[0], o[rt][c], 0, 0, 0);
        o[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vreg[c][1], pb[1], o[rt][c], 0, 0, 0);
      }
    }
  }

  // merge the four waves (fixed order), then write the block's result
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    lrun[rt] += __shfl_xor(lrun[rt], 32, 64);
    if (h == 0) { s_m[w][rt * 32 + r] = mrun[rt]; s_l[w][rt * 32 + r] = lrun[rt]; }
  }
  __syncthreads();
  float fscale[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int rr = rt * 32 + r;
    const float mm = fmaxf(fmaxf(s_m[0][rr], s_m[1][rr]), fmaxf(s_m[2][rr], s_m[3][rr]));
    fscale[rt] = (mrun[rt] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mrun[rt] - mm);
  }
  for (int ww = 0; ww < 4; ++ww) {
    if (w == ww) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        if (rt >= rtc) continue;
#pragma unroll
        for (int c = 0; c < VC; ++c)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            float *dst = s_o + (rt * 32 + r) * OSTR + 32 * c + 8 * g + 4 * h;
            float4 val = make_float4(o[rt][c][4 * g] * fscale[rt], o[rt][c][4 * g + 1] * fscale[rt],
                                     o[rt][c][4 * g + 2] * fscale[rt], o[rt][c][4 * g + 3] * fscale[rt]);
            if (ww > 0) {
              float4 old = *reinterpret_cast<float4 *>(dst);
              val.x += old.x; val.y += old.y; val.z += old.z; val.w += old.w;
            }
            *reinterpret_cast<float4 *>(dst) = val;
          }
      }
    }
    __syncthreads();
  }
  // every thread: rows rr = tid / (HD/8) + k * (256 / (HD/8)), eight features each
  constexpr int TPR = HD / 8;
  for (int rr = tid / TPR; rr < R; rr += 256 / TPR) {
    const int e0 = (tid % TPR) * 8;
    const float m0 = s_m[0][rr], m1 = s_m[1][rr], m2 = s_m[2][rr], m3 = s_m[3][rr];
    const float mm = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
    auto sf = [&](float mw) { return (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mm); };
    const float ll = ((s_l[0][rr] * sf(m0) + s_l[1][rr] * sf(m1)) + s_l[2][rr] * sf(m2)) + s_l[3][rr] * sf(m3);
    const float *src = s_o + rr * OSTR + e0;
    if (nsplit == 1) {
      const float inv = 1.0f / ll;
      uint32_t pk[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) pk[j] = (uint32_t)f2bf(src[2 * j] * inv) | ((uint32_t)f2bf(src[2 * j + 1] * inv) << 16);
      const int m = rs + rr / group, col = (kvh * group + rr % group) * HD + e0;
      reinterpret_cast<uint4 *>(out)[tile_unit(m, col, KBq)] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    } else {
      const size_t prow = (((size_t)b * Hkv + kvh) * max_splits + split) * rows_max + rr;
      float *dst = part_o + prow * HD + e0;
      *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src);
      *reinterpret_cast<float4 *>(dst + 4) = *reinterpret_cast<const float4 *>(src + 4);
      if (e0 == 0) { part_ml[prow * 2] = mm; part_ml[prow * 2 + 1] = ll; }
    }
  }
}

// merge the key-range partials of requests that were split, in split order
template <int HD>
__global__ __launch_bounds__(256) void k_attn_combine(int Hkv, int group, int CH, int rows_max, int max_splits,
                                                      const int32_t *__restrict__ seq_lens,
                                                      const int32_t *__restrict__ off,
                                                      const float *__restrict__ part_o,
                                                      const float *__restrict__ part_ml, uint16_t *__restrict__ out,
                                                      int KBq) {
  const int b = blockIdx.y, kvh = blockIdx.x, tid = threadIdx.x;
  const int L = seq_lens[b], gamma = off[b + 1] - off[b], rs = off[b] + b;
  const int nk = L + gamma + 1, R = group * (gamma + 1), nsplit = (nk + CH - 1) / CH;
  if (nsplit <= 1) return;
  constexpr int TPR = HD / 8;
  for (int rr = tid / TPR; rr < R; rr += 256 / TPR) {
    const int e0 = (tid % TPR) * 8;
    const size_t base = (((size_t)b * Hkv + kvh) * max_splits) * rows_max + rr;
    float mm = -INFINITY;
    for (int s = 0; s < nsplit; ++s) mm = fmaxf(mm, part_ml[(base + (size_t)s * rows_max) * 2]);
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, ll = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const size_t prow = base + (size_t)s * rows_max;
      const float ms = part_ml[prow * 2];
      const float f = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - mm);
      ll += part_ml[prow * 2 + 1] * f;
      const float *src = part_o + prow * HD + e0;
      float4 a = *reinterpret_cast<const float4 *>(src), c = *reinterpret_cast<const float4 *>(src + 4);
      acc[0] += a.x * f; acc[1] += a.y * f; acc[2] += a.z * f; acc[3] += a.w * f;
      acc[4] += c.x * f; acc[5] += c.y * f; acc[6] += c.z * f; acc[7] += c.w * f;
    }
    const float inv = 1.0f / ll;
    uint32_t pk[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) pk[j] = (uint32_t)f2bf(acc[2 * j] * inv) | ((uint32_t)f2bf(acc[2 * j + 1] * inv) << 16);
    const int m = rs + rr / group, col = (kvh * group + rr % group) * HD + e0;
    reinterpret_cast<uint4 *>(out)[tile_unit(m, col, KBq)] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
  }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct gemm_shape {
  int N, K, NTpad, mode;  // mode 1 = gate|up interleave
};

gemm_shape shape_of(const fsv_ctx *c, int which) {
  const fsv_model_desc &d = c->d;
  const int qd = d.n_heads * d.head_dim, qkvd = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  gemm_shape s{};
  switch (which) {
    case FSV_W_QKV: s.N = qkvd; s.K = d.d_model; break;
    case FSV_W_O: s.N = d.d_model; s.K = qd; break;
    case FSV_W_GATE_UP: s.N = 2 * d.d_ffn; s.K = d.d_model; s.mode = 1; break;
    case FSV_W_DOWN: s.N = d.d_model; s.K = d.d_ffn; break;
    default: s.N = d.vocab; s.K = d.d_model; break;
  }
  s.NTpad = fsv_ceil_div(fsv_ceil_div(s.N, 32), 4) * 4;
  return s;
}

int target_blocks() {
  static int v = 0;
  if (!v) {
    const char *e = getenv("FSV_GEMM_BLOCKS");
    v = e ? atoi(e) : 512;
    if (v < 1) v = 512;
  }
  return v;
}

// K splits so that feature tiles x splits x row blocks comes to about two blocks per compute unit
int pick_splits(const gemm_shape &s, int Mt, bool allow) {
  if (!allow) return 1;
  const int nchunks = s.K / KCHUNK, base = (s.NTpad / 4) * fsv_ceil_div(Mt, 4);
  int sp = target_blocks() / base;
  sp = max(1, min(sp, nchunks));
  const int cps = fsv_ceil_div(nchunks, sp);
  return fsv_ceil_div(nchunks, cps);  // no empty split
}

int pack_weight(fsv_ctx *c, const void *src, int which, void **dst) {
  gemm_shape s = shape_of(c, which);
  const size_t units = (size_t)s.NTpad * (s.K / 16) * 64;
  FSV_HIP(c, hipMalloc(dst, units * 16));
  hipLaunchKernelGGL(k_pack_w, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, 0, (const uint16_t *)src, s.N, s.K,
                     s.NTpad, s.mode, c->d.d_ffn, (uint4 *)*dst);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int copy_dev(fsv_ctx *c, void **dst, const void *src, size_t bytes) {
  FSV_HIP(c, hipMalloc(dst, bytes));
  FSV_HIP(c, hipMemcpy(*dst, src, bytes, hipMemcpyDeviceToDevice));
  return FSV_OK;
}

template <int EPI>
int launch_gemm(fsv_ctx *c, int cls, const void *Wp, const void *Ap, void *out, const gemm_shape &s, int M, int splits,
                hipStream_t st) {
  const int Mt = fsv_ceil_div(M, 32), Mpad = Mt * 32, KB = s.K / 16, nchunks = s.K / KCHUNK;
  const int cps = fsv_ceil_div(nchunks, splits);
  const int mt_blk = Mt >= 4 ? 4 : Mt, mblocks = fsv_ceil_div(Mt, mt_blk);
  dim3 grid(s.NTpad / 4, splits, mblocks);
  const int KBo = (EPI == EPI_SWIGLU) ? c->d.d_ffn / 16 : 0;
  const double bytes = (double)s.N * s.K * 2;
  fsv_prof_scope ps(c, st, cls, bytes);
#define FSV_GEMM_CASE(MTV)                                                                                      \
  hipLaunchKernelGGL((k_gemm<MTV, EPI>), grid, dim3(256), 0, st, (const bf16x8_t *)Wp, (const uint4 *)Ap, out, s.N, \
                     KB, Mt, M, Mpad, cps, nchunks, KBo)
  switch (mt_blk) {
    case 1: FSV_GEMM_CASE(1); break;
    case 2: FSV_GEMM_CASE(2); break;
    case 3: FSV_GEMM_CASE(3); break;
    default: FSV_GEMM_CASE(4); break;
  }
#undef FSV_GEMM_CASE
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int attn_chunk() {
  static int v = 0;
  if (!v) {
    const char *e = getenv("FSV_ATTN_CHUNK");
    v = e ? atoi(e) : 512;
    if (v < 128 || v % 128) v = 512;
  }
  return v;
}

int launch_attention(fsv_ctx *c, const fsv_batch *b, size_t layer_off, hipStream_t st) {
  const fsv_model_desc &d = c->d;
  const int CH = attn_chunk(), group = c->group, KBq = d.n_heads * d.head_dim / 16;
  const int rows_max = group * (d.max_gamma + 1);
  int max_nk = 0, max_rows = 0;
  double kv_tokens = 0;
  for (int i = 0; i < b->batch; ++i) {
    const int g = b->draft_offsets_host[i + 1] - b->draft_offsets_host[i], nk = b->seq_lens_host[i] + g + 1;
    max_nk = max(max_nk, nk);
    max_rows = max(max_rows, group * (g + 1));
    kv_tokens += nk;
  }
  const int nsplit = fsv_ceil_div(max_nk, CH), rt = fsv_ceil_div(max_rows, 32);
  if (nsplit > c->attn_max_splits) FSV_FAIL(c, FSV_E_CAPACITY, "%d key ranges > %d the workspace holds", nsplit, c->attn_max_splits);
  dim3 grid(nsplit, d.n_kv_heads, b->batch);
  {
    fsv_prof_scope ps(c, st, FSV_K_ATTENTION, kv_tokens * d.n_kv_heads * d.head_dim * 4.0);
    float *po = (float *)c->attn_part;
    float *pml = po + (size_t)d.max_batch * d.n_kv_heads * c->attn_max_splits * rows_max * d.head_dim;
    uint16_t *out = (uint16_t *)c->buf_att;
#define FSV_ATTN_LAUNCH(HDV, RTV)                                                                                  \
  hipLaunchKernelGGL((k_attention<HDV, RTV>), grid, dim3(256), 0, st, d.n_kv_heads, group, CH, rows_max,           \
                     c->attn_max_splits, (const uint4 *)c->buf_q, b->seq_lens, b->draft_offsets, b->page_table,    \
                     d.max_pages_per_req, b->num_pages, (const uint16_t *)b->k_pool, (const uint16_t *)b->v_pool,  \
                     layer_off, po, pml, out, KBq)
    if (d.head_dim == 128) {
      if (rt <= 1) FSV_ATTN_LAUNCH(128, 1); else if (rt == 2) FSV_ATTN_LAUNCH(128, 2); else FSV_ATTN_LAUNCH(128, 3);
    } else {
      if (rt <= 1) FSV_ATTN_LAUNCH(64, 1); else if (rt == 2) FSV_ATTN_LAUNCH(64, 2); else FSV_ATTN_LAUNCH(64, 3);
    }
#undef FSV_ATTN_LAUNCH
    FSV_HIP(c, hipGetLastError());
    if (nsplit > 1) {
      fsv_prof_scope pc(c, st, FSV_K_ATTN_COMBINE, 0.0);
      dim3 cg(d.n_kv_heads, b->batch);
      if (d.head_dim == 128)
        hipLaunchKernelGGL((k_attn_combine<128>), cg, dim3(256), 0, st, d.n_kv_heads, group, CH, rows_max,
                           c->attn_max_splits, b->seq_lens, b->draft_offsets, po, pml, out, KBq);
      else
        hipLaunchKernelGGL((k_attn_combine<64>), cg, dim3(256), 0, st, d.n_kv_heads, group, CH, rows_max,
                           c->attn_max_splits, b->seq_lens, b->draft_offsets, po, pml, out, KBq);
      FSV_HIP(c, hipGetLastError());
    }
  }
  return FSV_OK;
}

size_t layer_stride(const fsv_ctx *c, int num_pages) {
  return (size_t)num_pages * c->d.n_kv_heads * 16 * c->d.head_dim;
}

}  // namespace

int fsv_bf16_create(fsv_ctx *c, const fsv_weights *w) {
  const fsv_model_desc &d = c->d;
  const int qd = d.n_heads * d.head_dim, qkvd = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  int rc;
  if ((rc = copy_dev(c, &c->embed, w->embed, (size_t)2 * d.vocab * d.d_model))) return rc;
  if ((rc = copy_dev(c, &c->final_norm, w->final_norm, (size_t)2 * d.d_model))) return rc;
  if ((rc = pack_weight(c, w->lm_head, FSV_W_LM_HEAD, &c->lm_head))) return rc;
  c->layers.resize(d.n_layers);
  for (int l = 0; l < d.n_layers; ++l) {
    fsv_layer_w &L = c->layers[l];
    if ((rc = copy_dev(c, &L.attn_norm, w->attn_norm[l], (size_t)2 * d.d_model))) return rc;
    if ((rc = copy_dev(c, &L.mlp_norm, w->mlp_norm[l], (size_t)2 * d.d_model))) return rc;
    if ((rc = pack_weight(c, w->w_qkv[l], FSV_W_QKV, &L.w_qkv))) return rc;
    if ((rc = pack_weight(c, w->w_o[l], FSV_W_O, &L.w_o))) return rc;
    if ((rc = pack_weight(c, w->w_gate_up[l], FSV_W_GATE_UP, &L.w_gate_up))) return rc;
    if ((rc = pack_weight(c, w->w_down[l], FSV_W_DOWN, &L.w_down))) return rc;
  }
  // rotary frequencies theta^(-2i/hd) in fp64
  {
    std::vector<double> f(d.head_dim / 2);
    for (int i = 0; i < d.head_dim / 2; ++i) f[i] = pow((double)d.rope_theta, -2.0 * i / d.head_dim);
    FSV_HIP(c, hipMalloc((void **)&c->inv_freq, sizeof(double) * f.size()));
    FSV_HIP(c, hipMemcpy(c->inv_freq, f.data(), sizeof(double) * f.size(), hipMemcpyHostToDevice));
  }
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
  if ((rc = zalloc(&c->buf_q, (size_t)d.max_batch * RTMAX * d.n_kv_heads * d.head_dim * 32 * 2))) return rc;
  // split-K partials: worst case over row counts
  size_t part = 0;
  for (int which = FSV_W_QKV; which <= FSV_W_LM_HEAD; ++which) {
    gemm_shape s = shape_of(c, which);
    if (which == FSV_W_LM_HEAD) continue;  // written straight to the logits
    for (int Mt = 1; Mt <= MtMax; ++Mt)
      part = max(part, (size_t)pick_splits(s, Mt, which != FSV_W_GATE_UP) * Mt * 32 * s.N * 4);
  }
  c->part_bytes = part;
  if ((rc = zalloc(&c->buf_part, part))) return rc;
  // attention key-range partials
  const int CH = attn_chunk(), rows_max = c->group * (d.max_gamma + 1);
  c->attn_max_splits = fsv_ceil_div(d.max_pages_per_req * 16, CH);
  const size_t prow = (size_t)d.max_batch * d.n_kv_heads * c->attn_max_splits * rows_max;
  c->attn_part_bytes = prow * (d.head_dim + 2) * 4;
  if ((rc = zalloc(&c->attn_part, c->attn_part_bytes))) return rc;
  FSV_HIP(c, hipDeviceSynchronize());
  return FSV_OK;
}

int fsv_bf16_forward(fsv_ctx *c, const fsv_batch *b, int M, float *logits, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  const int Mt = fsv_ceil_div(M, 32), Mpad = Mt * 32;
  const gemm_shape sq = shape_of(c, FSV_W_QKV), so = shape_of(c, FSV_W_O), sg = shape_of(c, FSV_W_GATE_UP),
                   sd = shape_of(c, FSV_W_DOWN), sl = shape_of(c, FSV_W_LM_HEAD);
  const int spq = pick_splits(sq, Mt, true), spo = pick_splits(so, Mt, true), spd = pick_splits(sd, Mt, true);
  float *part = (float *)c->buf_part;
  int rc;
  {
    fsv_prof_scope ps(c, s, FSV_K_NORM, 0.0);
    hipLaunchKernelGGL(k_resid_norm<1>, dim3(Mpad), dim3(256), 0, s, M, d.d_model, d.rms_eps, c->row_tok,
                       (const uint16_t *)c->embed, nullptr, 0, Mpad, c->x, (const uint16_t *)c->layers[0].attn_norm,
                       (uint4 *)c->buf_a);
  }
  for (int l = 0; l < d.n_layers; ++l) {
    const fsv_layer_w &L = c->layers[l];
    const size_t lo = (size_t)l * layer_stride(c, b->num_pages);
    if ((rc = launch_gemm<EPI_PARTIAL>(c, FSV_K_GEMM_QKV, L.w_qkv, c->buf_a, part, sq, M, spq, s))) return rc;
    {
      fsv_prof_scope ps(c, s, FSV_K_ROPE_APPEND, 0.0);
      hipLaunchKernelGGL(k_rope_append, dim3(M), dim3(256), 0, s, d.n_heads, d.n_kv_heads, d.head_dim,
                         (const double *)c->inv_freq, part, spq, Mpad, c->row_req, c->row_idx, c->row_pos, b->page_table,
                         d.max_pages_per_req, b->num_pages, lo, (uint16_t *)c->buf_q, (uint16_t *)b->k_pool,
                         (uint16_t *)b->v_pool);
    }
    if ((rc = launch_attention(c, b, lo, s))) return rc;
    if ((rc = launch_gemm<EPI_PARTIAL>(c, FSV_K_GEMM_O, L.w_o, c->buf_att, part, so, M, spo, s))) return rc;
    {
      fsv_prof_scope ps(c, s, FSV_K_NORM, 0.0);
      hipLaunchKernelGGL(k_resid_norm<0>, dim3(Mpad), dim3(256), 0, s, M, d.d_model, d.rms_eps, c->row_tok, nullptr, part,
                         spo, Mpad, c->x, (const uint16_t *)L.mlp_norm, (uint4 *)c->buf_a);
    }
    if ((rc = launch_gemm<EPI_SWIGLU>(c, FSV_K_GEMM_GATE_UP, L.w_gate_up, c->buf_a, c->buf_act, sg, M, 1, s))) return rc;
    if ((rc = launch_gemm<EPI_PARTIAL>(c, FSV_K_GEMM_DOWN, L.w_down, c->buf_act, part, sd, M, spd, s))) return rc;
    {
      fsv_prof_scope ps(c, s, FSV_K_NORM, 0.0);
      const void *gain = (l + 1 < d.n_layers) ? c->layers[l + 1].attn_norm : c->final_norm;
      hipLaunchKernelGGL(k_resid_norm<0>, dim3(Mpad), dim3(256), 0, s, M, d.d_model, d.rms_eps, c->row_tok, nullptr, part,
                         spd, Mpad, c->x, (const uint16_t *)gain, (uint4 *)c->buf_a);
    }
  }
  if ((rc = launch_gemm<EPI_F32>(c, FSV_K_GEMM_LM_HEAD, c->lm_head, c->buf_a, logits, sl, M, 1, s))) return rc;
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_bf16_linear(fsv_ctx *c, int which, int layer, const void *x, int M, float *y, hipStream_t s) {
  const gemm_shape sh = shape_of(c, which);
  const int Mt = fsv_ceil_div(M, 32), Mpad = Mt * 32;
  const void *Wp;
  int cls;
  switch (which) {
    case FSV_W_QKV: Wp = c->layers[layer].w_qkv; cls = FSV_K_GEMM_QKV; break;
    case FSV_W_O: Wp = c->layers[layer].w_o; cls = FSV_K_GEMM_O; break;
    case FSV_W_GATE_UP: Wp = c->layers[layer].w_gate_up; cls = FSV_K_GEMM_GATE_UP; break;
    case FSV_W_DOWN: Wp = c->layers[layer].w_down; cls = FSV_K_GEMM_DOWN; break;
    default: Wp = c->lm_head; cls = FSV_K_GEMM_LM_HEAD; break;
  }
  const size_t nact = (size_t)Mpad * (sh.K / 8);
  hipLaunchKernelGGL(k_pack_act, dim3((unsigned)((nact + 255) / 256)), dim3(256), 0, s, (const uint16_t *)x, M, Mpad, sh.K,
                     (uint4 *)c->buf_a);
  int rc;
  if (which == FSV_W_LM_HEAD) return launch_gemm<EPI_F32>(c, cls, Wp, c->buf_a, y, sh, M, 1, s);
  const int sp = pick_splits(sh, Mt, which != FSV_W_GATE_UP);
  if ((rc = launch_gemm<EPI_PARTIAL>(c, cls, Wp, c->buf_a, c->buf_part, sh, M, sp, s))) return rc;
  const size_t n = (size_t)M * sh.N;
  hipLaunchKernelGGL(k_reduce_part, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float *)c->buf_part, sp, Mpad,
                     M, sh.N, sh.mode, c->d.d_ffn, y);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_bf16_attention(fsv_ctx *c, int layer, const void *q, const fsv_batch *b, int M, float *out, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  hipLaunchKernelGGL(k_pack_q, dim3(M), dim3(256), 0, s, d.n_heads, d.n_kv_heads, d.head_dim, (const uint16_t *)q,
                     c->row_req, c->row_idx, (uint16_t *)c->buf_q);
  int rc = launch_attention(c, b, (size_t)layer * layer_stride(c, b->num_pages), s);
  if (rc) return rc;
  const int qd = d.n_heads * d.head_dim;
  const size_t n = (size_t)M * (qd / 8);
  hipLaunchKernelGGL(k_unpack_act, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const uint4 *)c->buf_att, M, qd, out);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int fsv_bf16_kv_copy(fsv_ctx *c, void *k_pool, void *v_pool, int num_pages, const int32_t *pt_row, int pos0, int n,
                     void *k_lin, void *v_lin, bool import, hipStream_t s) {
  const fsv_model_desc &d = c->d;
  hipLaunchKernelGGL(k_kv_copy, dim3(n, d.n_layers), dim3(256), 0, s, d.n_kv_heads, d.head_dim, num_pages, pt_row, pos0, n,
                     (uint16_t *)k_pool, (uint16_t *)v_pool, (uint16_t *)k_lin, (uint16_t *)v_lin, import ? 1 : 0);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}
