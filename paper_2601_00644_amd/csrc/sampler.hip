// Vocabulary-wide softmax statistics, acceptance tests, residual / bonus token selection and KV
// rollback: the accept / reject part of Alg. 2 step 2 (greedy form as printed there; for
// temperature > 0 the speculative-sampling rule that keeps the output law equal to the target's,
// Sec. II and Regime B of Sec. V) and the rollback of Sec. IV-C.
//
// Two launches, both streaming logits from HBM:
//   k_row_stats   grid (chunks / 4, row of the request, request)   one pass over every logits row: per chunk
//                 (max, sum e^{(l-max)/T}) or the argmax
//   k_decide      grid (sub-blocks / 4, requests)   every block first repeats the request's acceptance tests (row
//                 statistics combined, two gathered scalars per draft: cheap, and it saves a launch and a round trip
//                 through memory), then the blocks of a request stream the one row its token is drawn from (and the
//                 draft-law row) into the masses of its 2048-id sub-blocks; the block that finishes last (an integer
//                 ticket per request) locates the sub-block and the id by inverse CDF, emits the outputs and rolls back
// plus, when a request asks for a top-k / nucleus (top-p) cut of the target law, between the two: for bf16 logits
// k_nucleus_top, ONE pass per stage that settles every row whose cut lies within one (first try) or two (second try)
// binades of the row maximum; for the rows it leaves, and for fp32 logits, k_nucleus: one pass over the row per digit
// of the cut value (two for bf16 logits, three for fp32) and stage.
// Rows are addressed as (request, row within the request), so the step needs no row map.  Every floating-point sum is
// taken in a fixed order (the ticket only decides WHICH block adds the sub-block masses up, in sub-block order); the only
// other atomics are integer adds into the nucleus histograms, whose result does not depend on their order.
#include <limits.h>
#include <math.h>
#include <stdlib.h>
#include <type_traits>
#include <mutex>

#include "fsv_internal.h"

namespace {

constexpr double kLog2e = 1.4426950408889634074;

// e^{d / T} for d <= 0 as 2^{d * k}, k = log2(e) / T carried as a float pair (k_hi + k_lo) so that its rounding does not
// tilt large against small terms; the product is formed in fp32 (the error it leaves is relative to a term's own size,
// 1e-7 for the terms that carry the mass) and 2^z comes from the transcendental unit.  Vocabulary-wide sums are bound by
// this arithmetic, not by HBM, if it is done in fp64.
struct exp_scale {
  float hi, lo;
};
__device__ inline exp_scale make_exp_scale(double k) {
  exp_scale s;
  s.hi = (float)k;
  s.lo = (float)(k - (double)s.hi);
  return s;
}
__device__ inline float exp_scaled(float d, exp_scale k) {
  const float z = fmaf(d, k.lo, d * k.hi);
  return (z > -150.f) ? __builtin_amdgcn_exp2f(z) : 0.f;  // also catches -inf and NaN (a chunk that is all -inf)
}

template <typename LT>
struct loader;

template <>
struct loader<uint16_t> {  // bf16 bit patterns
  // eight ids from a 16-byte aligned, fully in-range address: no bounds logic, so that a run of these loads is
  // issued back to back (a branch per load makes the wave wait for each load before the next)
  static __device__ inline void load8_fast(const uint16_t *row, int i0, float (&v)[8]) {
    uint4 raw = *reinterpret_cast<const uint4 *>(row + i0);
    uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[2 * j] = __uint_as_float(w[j] << 16);
      v[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
  }
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
  static __device__ inline void load8_fast(const float *row, int i0, float (&v)[8]) {
    float4 a = *reinterpret_cast<const float4 *>(row + i0);
    float4 b = *reinterpret_cast<const float4 *>(row + i0 + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
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

// One wave per 8192-id chunk of a row: all of the chunk's loads are issued before the first use (sixteen 16-byte loads
// per lane for bf16), the maximum and the sum are reduced over the wave with shuffles, and no LDS or barrier is
// involved; waves are independent, so a compute unit keeps a dozen of them streaming.
// grid = (chunks / 4, largest gamma of the batch + 1, requests): row i of request b is logits row off[b] + b + i.
template <typename LT>
__global__ __launch_bounds__(256) void k_row_stats(const LT *__restrict__ logits, int V, int nc,
                                                   const int32_t *__restrict__ off,
                                                   const float *__restrict__ temperature, float *__restrict__ pmax,
                                                   double *__restrict__ psum, int32_t *__restrict__ parg, int vec) {
  constexpr int P = FSV_CHUNK / 512;  // passes of 64 lanes x 8 ids
  const int tid = threadIdx.x, lane = tid & 63, c = blockIdx.x * 4 + (tid >> 6), bq = blockIdx.z;
  if (c >= nc) return;
  const int o = off[bq];
  if ((int)blockIdx.y > off[bq + 1] - o) return;   // the request has fewer rows
  const int r = o + bq + blockIdx.y;
  const LT *row = logits + (size_t)r * V;
  const float T = temperature[bq];
  float v[P][8];
  const int base = c * FSV_CHUNK + lane * 8;
  if (vec && (c + 1) * FSV_CHUNK <= V) {  // wave-uniform: every chunk but a ragged last one
#pragma unroll
    for (int p = 0; p < P; ++p) loader<LT>::load8_fast(row, base + p * 512, v[p]);
  } else {
#pragma unroll
    for (int p = 0; p < P; ++p) loader<LT>::load8(row, base + p * 512, V, vec != 0, -INFINITY, v[p]);
  }
  // A row needs either the argmax (greedy, T = 0) or the sum of exponentials (T > 0), never both; the vocabulary-wide
  // pass is bound by its arithmetic as soon as it carries more than a handful of operations per id.
  float mx = -INFINITY;
  int ai = INT_MAX;
  double sum = 0.0;
  if (T > 0.f) {
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
      for (int j = 0; j < 8; ++j) mx = fmaxf(mx, v[p][j]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (mx > -INFINITY) {  // wave-uniform; an all -inf chunk carries no mass
      // 2^{(l - max) k} with k in fp32: its rounding moves a term by 6e-8 of its own exponent, nothing for the terms
      // that carry the sum; ids beyond the vocabulary were loaded as -inf and come out as 0
      const float k = (float)(kLog2e / (double)T);
#pragma unroll
      for (int p = 0; p < P; ++p) {  // eight terms at a time in fp32, the groups in fp64
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) part += __builtin_amdgcn_exp2f((v[p][j] - mx) * k);
        sum += (double)part;
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    }
  } else {
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (v[p][j] > mx) { mx = v[p][j]; ai = base + p * 512 + j; }   // ids ascend with (p, j): the first maximum stays
    // wave (max, lowest id attaining it)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      float om = __shfl_xor(mx, off, 64);
      int oi = __shfl_xor(ai, off, 64);
      if (om > mx || (om == mx && oi < ai)) { mx = om; ai = oi; }
    }
  }
  if (lane == 0) {
    pmax[(size_t)r * nc + c] = mx;
    psum[(size_t)r * nc + c] = sum;
    parg[(size_t)r * nc + c] = ai;
  }
}

// ---- top-k / nucleus (top-p) cut of the target law ----------------------------------------------------------
// The cut keeps every token whose logit is at least the cut value: for top-k the value of the top_k-th most probable
// token, for top-p the largest value for which the kept mass reaches top_p of what the top-k cut left (tokens tied at
// the cut value are all kept, so the set does not depend on an order among ties).  The cut value
// is found digit by digit on a monotone 32-bit key of the logit: one pass over the row per digit builds a histogram of
// the mass per digit value (in LDS, in 2^-40 fixed point, so that the sums do not depend on the order of the atomic
// adds), and a scan from the top picks the digit at which the kept mass crosses top_p of the total.
__device__ inline uint32_t okey(float f) {  // monotone: a < b  <=>  okey(a) < okey(b)
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int FSV_NUC_BINS = 2048;
constexpr double kNucScale = 1099511627776.0;  // 2^40

// LEVEL 0: key bits 31..21, LEVEL 1: bits 20..10, LEVEL 2: bits 9..0.  LAST marks the level that fixes the whole key
// (level 1 for bf16 logits, whose keys have no information below bit 16; level 2 for fp32 logits).  grid = rows.
// MODE 1 (top-k) selects the key of the top_k-th most probable token by COUNT (a second, integer histogram) and leaves
// the cut key and the mass at or above it per row; MODE 0 (top-p) selects by mass among the tokens the top-k cut kept
// (all of them when the row has none) and writes the row's final cut key and kept mass.  A row that asks for neither
// gets key 0 (nothing is cut); one that asks for top-k only gets the top-k cut as its final one.
template <typename LT, int LEVEL, bool LAST, int MODE>
__global__ __launch_bounds__(1024) void k_nucleus(const LT *__restrict__ logits, int V, int nc,
                                                  const int32_t *__restrict__ off,
                                                  const float *__restrict__ temperature, const float *__restrict__ top_p,
                                                  const int32_t *__restrict__ top_k, const float *__restrict__ pmax,
                                                  uint32_t *__restrict__ st_prefix, unsigned long long *__restrict__ st_above,
                                                  uint32_t *__restrict__ st_cabove, unsigned long long *__restrict__ st_total,
                                                  uint32_t *__restrict__ kkey, unsigned long long *__restrict__ kmass,
                                                  uint32_t *__restrict__ nuc_key, double *__restrict__ nuc_S,
                                                  int32_t *__restrict__ nuc_near, const int32_t *__restrict__ done, int vec) {
  constexpr int SHIFT = (LEVEL == 0) ? 21 : (LEVEL == 1 ? 10 : 0), BITS = (LEVEL == 2) ? 10 : 11;
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63;   // grid = (largest gamma + 1, requests)
  if ((int)blockIdx.x > off[b + 1] - off[b]) return;
  const int r = off[b] + b + blockIdx.x;
  if (done && done[r]) return;   // k_nucleus_top has settled this row
  const float T = temperature[b], tp = top_p ? top_p[b] : 1.f;
  const int tk = top_k ? top_k[b] : 0;
  const bool use_k = T > 0.f && tk > 0 && tk < V, use_p = T > 0.f && tp < 1.f;
  if (MODE == 1) {
    if (!use_k) {
      if (LEVEL == 0 && tid == 0) kkey[r] = 0u;
      return;
    }
  } else if (!use_p) {  // no top-p for this row: its final cut is the top-k one, if any
    if (LEVEL == 0 && tid == 0) {
      const uint32_t kk = use_k ? kkey[r] : 0u;
      nuc_key[r] = kk;
      nuc_S[r] = kk ? (double)kmass[r] / kNucScale : -1.0;
      nuc_near[r] = 0;
    }
    return;
  }
  __shared__ unsigned long long hist[FSV_NUC_BINS];
  __shared__ uint32_t hcnt[(MODE == 1) ? FSV_NUC_BINS : 1];
  __shared__ float s_m;
  for (int i = tid; i < FSV_NUC_BINS; i += 1024) {
    hist[i] = 0ull;
    if (MODE == 1) hcnt[i] = 0u;
  }
  if (tid < 64) {
    float mx = -INFINITY;
    for (int c = lane; c < nc; c += 64) mx = fmaxf(mx, pmax[(size_t)r * nc + c]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (lane == 0) s_m = mx;
  }
  __syncthreads();
  const float m = s_m;
  const exp_scale k = make_exp_scale(kLog2e / (double)T);
  const uint32_t prefix = (LEVEL > 0) ? st_prefix[r] : 0u;
  const uint32_t lowkey = (MODE == 0 && use_k) ? kkey[r] : 0u;   // top-p works on what the top-k cut kept
  const LT *row = logits + (size_t)r * V;
  auto add8 = [&](int i0, const float (&v)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (i0 + j >= V) continue;   // ids beyond the vocabulary are not tokens (they would count for top-k)
      const uint32_t key = okey(v[j]);
      if (LEVEL > 0 && (key >> (SHIFT + BITS)) != prefix) continue;
      if (MODE == 0 && key < lowkey) continue;
      const unsigned long long q = (unsigned long long)((double)exp_scaled(v[j] - m, k) * kNucScale + 0.5);
      const uint32_t bin = (key >> SHIFT) & ((1u << BITS) - 1u);
      if (q) atomicAdd(&hist[bin], q);
      if (MODE == 1) atomicAdd(&hcnt[bin], 1u);
    }
  };
  // Rounds of U loads per thread issued back to back, without a branch between them (a branch per load makes the wave
  // wait for each load before the next, and the pass then runs at one memory round trip per 8192 ids of the row); the
  // ragged end of the row takes the guarded loads one by one.
  constexpr int U = 4, STEP = 1024 * 8;
  int base = tid * 8;
  if (vec) {
    for (; base + (U - 1) * STEP + 8 <= V; base += U * STEP) {
      float v[U][8];
#pragma unroll
      for (int u = 0; u < U; ++u) loader<LT>::load8_fast(row, base + u * STEP, v[u]);
#pragma unroll
      for (int u = 0; u < U; ++u) add8(base + u * STEP, v[u]);
    }
  }
  for (; base < V; base += STEP) {
    float v[8];
    loader<LT>::load8(row, base, V, vec != 0, -INFINITY, v);
    add8(base, v);
  }
  __syncthreads();
  if (tid >= 64) return;
  // lane l owns the 32 digit values below (64 - l) * 32, the highest values in lane 0: masses above each lane's group
  constexpr int PER = FSV_NUC_BINS / 64;
  unsigned long long mine = 0ull;
  uint32_t minec = 0u;
  const int top = (63 - lane) * PER + PER - 1;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    mine += hist[top - i];
    if (MODE == 1) minec += hcnt[top - i];
  }
  unsigned long long incl = mine;
  uint32_t inclc = minec;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long t = __shfl_up(incl, off, 64);
    const uint32_t tc = __shfl_up(inclc, off, 64);
    if (lane >= off) { incl += t; inclc += tc; }
  }
  const unsigned long long above0 = (LEVEL == 0) ? 0ull : st_above[r];
  const unsigned long long before = above0 + (incl - mine);  // mass strictly above this lane's group
  if (MODE == 1) {
    const uint32_t cabove0 = (LEVEL == 0) ? 0u : st_cabove[r];
    const uint32_t beforec = cabove0 + (inclc - minec);     // tokens strictly above this lane's group
    const unsigned long long ballot = __ballot(beforec + minec >= (uint32_t)tk);
    // level 0 always has a crossing (tk < V tokens are counted); deeper levels were chosen because they cross
    const int pick_lane = ballot ? (int)__builtin_ctzll(ballot) : 63;
    if (lane != pick_lane) return;
    unsigned long long acc = before;
    uint32_t accc = beforec;
    int digit = top - (PER - 1);
    for (int i = 0; i < PER; ++i) {
      if (accc + hcnt[top - i] >= (uint32_t)tk || i == PER - 1) { digit = top - i; break; }
      accc += hcnt[top - i];
      acc += hist[top - i];
    }
    const uint32_t newprefix = (prefix << BITS) | (uint32_t)digit;
    if (!LAST) {
      st_prefix[r] = newprefix;
      st_above[r] = acc;
      st_cabove[r] = accc;
    } else {
      kkey[r] = newprefix << SHIFT;
      kmass[r] = acc + hist[digit];
    }
    return;
  }
  unsigned long long total = (LEVEL == 0) ? __shfl(incl, 63, 64) : st_total[r];
  const double target = (double)tp * (double)total;
  const bool crosses = (double)(before + mine) >= target;
  const unsigned long long ballot = __ballot(crosses);
  // rounding cannot leave the ballot empty at level 0 (the last lane holds the total); at deeper levels the digit group
  // was chosen because it crosses, so some lane does as well; the guard only keeps the index in range
  const int pick_lane = ballot ? (int)__builtin_ctzll(ballot) : 63;
  if (lane != pick_lane) return;
  unsigned long long acc = before;
  int digit = top - (PER - 1);
  for (int i = 0; i < PER; ++i) {
    const unsigned long long hbin = hist[top - i];
    if ((double)(acc + hbin) >= target || i == PER - 1) { digit = top - i; break; }
    acc += hbin;
  }
  const uint32_t newprefix = (prefix << BITS) | (uint32_t)digit;
  if (!LAST) {
    st_prefix[r] = newprefix;
    st_above[r] = acc;
    if (LEVEL == 0) st_total[r] = total;
  } else {
    const unsigned long long kept = acc + hist[digit];
    nuc_key[r] = newprefix << SHIFT;
    nuc_S[r] = (double)kept / kNucScale;
    const double lo = target - (double)acc, hi = (double)kept - target;
    nuc_near[r] = (fmin(lo, hi) < 1e-6 * (double)total) ? 1 : 0;
  }
}

// The same selection for bf16 logits in ONE pass whenever the cut lies near the top of the row, which is where a top-p
// or top-k cut lies in practice: only the W highest digit values at and below the row maximum's digit (W = 4: one binade
// of the logit, tried first; W = 8: two binades, for the rows the first try leaves) get histogram bins, 32 each (a bf16 key has five bits below the digit, so a bin is one key: the second
// level comes for free).  Every other token is dismissed after a look at its key: the pass needs no exponential and no
// LDS atomic for it, which is what bounds the full pass.  The row's total mass, against which top_p is measured, is not
// summed again either: it is the normaliser the statistics pass already left (or, after a top-k cut, the mass that
// cut kept).  That total differs from the integer sum the full passes form by the rounding of a floating-point sum
// (1e-7 relative); the rows where that could matter are the ones within 1e-6 of the cut, which are flagged in any case.
// A row whose cut lies below the window is left to the full passes (done[r] = 0).
template <int MODE, int W, bool FIRST>
__global__ __launch_bounds__(1024) void k_nucleus_top(const uint16_t *__restrict__ logits, int V, int nc,
                                                      const int32_t *__restrict__ off,
                                                      const float *__restrict__ temperature,
                                                      const float *__restrict__ top_p, const int32_t *__restrict__ top_k,
                                                      const float *__restrict__ pmax, const double *__restrict__ psum,
                                                      uint32_t *__restrict__ kkey, unsigned long long *__restrict__ kmass,
                                                      uint32_t *__restrict__ nuc_key, double *__restrict__ nuc_S,
                                                      int32_t *__restrict__ nuc_near, int32_t *__restrict__ done, int vec) {
  constexpr int FB = 32;
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
  if ((int)blockIdx.x > off[b + 1] - off[b]) return;
  const int r = off[b] + b + blockIdx.x;
  if (!FIRST && done[r]) return;   // settled by the narrower window
  const float T = temperature[b], tp = top_p ? top_p[b] : 1.f;
  const int tk = top_k ? top_k[b] : 0;
  const bool use_k = T > 0.f && tk > 0 && tk < V, use_p = T > 0.f && tp < 1.f;
  if (MODE == 1) {
    if (!use_k) {
      if (tid == 0) { kkey[r] = 0u; done[r] = 1; }
      return;
    }
  } else if (!use_p) {  // no top-p for this row: its final cut is the top-k one, if any
    if (tid == 0) {
      const uint32_t kk = use_k ? kkey[r] : 0u;
      nuc_key[r] = kk;
      nuc_S[r] = kk ? (double)kmass[r] / kNucScale : -1.0;
      nuc_near[r] = 0;
      done[r] = 1;
    }
    return;
  }
  __shared__ unsigned long long hist[W * FB];
  __shared__ uint32_t hcnt[(MODE == 1) ? W * FB : 1];
  __shared__ float s_m;
  __shared__ double s_total;
  for (int i = tid; i < W * FB; i += 1024) {
    hist[i] = 0ull;
    if (MODE == 1) hcnt[i] = 0u;
  }
  if (tid < 64) {   // the row's maximum and normaliser from the per-chunk statistics (chunks in lanes, 64 at a time)
    float mx = -INFINITY;
    for (int c = lane; c < nc; c += 64) mx = fmaxf(mx, pmax[(size_t)r * nc + c]);
#pragma unroll
    for (int o2 = 32; o2 > 0; o2 >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o2, 64));
    double term = 0.0;
    if (MODE == 0 && !use_k) {
      const double invT = 1.0 / (double)T;
      for (int c = lane; c < nc; c += 64) {
        const float pm = pmax[(size_t)r * nc + c];
        term += psum[(size_t)r * nc + c] * ((pm == mx) ? 1.0 : exp(((double)pm - (double)mx) * invT));
      }
#pragma unroll
      for (int o2 = 32; o2 > 0; o2 >>= 1) term += __shfl_xor(term, o2, 64);
    }
    if (lane == 0) {
      s_m = mx;
      s_total = (MODE == 0) ? (use_k ? (double)kmass[r] : term * kNucScale) : 0.0;
    }
  }
  __syncthreads();
  const float m = s_m;
  const exp_scale k = make_exp_scale(kLog2e / (double)T);
  const uint32_t d0 = okey(m) >> 21;                              // the row's highest digit
  const uint32_t lowkey = (MODE == 0 && use_k) ? kkey[r] : 0u;   // top-p works on what the top-k cut kept
  const uint16_t *row = logits + (size_t)r * V;
  // the lowest value inside the window (and, after a top-k cut, inside that cut): the value whose key is the window's
  // lowest key; keys below 2^31 belong to negative values (the key is the complement of their bits)
  const uint32_t wlow = (d0 >= (uint32_t)(W - 1)) ? ((d0 - (uint32_t)(W - 1)) << 21) : 0u, klow = max(wlow, lowkey);
  float vlow = __uint_as_float((klow & 0x80000000u) ? (klow & 0x7FFFFFFFu) : ~klow);
  if (!(vlow == vlow)) vlow = (klow & 0x80000000u) ? INFINITY : -INFINITY;   // (keys of NaN patterns: only when the row holds them)
  // Eight ids of a thread at a time: a bit per id that falls into the window, then the wave works through the set bits,
  // every lane on its next one, so that the exponential and the atomics are issued about as often as the busiest lane
  // has window tokens among its eight, not once per id.
  auto add8 = [&](int i0, const float (&v)[8], auto in_range) {
    uint32_t mask = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      bool ok = v[j] >= vlow;   // the key order is the order of the values: one comparison places a token
      if (!decltype(in_range)::value) ok = ok && (i0 + j < V);   // ids beyond the vocabulary are not tokens
      mask |= ok ? (1u << j) : 0u;
    }
    while (__any(mask != 0u)) {
      if (mask) {
        const int j = __builtin_ctz(mask);
        mask &= mask - 1u;
        const float a0 = (j & 1) ? v[1] : v[0], a1 = (j & 1) ? v[3] : v[2], a2 = (j & 1) ? v[5] : v[4], a3 = (j & 1) ? v[7] : v[6];
        const float b0 = (j & 2) ? a1 : a0, b1 = (j & 2) ? a3 : a2;
        const float val = (j & 4) ? b1 : b0;
        const uint32_t key = okey(val);
        const unsigned long long q = (unsigned long long)((double)exp_scaled(val - m, k) * kNucScale + 0.5);
        const uint32_t idx = (d0 - (key >> 21)) * FB + ((key >> 16) & (FB - 1));
        if (q) atomicAdd(&hist[idx], q);
        if (MODE == 1) atomicAdd(&hcnt[idx], 1u);
      }
    }
  };
  constexpr int U = 4, STEP = 1024 * 8;
  int base = tid * 8;
  if (vec) {
    for (; base + (U - 1) * STEP + 8 <= V; base += U * STEP) {
      float v[U][8];
#pragma unroll
      for (int u = 0; u < U; ++u) loader<uint16_t>::load8_fast(row, base + u * STEP, v[u]);
#pragma unroll
      for (int u = 0; u < U; ++u) add8(base + u * STEP, v[u], std::true_type{});
    }
  }
  for (; base < V; base += STEP) {
    float v[8];
    loader<uint16_t>::load8(row, base, V, vec != 0, -INFINITY, v);
    add8(base, v, std::false_type{});
  }
  __syncthreads();
  if (tid >= 64) return;
  // lane l < W owns the window's digit d0 - l: the highest keys in lane 0
  unsigned long long mine = 0ull;
  uint32_t minec = 0u;
  if (lane < W) {
#pragma unroll
    for (int f = 0; f < FB; ++f) {
      mine += hist[lane * FB + f];
      if (MODE == 1) minec += hcnt[lane * FB + f];
    }
  }
  unsigned long long incl = mine;
  uint32_t inclc = minec;
#pragma unroll
  for (int o2 = 1; o2 < W; o2 <<= 1) {
    const unsigned long long t = __shfl_up(incl, o2, 64);
    const uint32_t tc = __shfl_up(inclc, o2, 64);
    if (lane >= o2) { incl += t; inclc += tc; }
  }
  const unsigned long long before = incl - mine;   // mass strictly above this lane's digit
  const uint32_t beforec = inclc - minec;
  const double total = s_total, target = (double)tp * total;
  const bool crosses = (MODE == 1) ? (beforec + minec >= (uint32_t)tk) : ((double)(before + mine) >= target);
  const unsigned long long ballot = __ballot(crosses && lane < W && lane <= (int)d0);   // digits below zero do not exist
  if (!ballot || (MODE == 0 && !(total > 0.0))) {   // the cut lies below the window: the full passes take the row
    if (lane == 0) done[r] = 0;
    return;
  }
  if (lane != (int)__builtin_ctzll(ballot)) return;
  unsigned long long acc = before;
  uint32_t accc = beforec;
  int fsel = 0;
  for (int f = FB - 1; f >= 0; --f) {
    const unsigned long long hbin = hist[lane * FB + f];
    const bool hit = (MODE == 1) ? (accc + hcnt[lane * FB + f] >= (uint32_t)tk) : ((double)(acc + hbin) >= target);
    if (hit || f == 0) { fsel = f; break; }
    acc += hbin;
    if (MODE == 1) accc += hcnt[lane * FB + f];
  }
  const uint32_t cut = ((d0 - (uint32_t)lane) << 21) | ((uint32_t)fsel << 16);
  const unsigned long long kept = acc + hist[lane * FB + fsel];
  if (MODE == 1) {
    kkey[r] = cut;
    kmass[r] = kept;
  } else {
    nuc_key[r] = cut;
    nuc_S[r] = (double)kept / kNucScale;
    const double lo = target - (double)acc, hi = (double)kept - target;
    nuc_near[r] = (fmin(lo, hi) < 1e-6 * total) ? 1 : 0;
  }
  done[r] = 1;
}

#define FSV_MAX_GAMMA 16

template <typename LT>
__device__ inline double thread_masses(const LT *lrow, const float *qrow, int i0, int V, bool lvec, bool qvec,
                                       float m, exp_scale k, double invS, bool residual, bool fast, uint32_t cutkey,
                                       double (&mass)[8]) {
  float lv[8], qv[8];
  if (fast) {  // the caller has checked alignment and range for the whole sub-block
    loader<LT>::load8_fast(lrow, i0, lv);
    if (residual) loader<float>::load8_fast(qrow, i0, qv);
  } else {
    loader<LT>::load8(lrow, i0, V, lvec, -INFINITY, lv);
    if (residual) loader<float>::load8(qrow, i0, V, qvec, 0.f, qv);
  }
  double t = 0.0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    double p = (okey(lv[j]) >= cutkey) ? (double)exp_scaled(lv[j] - m, k) * invS : 0.0;  // cutkey 0: nothing is cut
    if (residual) {
      p -= (double)qv[j];
      p = p > 0.0 ? p : 0.0;
    }
    mass[j] = p;
    t += p;
  }
  return t;
}

#define FSV_MAX_NSB 160

// Acceptance tests, masses and token selection of one request.  grid = (ceil(sub-blocks / 4), requests).
//
// Phase 1, every block: the acceptance tests.  Wave w combines the per-chunk statistics of rows w, w+4, ... (one chunk per
//   lane: row max with the lowest id attaining it, then the sum of the rescaled chunk sums over a fixed shuffle tree; the
//   loads of all of a wave's rows are issued together); then thread i tests draft i+1 from two gathered scalars, and
//   thread 0 takes the accepted prefix.  Every block of the request repeats this (a few KB from L2) instead of waiting
//   for a launch of its own.
// Phase 2: wave w of block x takes sub-block 4x + w of the row the emitted token is drawn from (the residual
//   max(0, p - q) after a rejection, p itself when every draft passed): four passes of 512 ids, mass to bsum.
// Phase 3: the blocks of a request take a ticket; the one that draws the last ticket adds the sub-block masses up in
//   sub-block order, finds the sub-block and the id by inverse CDF, writes every output of the request (accepted length,
//   token, flags, rollback) and clears the ticket for the next call.
template <typename LT>
__global__ __launch_bounds__(256) void k_decide(
    const LT *__restrict__ logits, int V, int nc, int nsb, const int32_t *__restrict__ off,
    const int32_t *__restrict__ draft, const float *__restrict__ q, const float *__restrict__ u_acc,
    const float *__restrict__ u_smp, const float *__restrict__ temperature, const float *__restrict__ pmax,
    const double *__restrict__ psum, const int32_t *__restrict__ parg, const uint32_t *__restrict__ nuc_key,
    const double *__restrict__ nuc_S, const int32_t *__restrict__ nuc_near, double *__restrict__ bsum,
    int32_t *__restrict__ ticket, int32_t *__restrict__ accepted_len, int32_t *__restrict__ next_token,
    uint32_t *__restrict__ flags, const int32_t *__restrict__ seq_lens, int32_t *__restrict__ new_seq_lens,
    int32_t *__restrict__ pages_released, int page_size, int lvec, int qvec) {
  const int b = blockIdx.y, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int o = off[b], gamma_all = off[b + 1] - o, gamma = min(gamma_all, FSV_MAX_GAMMA), rs = o + b;
  const float T = temperature[b];
  const double invT = (T > 0.f) ? 1.0 / (double)T : 0.0;
  __shared__ double s_m[FSV_MAX_GAMMA + 1], s_S[FSV_MAX_GAMMA + 1];
  __shared__ int s_arg[FSV_MAX_GAMMA + 1], s_acc[FSV_MAX_GAMMA], s_near[FSV_MAX_GAMMA];
  __shared__ int s_tau, s_last;
  __shared__ uint32_t s_flags;
  auto rollback = [&](int tau) {  // KV rollback: keep [0, L+1+tau)
    if (seq_lens && new_seq_lens) {
      const int L = seq_lens[b], keep = L + 1 + tau, written = L + 1 + gamma_all;
      new_seq_lens[b] = keep;
      if (pages_released) pages_released[b] = (written + page_size - 1) / page_size - (keep + page_size - 1) / page_size;
    }
  };

  // ---- phase 1: acceptance ----
  {
    constexpr int RW = (FSV_MAX_GAMMA + 1 + 3) / 4;   // rows a wave combines at most
    float pm[RW];
    double ps[RW];
    int pa[RW];
#pragma unroll
    for (int j = 0; j < RW; ++j) {
      const int i = w + 4 * j;
      const bool live = i <= gamma && lane < nc;
      const size_t at = (size_t)(rs + min(i, gamma)) * nc + min(lane, nc - 1);
      pm[j] = live ? pmax[at] : -INFINITY;
      ps[j] = live ? psum[at] : 0.0;
      pa[j] = live ? parg[at] : INT_MAX;
    }
#pragma unroll
    for (int j = 0; j < RW; ++j) {
      const int i = w + 4 * j;
      if (i > gamma) continue;   // wave-uniform
      float mx = pm[j];
      int ai = pa[j];
#pragma unroll
      for (int sh = 32; sh > 0; sh >>= 1) {
        const float om = __shfl_xor(mx, sh, 64);
        const int oi = __shfl_xor(ai, sh, 64);
        if (om > mx || (om == mx && oi < ai)) { mx = om; ai = oi; }
      }
      double term = 0.0;
      if (T > 0.f && lane < nc) term = ps[j] * ((pm[j] == mx) ? 1.0 : exp(((double)pm[j] - (double)mx) * invT));
#pragma unroll
      for (int sh = 32; sh > 0; sh >>= 1) term += __shfl_xor(term, sh, 64);
      if (lane == 0) {
        s_m[i] = (double)mx;
        // a row cut to its most probable tokens is normalised by the kept mass; its cut key masks the tokens outside
        s_S[i] = (nuc_S && nuc_S[rs + i] >= 0.0) ? nuc_S[rs + i] : term;
        s_arg[i] = ai;
      }
    }
  }
  __syncthreads();
  if (T <= 0.f) {  // greedy (Alg. 2): accept while the draft equals the argmax, emit the argmax
    if (blockIdx.x == 0 && tid == 0) {
      int tau = 0;
      while (tau < gamma && draft[o + tau] == s_arg[tau]) ++tau;
      accepted_len[b] = tau;
      next_token[b] = s_arg[tau];
      flags[b] = 0u;
      rollback(tau);
    }
    return;
  }
  if (tid < gamma) {  // row rs + tid scores draft tid + 1
    const int r = rs + tid, d = min(max(draft[o + tid], 0), V - 1);
    float lv;
    if constexpr (sizeof(LT) == 2) lv = __uint_as_float((uint32_t)logits[(size_t)r * V + d] << 16);
    else lv = logits[(size_t)r * V + d];
    const bool kept = !nuc_key || okey(lv) >= nuc_key[r];
    const double p = kept ? exp(((double)lv - s_m[tid]) * invT) / s_S[tid] : 0.0;
    const double qd = (double)q[(size_t)(o + tid) * V + d];
    const double ratio = p / qd;
    double a = (ratio >= 1.0) ? 1.0 : ratio;
    if (!(a == a)) a = 0.0;
    const double u = (double)u_acc[o + tid];
    s_acc[tid] = (u < a) ? 1 : 0;
    s_near[tid] = (fabs(u - a) < 1e-4) ? 1 : 0;
  }
  __syncthreads();
  if (tid == 0) {
    int tau = 0;
    while (tau < gamma && s_acc[tau]) ++tau;
    uint32_t f = (tau < gamma) ? 4u : 0u;
    for (int i = 0; i < gamma && i <= tau; ++i) f |= s_near[i] ? 1u : 0u;
    if (nuc_near)
      for (int i = 0; i <= tau; ++i) f |= nuc_near[rs + i] ? 8u : 0u;   // rows 0..tau are the ones the outcome rests on
    s_tau = tau;
    s_flags = f;
  }
  __syncthreads();
  const int tau = s_tau;
  bool residual = tau < gamma;
  const double m = s_m[tau], invS = 1.0 / s_S[tau];
  const uint32_t cutkey = nuc_key ? nuc_key[rs + tau] : 0u;
  const exp_scale k = make_exp_scale(kLog2e / (double)T);
  const LT *lrow = logits + (size_t)(rs + tau) * V;
  const float *qrow = residual ? q + (size_t)(o + tau) * V : nullptr;

  // ---- phase 2: mass of this wave's sub-block ----
  {
    const int sb = blockIdx.x * 4 + w;
    if (sb < nsb) {
      double tot = 0.0;
      const bool fast = lvec && qvec && (sb + 1) * FSV_SBK <= V;  // wave-uniform
#pragma unroll
      for (int part = 0; part < FSV_SBK / 512; ++part) {
        double mass[8];
        tot += thread_masses<LT>(lrow, qrow, sb * FSV_SBK + part * 512 + lane * 8, V, lvec != 0, qvec != 0, (float)m, k, invS,
                                 residual, fast, cutkey, mass);
      }
#pragma unroll
      for (int sh = 32; sh > 0; sh >>= 1) tot += __shfl_xor(tot, sh, 64);
      // a device-scope atomic store: written through to where every XCD sees it (a plain store would stay in this XCD's L2)
      if (lane == 0)
        __hip_atomic_store(reinterpret_cast<unsigned long long *>(bsum) + (size_t)b * nsb + sb,
                           (unsigned long long)__double_as_longlong(tot), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // ---- phase 3: the last block of the request selects the token ----
  // The masses travel between blocks as device-scope atomics (stores above, loads below), which bypass the non-coherent
  // caches by themselves; what is left to order is completion: every wave waits for its store (a workgroup-scope
  // release is a plain wait on the memory counters), the barrier collects the four waves, and only then is the ticket
  // drawn.  No device-wide fence: that would write back and invalidate the whole L2 of the XCD for every block (measured:
  // 40 us on top of a 30 us kernel).
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (tid == 0)
    s_last = (__hip_atomic_fetch_add(&ticket[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1) ? 1 : 0;
  __syncthreads();
  if (!s_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  __shared__ double s_sb[FSV_MAX_NSB];
  __shared__ double s_w[4];
  __shared__ double s_Z, s_lo;
  __shared__ int s_pick, s_first, s_lastpos;
  for (int sb = tid; sb < nsb; sb += 256)
    s_sb[sb] = __longlong_as_double((long long)__hip_atomic_load(
        reinterpret_cast<const unsigned long long *>(bsum) + (size_t)b * nsb + sb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  if (tid == 0) {
    __hip_atomic_store(&ticket[b], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
    accepted_len[b] = tau;
    rollback(tau);
  }
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
                                   false, false, cutkey, mass);
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
  double t = thread_masses<LT>(lrow, qrow, i0, V, lvec != 0, qvec != 0, (float)m, k, invS, residual, false, cutkey, mass);
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
      flags[b] = (s_flags & (residual ? ~0u : ~4u)) | 2u;
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
    uint32_t f = s_flags;
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
  int gmax = 0;
  for (int i = 0; i < B; ++i) gmax = max(gmax, b->draft_offsets_host[i + 1] - b->draft_offsets_host[i]);
  {
    fsv_prof_scope ps(c, s, FSV_K_SAMPLE_STATS, (double)M * V * sizeof(LT));
    hipLaunchKernelGGL(k_row_stats<LT>, dim3(fsv_ceil_div(nc, 4), gmax + 1, B), dim3(256), 0, s, logits, V, nc,
                       b->draft_offsets, b->temperature, c->pmax, c->psum, c->parg, lvec);
  }
  // Top-k / top-p cut: only when some request asks for it; one pass over every logits row per key digit and stage.
  bool any_k = false, any_p = false;
  for (int i = 0; i < B; ++i) {
    const bool sampled = !b->temperature_host || b->temperature_host[i] > 0.f;
    any_p |= sampled && b->top_p && b->top_p_host && b->top_p_host[i] < 1.f;
    any_k |= sampled && b->top_k && b->top_k_host && b->top_k_host[i] > 0 && b->top_k_host[i] < V;
  }
  const bool nucleus = any_k || any_p;
  if (nucleus) {
    const int levels = (sizeof(LT) == 2) ? 2 : 3;
    const int passes = (any_k ? levels : 0) + 1 + (any_p ? levels - 1 : 0);
    fsv_prof_scope ps(c, s, FSV_K_SAMPLE_NUCLEUS, (double)M * V * sizeof(LT) * passes);
    // bf16 logits: one windowed pass settles the rows whose cut lies near the top of the row (all of them in practice);
    // the full passes then find every row done and return at once.  fp32 logits take the full passes.
    // (FSV_NUCLEUS_FULL=1 in the environment sends every row through the digit-by-digit passes: a test compares the two)
    const char *full_env = getenv("FSV_NUCLEUS_FULL");
    const bool windowed = sizeof(LT) == 2 && !(full_env && full_env[0] == '1');
    int32_t *done = windowed ? c->nuc_done : nullptr;
#define FSV_NUC(LEVEL, LAST, MODE)                                                                                     \
  hipLaunchKernelGGL((k_nucleus<LT, LEVEL, LAST, MODE>), dim3(gmax + 1, B), dim3(1024), 0, s, logits, V, nc,             \
                     b->draft_offsets, b->temperature, b->top_p, b->top_k, c->pmax, c->nuc_prefix, c->nuc_above,          \
                     c->nuc_cabove, c->nuc_total, c->nuc_kkey, c->nuc_kmass, c->nuc_key, c->nuc_S, c->nuc_near, done, lvec)
#define FSV_NUC_TOP1(MODE, WV, FIRSTV)                                                                                 \
  hipLaunchKernelGGL((k_nucleus_top<MODE, WV, FIRSTV>), dim3(gmax + 1, B), dim3(1024), 0, s, (const uint16_t *)logits,  \
                     V, nc, b->draft_offsets, b->temperature, b->top_p, b->top_k, c->pmax, c->psum, c->nuc_kkey,        \
                     c->nuc_kmass, c->nuc_key, c->nuc_S, c->nuc_near, c->nuc_done, lvec)
#define FSV_NUC_TOP(MODE)                                                                                              \
  if (windowed) {                                                                                               \
    FSV_NUC_TOP1(MODE, 4, true);                                                                                       \
    FSV_NUC_TOP1(MODE, 8, false);                                                                                      \
  }
    if (any_k) {
      FSV_NUC_TOP(1);
      FSV_NUC(0, false, 1);
      if (sizeof(LT) == 2) {
        FSV_NUC(1, true, 1);
      } else {
        FSV_NUC(1, false, 1);
        FSV_NUC(2, true, 1);
      }
    }
    FSV_NUC_TOP(0);
    FSV_NUC(0, false, 0);   // also settles the rows that take the top-k cut (or none) as their final one
    if (any_p) {
      if (sizeof(LT) == 2) {
        FSV_NUC(1, true, 0);
      } else {
        FSV_NUC(1, false, 0);
        FSV_NUC(2, true, 0);
      }
    }
#undef FSV_NUC_TOP
#undef FSV_NUC_TOP1
#undef FSV_NUC
  }
  {
    fsv_prof_scope ps(c, s, FSV_K_SAMPLE_DECIDE, (double)B * V * (sizeof(LT) + 4));
    hipLaunchKernelGGL(k_decide<LT>, dim3(fsv_ceil_div(nsb, 4), B), dim3(256), 0, s, logits, V, nc, nsb, b->draft_offsets,
                       b->draft_tokens, b->draft_probs, b->u_accept, b->u_sample, b->temperature, c->pmax, c->psum, c->parg,
                       nucleus ? c->nuc_key : nullptr, nucleus ? c->nuc_S : nullptr, nucleus ? c->nuc_near : nullptr, c->bsum,
                       c->sel_ticket, acc, r->next_token, r->flags, with_rollback ? b->seq_lens : nullptr,
                       with_rollback ? r->new_seq_lens : nullptr, with_rollback ? r->pages_released : nullptr,
                       c->d.page_size, lvec, qvec);
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

// ---------------------------------------------------------------------------------------------
// fsv_sample_static: the accept / resample step for callers that cannot allocate device memory.
// ---------------------------------------------------------------------------------------------
// The sampler's workspace (row map, per-chunk statistics, per-sub-block masses, nucleus state) lives in a device array
// of fixed size that is part of the library's code object: every GPU the library runs on holds its own copy at its own
// address for the life of the process.  The array's name is only a host-side handle; the address kernels can use is
// asked for once per device (hipGetSymbolAddress, with that device current) and kept.
#define FSV_STATIC_MAX_BATCH 128
#define FSV_STATIC_MAX_ROWS 1024
#define FSV_STATIC_MAX_NSB 160                                            /* vocabulary <= 160 * 2048 = 327680 */
#define FSV_STATIC_MAX_NC ((FSV_STATIC_MAX_NSB + FSV_SPC - 1) / FSV_SPC)
#define FSV_STATIC_BYTES (1u << 20)

static __device__ __align__(256) unsigned char scratch[FSV_STATIC_BYTES];

namespace {

struct static_slot {
  bool ready = false;
  fsv_ctx ctx;   // a context whose workspace pointers point into this device's copy of `scratch`; owns nothing
};
constexpr int kMaxDevices = 64;
static_slot *g_slots[kMaxDevices] = {};
std::mutex g_static_mu;

// Carve the workspace out of the array (256-byte aligned pieces, sized for the maxima above).  Returns false if it
// does not fit, which would be a mistake in the constants above.
bool carve_static(fsv_ctx &c, unsigned char *base) {
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void *p = base + off;
    off += (bytes + 255) & ~(size_t)255;
    return p;
  };
  const size_t R = FSV_STATIC_MAX_ROWS, B = FSV_STATIC_MAX_BATCH, NC = FSV_STATIC_MAX_NC, NSB = FSV_STATIC_MAX_NSB;
  c.row_req = (int32_t *)take(4 * R); c.row_idx = (int32_t *)take(4 * R); c.row_pos = (int32_t *)take(4 * R);
  c.row_tok = (int32_t *)take(4 * R);
  c.pmax = (float *)take(4 * R * NC); c.psum = (double *)take(8 * R * NC); c.parg = (int32_t *)take(4 * R * NC);
  c.bsum = (double *)take(8 * B * NSB);
  c.acc_scratch = (int32_t *)take(4 * B);
  c.nuc_prefix = (uint32_t *)take(4 * R); c.nuc_key = (uint32_t *)take(4 * R);
  c.nuc_above = (unsigned long long *)take(8 * R); c.nuc_total = (unsigned long long *)take(8 * R);
  c.nuc_S = (double *)take(8 * R); c.nuc_near = (int32_t *)take(4 * R);
  c.nuc_cabove = (uint32_t *)take(4 * R); c.nuc_kkey = (uint32_t *)take(4 * R); c.nuc_done = (int32_t *)take(4 * R);
  c.nuc_kmass = (unsigned long long *)take(8 * R);
  c.sel_ticket = (int32_t *)take(4 * B);   // starts at zero with the array and is left at zero by every call
  return off <= FSV_STATIC_BYTES;
}

}  // namespace

extern "C" int fsv_sample_static(int32_t vocab, const void *logits, int32_t logits_dtype, const fsv_batch *b,
                                 const fsv_result *r, void *stream) {
  if (!logits || !b || !r || !r->next_token || !r->flags) return FSV_E_INVALID_ARG;
  if (logits_dtype != FSV_F32 && logits_dtype != FSV_BF16) return FSV_E_INVALID_ARG;
  if (vocab <= 0) return FSV_E_INVALID_ARG;
  if (fsv_ceil_div(vocab, FSV_SBK) > FSV_STATIC_MAX_NSB) return FSV_E_CAPACITY;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return FSV_E_HIP;
  if (dev < 0 || dev >= kMaxDevices) return FSV_E_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_static_mu);   // the per-device context below is shared by every call on that device
  if (!g_slots[dev]) g_slots[dev] = new (std::nothrow) static_slot();   // host memory, once per device
  static_slot *slot = g_slots[dev];
  if (!slot) return FSV_E_HIP;
  if (!slot->ready) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return FSV_E_HIP;
    if (!carve_static(slot->ctx, (unsigned char *)ptr)) return FSV_E_UNSUPPORTED;
    slot->ctx.d.max_batch = FSV_STATIC_MAX_BATCH;
    slot->ctx.d.max_gamma = FSV_MAX_GAMMA;
    slot->ctx.d.page_size = 16;
    slot->ctx.max_rows = FSV_STATIC_MAX_ROWS;
    slot->ready = true;
  }
  fsv_ctx *c = &slot->ctx;
  c->d.vocab = vocab;
  c->nsb = fsv_ceil_div(vocab, FSV_SBK);
  c->nc = fsv_ceil_div(vocab, FSV_CHUNK);
  const int M = fsv_check_batch(c, b, false, true);   // batch <= 128, gamma <= 16, rows <= 1024, pointers, temperatures
  if (M <= 0) return M;
  return fsv_launch_sampler(c, logits, logits_dtype, b, r, M, false, (hipStream_t)stream);
}
