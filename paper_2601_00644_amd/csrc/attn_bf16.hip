// Multi-query paged attention of the FSV_BF16 path (the attention step of the target forward in Alg. 2
// step 2, over the user's restored KV session plus the rows appended in this call, Sec. IV-C).
// Built with -mllvm -amdgpu-mfma-vgpr-form: the MFMA accumulators stay in the architectural registers,
// where the softmax arithmetic reaches them, and the accumulation registers hold the K/V tiles in flight.
#include <hip/hip_ext.h>
#include <math.h>
#include <stdlib.h>

#include "bf16_common.h"

using namespace fsv_bf16;

namespace {

// ---------------------------------------------------------------------------------------------
// Work decomposition.  The keys of request b are cut into tiles of 32 (two pages); a "part" is a run of
// tp_b consecutive tiles, s_b parts per request, chosen so that every part of every request has about the
// same length and parts x kv heads fills the machine once (one wave per part and kv head, about three waves per
// compute unit, every wave resident from the start).  A wave owns its part completely: it streams the K and
// V page tiles of its key range straight from HBM into MFMA operand registers, NB - 1 tiles ahead of their
// use (each byte of the KV stream is read by exactly one wave; all `group` query heads and all gamma+1
// positions share it), forms S^T = K Q^T (rows = keys, so a query row's scores sit in two lanes), does the
// online softmax in registers, and feeds the probabilities back as the B operand of O^T += V^T P^T without
// any shuffle: the V tile is stored in the key order the score accumulators produce.  Waves never talk to
// each other; a request with one part writes its result directly, the others leave (m, l, O) per part for
// k_attn_combine.
//
// Precision: K and V are the bf16 bits of the cache.  The two operands the kernel itself produces for the matrix
// cores are carried as a pair of bf16 values (hi + lo, hi = the nearest bf16, lo = the nearest bf16 of the rest: 16
// significant bits together) and take two MFMAs each: the rotated queries (two planes of the query buffer) and the
// probabilities.  The matrix cores have the time (the kernel waits for HBM), and the result then differs from exact
// arithmetic on the stored K / V only by fp32 accumulation.
//
// K/V loads go through a buffer descriptor over the layer's pool: a load of a tile beyond the wave's range
// gets an offset outside the descriptor, for which the hardware returns zeros without touching memory, so
// the software pipeline needs no branch around its loads and no over-read.

// Pins a value to the accumulation half of the register file.  The K/V tiles in flight are only ever written
// by loads and read by MFMAs, both of which reach that half directly; keeping them there leaves the
// architectural half to the softmax arithmetic and the output accumulators.
#define FSV_IN_AGPR(x) asm("" : "+a"(x))

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// parts of a request with n key tiles when a part of a request with ONE query-row tile should hold about tpw tiles;
// *tp = tiles per part.  A key tile costs a wave more when the request has more query rows (every further row tile
// repeats the score and value products and the softmax arithmetic on the same K/V registers), so such a request is
// cut into shorter parts, by the measured cost ratio w16 / 16: all waves then finish at about the same time.
__device__ __host__ inline int attn_parts(int n, int tpw, int w16, int *tp) {
  tpw = max(1, tpw * 16 / w16);
  const int s0 = (n + tpw - 1) / tpw;
  *tp = (n + s0 - 1) / s0;
  return (n + *tp - 1) / *tp;
}

// part_prefix[b] = parts of requests before b (the merge kernel's index); part_desc[global part] = everything a wave of
// the attention kernel needs to start, in one 48-byte record: request, first tile, tiles, parts of the request, cached
// length, drafts, first row, (pad), and the physical pages of the part's first two tiles -- a wave fetches it with three
// scalar loads and can issue its first K/V loads at once, instead of after a chain of dependent ones
constexpr int kDescInts = 12;
__global__ void k_attn_plan(int B, int tpw, int group, int w2, int w3, const int32_t *__restrict__ seq_lens,
                            const int32_t *__restrict__ off, const int32_t *__restrict__ page_table, int max_pages,
                            int num_pages, int32_t *__restrict__ part_prefix, int32_t *__restrict__ part_desc, int map_cap) {
  if (blockIdx.x != 0) return;
  __shared__ int total;
  if (threadIdx.x == 0) {
    int run = 0;
    for (int b = 0; b < B; ++b) {
      const int L = seq_lens[b], gamma = off[b + 1] - off[b], nk = L + gamma + 1, n = (nk + 31) >> 5;
      const int rtc = (group * (gamma + 1) + 31) >> 5;
      int tp;
      const int s = attn_parts(n, tpw, rtc <= 1 ? 16 : rtc == 2 ? w2 : w3, &tp);
      part_prefix[b] = run;
      for (int p = 0; p < s && run + p < map_cap; ++p) {
        int32_t *d = part_desc + (size_t)(run + p) * kDescInts;
        d[0] = b; d[1] = p * tp; d[2] = min(n, (p + 1) * tp) - p * tp; d[3] = s;
        d[4] = L; d[5] = gamma; d[6] = off[b] + b; d[7] = 0;
      }
      run += s;
    }
    part_prefix[B] = run;
    total = min(run, map_cap);
  }
  __syncthreads();   // the records written above are read back below by other threads of this block
  for (int p = threadIdx.x; p < total; p += blockDim.x) {
    int32_t *d = part_desc + (size_t)p * kDescInts;
    const int b = d[0], t0 = d[1], npg = (d[4] + d[5] + 1 + 15) >> 4;
    const int32_t *pt = page_table + (size_t)b * max_pages;
#pragma unroll
    for (int i = 0; i < 4; ++i) d[8 + i] = min(max(pt[min(2 * t0 + i, npg - 1)], 0), num_pages - 1);
  }
}

template <int HD, int RT, int NB>
__global__ __launch_bounds__(64) void k_attention(
    int Hkv, int group, int rows_cap, const uint4 *__restrict__ qp, size_t q_plane_units,
    const int32_t *__restrict__ part_desc,
    const int32_t *__restrict__ page_table, int max_pages, int num_pages, const uint16_t *__restrict__ kpool,
    const uint16_t *__restrict__ vpool, uint32_t layer_bytes, float *__restrict__ part_o, float *__restrict__ part_ml,
    uint16_t *__restrict__ out, int KBq) {
  constexpr int KS = HD / 16, VC = HD / 32, TILEB = 16 * HD * 2;  // TILEB: bytes of one (page, kv head) tile
  constexpr uint32_t OOB = 0xFFFF0000u;                            // offset no descriptor here reaches
  constexpr int kStream = 2;  // non-temporal: K/V bytes are used once and should not displace the queries and partials in L2
  __shared__ uint4 s_q[2][RT * KS * 64];  // hi and lo planes of the query operand
  const int lane = threadIdx.x, h = lane >> 5, r = lane & 31;
  const int gw = blockIdx.x, pp = gw / Hkv, kvh = gw - pp * Hkv;
  const int4 d0 = *reinterpret_cast<const int4 *>(part_desc + (size_t)pp * kDescInts);
  const int4 d1 = *reinterpret_cast<const int4 *>(part_desc + (size_t)pp * kDescInts + 4);
  const int4 d2 = *reinterpret_cast<const int4 *>(part_desc + (size_t)pp * kDescInts + 8);
  const int b = d0.x, t0 = d0.y, myt = d0.z, nparts = d0.w, L = d1.x, gamma = d1.y, rs = d1.z;
  const int nk = L + gamma + 1, R = group * (gamma + 1);
  const int rtc = min(RT, (R + 31) >> 5);
  const int32_t *pt = page_table + (size_t)b * max_pages;
  const int npg = (nk + 15) >> 4;

  const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc((void *)kpool, 0, layer_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc((void *)vpool, 0, layer_bytes, 0x00020000);
  // lane part of the offsets inside a tile: K operand row = key r (rows 0-15 first page, 16-31 second page)
  const uint32_t klane = (uint32_t)((h * 16 + (r & 15)) * 16), vlane = (uint32_t)((h * 32 + r) * 16);

  bf16x8_t kb[NB][KS], vb[NB][VC][2];
  auto pages_of = [&](int j, int &g0, int &g1) {  // physical pages of the wave's j-th tile (indices kept in range)
    const int p0 = min(2 * (t0 + j), npg - 1), p1 = min(2 * (t0 + j) + 1, npg - 1);
    g0 = min(max(pt[p0], 0), num_pages - 1);
    g1 = min(max(pt[p1], 0), num_pages - 1);
  };
  auto issue = [&](int j, int g0, int g1, bf16x8_t(&kreg)[KS], bf16x8_t(&vreg)[VC][2]) {
    const bool live = j < myt;
    const uint32_t b0 = live ? (uint32_t)(g0 * Hkv + kvh) * TILEB : OOB, b1 = live ? (uint32_t)(g1 * Hkv + kvh) * TILEB : OOB;
    const uint32_t ko = ((r < 16) ? b0 : b1) + klane, v0 = b0 + vlane, v1 = b1 + vlane;
#pragma unroll
    for (int s = 0; s < KS; ++s)
      kreg[s] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(krs, ko + s * 512, 0, kStream));
#pragma unroll
    for (int c = 0; c < VC; ++c) {
      vreg[c][0] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(vrs, v0 + c * 1024, 0, kStream));
      vreg[c][1] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(vrs, v1 + c * 1024, 0, kStream));
    }
  };

  // Queries go from global memory straight into LDS (no staging registers; lane i of a load fills 16-byte unit i
  // of the addressed LDS block, which is the operand order already); rows beyond R hold whatever an earlier call
  // left there: they only feed their own output rows, which are never stored.  The wave waits for them here, before
  // the K/V stream starts: a wait placed after the first tiles were issued would have to drain those as well
  // (loads complete in order), and the pipeline would start empty.  The page ids of the first tiles are fetched by
  // scalar loads meanwhile.
#pragma unroll
  for (int i = 0; i < RT * KS; ++i) {
    if (i / KS >= rtc) continue;
    const uint4 *src = qp + (((size_t)b * RTMAX + i / KS) * Hkv + kvh) * (KS * 64) + (i % KS) * 64 + lane;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)&s_q[0][i * 64], 16, 0, 0);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + q_plane_units),
                                     (__attribute__((address_space(3))) void *)&s_q[1][i * 64], 16, 0, 0);
  }
  int gp0[NB], gp1[NB];   // pages of the first NB tiles: two tiles' worth came with the record
  gp0[0] = d2.x; gp1[0] = d2.y; gp0[1] = d2.z; gp1[1] = d2.w;
#pragma unroll
  for (int s = 2; s < NB; ++s) pages_of(s, gp0[s], gp1[s]);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the queries are in LDS
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < NB - 1; ++s) issue(s, gp0[s], gp1[s], kb[s], vb[s]);
  int g0n = gp0[NB - 1], g1n = gp1[NB - 1];
  __builtin_amdgcn_sched_barrier(0);

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

  auto consume = [&](int j, bf16x8_t(&kreg)[KS], bf16x8_t(&vreg)[VC][2]) {
    asm volatile("" ::: "memory");  // keep the query operand reads inside the loop (hoisted, they cost 32 VGPRs per row tile)
    // The pins sit at the point of use: placed after the loads they would count as a use and make the wave
    // wait for every load at once.
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) FSV_IN_AGPR(kreg[ks]);
#pragma unroll
    for (int c = 0; c < VC; ++c) {
      FSV_IN_AGPR(vreg[c][0]);
      FSV_IN_AGPR(vreg[c][1]);
    }
    const int kbase = (t0 + j) * 32;
    const bool need_mask = kbase + 31 > L;  // every query row sees all keys <= L
    if (kbase + 31 >= nk) {
      // (wave-uniform, the last tile of a request only) Slots beyond the last valid position may never have been written:
      // their probabilities are zero, but 0 * NaN is NaN, so the V values of those keys are cleared before they reach the
      // matrix cores.  Element e of vreg[c][pg] belongs to key kbase + 16 pg + 8 (e / 4) + 4 h + e % 4.
#pragma unroll
      for (int pg = 0; pg < 2; ++pg) {
        uint32_t m4[4];
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) {
          const int key = kbase + 16 * pg + 8 * (dw >> 1) + 4 * h + 2 * (dw & 1);
          m4[dw] = (key < nk ? 0x0000FFFFu : 0u) | (key + 1 < nk ? 0xFFFF0000u : 0u);
        }
#pragma unroll
        for (int c = 0; c < VC; ++c) {
          u32x4_t raw = __builtin_bit_cast(u32x4_t, vreg[c][pg]);
#pragma unroll
          for (int dw = 0; dw < 4; ++dw) raw[dw] &= m4[dw];
          vreg[c][pg] = __builtin_bit_cast(bf16x8_t, raw);
        }
      }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      if (rt >= rtc) continue;
      f32x16_t s;
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 raw = s_q[0][(rt * KS + ks) * 64 + lane], rlo = s_q[1][(rt * KS + ks) * 64 + lane];
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kreg[ks], *reinterpret_cast<bf16x8_t *>(&raw), s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kreg[ks], *reinterpret_cast<bf16x8_t *>(&rlo), s, 0, 0, 0);
      }
      // accumulator v of this lane: key kbase + 8*(v/4) + 4h + v%4, query row rt*32 + r
      float tmax = -INFINITY;
      if (need_mask) {
        const int limit = lim[rt];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = kbase + 8 * (v >> 2) + 4 * h + (v & 3);
          s[v] = (key <= limit) ? s[v] * sc : -INFINITY;
          tmax = fmaxf(tmax, s[v]);
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          s[v] *= sc;
          tmax = fmaxf(tmax, s[v]);
        }
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      // Lazy reference: the running reference m only moves when the tile maximum exceeds it by more than 2^8
      // (probabilities then stay below 256, exact enough in fp32 / bf16), so the accumulators are almost never
      // rescaled; the first tile of a row needs no rescale either (its accumulators are still zero).
      const float mold = mrun[rt];
      const float mnew = (tmax > mold + 8.0f || mold == -INFINITY) ? fmaxf(mold, tmax) : mold;
      const float muse = (mnew == -INFINITY) ? 0.f : mnew;
      const float alpha = __builtin_amdgcn_exp2f(mold - muse);
      const bool rescale = __any(mnew != mold && mold != -INFINITY);
      mrun[rt] = mnew;
      float psum = 0.f;
      bf16x8_t pb[2], pl[2];  // probabilities as hi + lo
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(s[v] - muse);
        psum += p;
        const __bf16 hi = (__bf16)p;
        pb[v >> 3][v & 7] = hi;
        pl[v >> 3][v & 7] = (__bf16)(p - (float)hi);
      }
      lrun[rt] = lrun[rt] * alpha + psum;
      if (rescale) {  // wave-uniform: once the running maxima have settled the accumulators are left alone
#pragma unroll
        for (int c = 0; c < VC; ++c)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[rt][c][v] *= alpha;
      }
#pragma unroll
      for (int c = 0; c < VC; ++c) {
        o[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vreg[c][0], pb[0], o[rt][c], 0, 0, 0);
        o[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vreg[c][1], pb[1], o[rt][c], 0, 0, 0);
        o[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vreg[c][0], pl[0], o[rt][c], 0, 0, 0);
        o[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vreg[c][1], pl[1], o[rt][c], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);  // row tiles one after the other: interleaved, their temporaries add up
    }
  };

  // Step S of an unrolled round consumes buffer S and refills buffer S - 1 (the one consumed just before) with the
  // tile NB - 1 ahead; buffers rotate by name.  Page ids are fetched one step before the loads that use them.
  const int myt_pad = (myt + NB - 1) / NB * NB;
  for (int j = 0; j < myt_pad; j += NB) {
#pragma unroll
    for (int S = 0; S < NB; ++S) {
      issue(j + S + NB - 1, g0n, g1n, kb[(S + NB - 1) % NB], vb[(S + NB - 1) % NB]);
      pages_of(j + S + NB, g0n, g1n);
      __builtin_amdgcn_sched_barrier(0);
      if (j + S < myt) consume(j + S, kb[S], vb[S]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // result of this wave: lane holds, for query row rt*32 + r, features 32c + 8g + 4h + (0..3)
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    if (rt >= rtc) continue;
    const int rr = rt * 32 + r;
    const float ll = lrun[rt] + __shfl_xor(lrun[rt], 32, 64);
    if (rr >= R) continue;
    if (nparts == 1) {
      const float inv = 1.0f / ll;
      const int m = rs + rr / group, col = (kvh * group + rr % group) * HD;
#pragma unroll
      for (int c = 0; c < VC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int e0 = 32 * c + 8 * g;
          // the output is a convex combination of cached values: bounded, so it is handed on in fp16
          const uint32_t lo = f2h2(o[rt][c][4 * g] * inv, o[rt][c][4 * g + 1] * inv);
          const uint32_t hi = f2h2(o[rt][c][4 * g + 2] * inv, o[rt][c][4 * g + 3] * inv);
          *reinterpret_cast<uint2 *>(out + tile_unit(m, col + e0, KBq) * 8 + 4 * h) = make_uint2(lo, hi);
        }
    } else {
      const size_t prow = (size_t)gw * rows_cap + rr;
      if (h == 0) *reinterpret_cast<float2 *>(part_ml + prow * 2) = make_float2(mrun[rt], ll);
      float *dst = part_o + prow * HD + 4 * h;
#pragma unroll
      for (int c = 0; c < VC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4 *>(dst + 32 * c + 8 * g) =
              make_float4(o[rt][c][4 * g], o[rt][c][4 * g + 1], o[rt][c][4 * g + 2], o[rt][c][4 * g + 3]);
    }
  }
}

// merge the parts of requests that have several, in part order.  grid = (kv heads, requests, row groups)
template <int HD>
__global__ __launch_bounds__(256) void k_attn_combine(int Hkv, int group, int rows_cap,
                                                      const int32_t *__restrict__ off,
                                                      const int32_t *__restrict__ part_prefix,
                                                      const float *__restrict__ part_o,
                                                      const float *__restrict__ part_ml, uint16_t *__restrict__ out,
                                                      int KBq) {
  constexpr int TPR = HD / 8, RPB = 256 / TPR;  // threads per row (eight features each), rows per block
  const int b = blockIdx.y, kvh = blockIdx.x, tid = threadIdx.x;
  const int p0 = part_prefix[b], nparts = part_prefix[b + 1] - p0;
  if (nparts <= 1) return;
  const int gamma = off[b + 1] - off[b], rs = off[b] + b, R = group * (gamma + 1);
  const int rr = blockIdx.z * RPB + tid / TPR, e0 = (tid % TPR) * 8;
  if (rr >= R) return;
  const size_t base = ((size_t)p0 * Hkv + kvh) * rows_cap + rr, pstr = (size_t)Hkv * rows_cap;
  // All loads of a batch of parts are issued before the first use: one part per iteration would put a full memory
  // round trip into every step of this short loop.  Up to sixteen parts (the usual case) are merged from one batch,
  // maxima and values fetched together; more take a pass for the maximum and a pass for the sums, eight at a time.
  // The sums always run in part order.
  float mm = -INFINITY, acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, ll = 0.f;
  auto merge = [&](int s0, int n, const float2 *ml, const float4 *a, const float4 *c) {
    for (int u = 0; u < n; ++u) {
      const float f = (s0 + u >= nparts || ml[u].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml[u].x - mm);
      ll += ml[u].y * f;
      acc[0] += a[u].x * f; acc[1] += a[u].y * f; acc[2] += a[u].z * f; acc[3] += a[u].w * f;
      acc[4] += c[u].x * f; acc[5] += c[u].y * f; acc[6] += c[u].z * f; acc[7] += c[u].w * f;
    }
  };
  auto fetch = [&](int s0, int u, float2 &ml, float4 &a, float4 &c) {
    const size_t prow = base + min(s0 + u, nparts - 1) * pstr;
    ml = *reinterpret_cast<const float2 *>(part_ml + prow * 2);
    a = *reinterpret_cast<const float4 *>(part_o + prow * HD + e0);
    c = *reinterpret_cast<const float4 *>(part_o + prow * HD + e0 + 4);
  };
  if (nparts <= 16) {
    float2 ml[16];
    float4 a[16], c[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) fetch(0, u, ml[u], a[u], c[u]);
#pragma unroll
    for (int u = 0; u < 16; ++u) mm = fmaxf(mm, ml[u].x);  // entries beyond nparts repeat the last part
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const float f = (u >= nparts || ml[u].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml[u].x - mm);
      ll += ml[u].y * f;
      acc[0] += a[u].x * f; acc[1] += a[u].y * f; acc[2] += a[u].z * f; acc[3] += a[u].w * f;
      acc[4] += c[u].x * f; acc[5] += c[u].y * f; acc[6] += c[u].z * f; acc[7] += c[u].w * f;
    }
  } else {
    constexpr int U = 8;
    for (int s0 = 0; s0 < nparts; s0 += U) {
      float mv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) mv[u] = part_ml[(base + min(s0 + u, nparts - 1) * pstr) * 2];
#pragma unroll
      for (int u = 0; u < U; ++u) mm = fmaxf(mm, mv[u]);
    }
    for (int s0 = 0; s0 < nparts; s0 += U) {
      float2 ml[U];
      float4 a[U], c[U];
#pragma unroll
      for (int u = 0; u < U; ++u) fetch(s0, u, ml[u], a[u], c[u]);
      merge(s0, U, ml, a, c);
    }
  }
  const float inv = 1.0f / ll;
  uint32_t pk[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) pk[j] = f2h2(acc[2 * j] * inv, acc[2 * j + 1] * inv);
  const int m = rs + rr / group, col = (kvh * group + rr % group) * HD + e0;
  reinterpret_cast<uint4 *>(out)[tile_unit(m, col, KBq)] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
}

constexpr int kAttnWavesPerCu = 3;  // a wave takes most of a SIMD's registers, so at most four fit; three measured best on MI355X

// Size the parts from the host copies of the lengths: the smallest part length for which parts x kv heads
// still fits the machine once (or one part per request when even that does not fit).
int plan_attention(fsv_ctx *c, const fsv_batch *b, fsv_attn_plan *pl) {
  const fsv_model_desc &d = c->d;
  int max_rows = 0;
  long total_tiles = 0;   // in units of the cost of a tile of a request with one query-row tile
  auto w16_of = [&](int g) {
    const int rtc = fsv_ceil_div(c->group * (g + 1), 32);
    return rtc <= 1 ? 16 : rtc == 2 ? c->attn_w2 : c->attn_w3;
  };
  for (int i = 0; i < b->batch; ++i) {
    const int g = b->draft_offsets_host[i + 1] - b->draft_offsets_host[i], nk = b->seq_lens_host[i] + g + 1;
    const int n = fsv_ceil_div(nk, 32);
    max_rows = max(max_rows, c->group * (g + 1));
    total_tiles += ((long)n * w16_of(g) + 15) / 16;
    pl->kv_tokens += nk;
  }
  // One round if it can be had: the smallest part length, up to twice the even share, for which parts x kv heads fit the
  // resident waves.  Otherwise (many requests, or a few very long ones among many short ones) parts of a quarter of the
  // even share, run in several rounds: waves are independent, so the hardware keeps every slot busy and the last round
  // is short.  Keeping whole requests as single parts instead would let the longest request set the kernel's time.
  const int target = c->attn_wave_target;
  auto count = [&](int tpw, bool *split) {
    int parts = 0;
    *split = false;
    for (int i = 0; i < b->batch; ++i) {
      const int g = b->draft_offsets_host[i + 1] - b->draft_offsets_host[i], nk = b->seq_lens_host[i] + g + 1;
      int tp;
      const int s = attn_parts(fsv_ceil_div(nk, 32), tpw, w16_of(g), &tp);
      parts += s;
      *split |= s > 1;
    }
    return parts * d.n_kv_heads;
  };
  const int even = (int)max((long)c->attn_min_tpw, (total_tiles * d.n_kv_heads + target - 1) / target);
  int tpw = 0;
  for (int t = even; t <= 2 * even; ++t) {
    bool sp;
    if (count(t, &sp) <= target) { tpw = t; break; }
  }
  if (!tpw) tpw = max(8, (even + 3) / 4);
  pl->tpw = tpw;
  pl->waves = count(tpw, &pl->split);
  pl->rt = fsv_ceil_div(max_rows, 32);
  if (pl->waves > c->attn_wave_cap) FSV_FAIL(c, FSV_E_CAPACITY, "%d attention parts > %d the workspace holds", pl->waves, c->attn_wave_cap);
  if ((size_t)b->num_pages * d.n_kv_heads * 16 * d.head_dim * 2 > 0xFFFF0000ull)
    FSV_FAIL(c, FSV_E_UNSUPPORTED, "one layer of a KV pool must stay below 4 GiB (%d pages given)", b->num_pages);
  return FSV_OK;
}

int launch_attn_plan(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan &pl, hipStream_t st) {
  hipLaunchKernelGGL(k_attn_plan, dim3(1), dim3(64), 0, st, b->batch, pl.tpw, c->group, c->attn_w2, c->attn_w3, b->seq_lens, b->draft_offsets,
                     b->page_table, c->d.max_pages_per_req, b->num_pages,
                     c->attn_part_prefix, c->attn_part_map, c->attn_wave_cap / c->d.n_kv_heads + 1);
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}

int launch_attention(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan &pl, size_t layer_off, hipStream_t st) {
  const fsv_model_desc &d = c->d;
  const int group = c->group, KBq = d.n_heads * d.head_dim / 16;
  const int rows_cap = group * (d.max_gamma + 1);
  const uint32_t layer_bytes = (uint32_t)((size_t)b->num_pages * d.n_kv_heads * 16 * d.head_dim * 2);
  float *po = (float *)c->attn_part;
  float *pml = po + (size_t)c->attn_wave_cap * rows_cap * d.head_dim;
  uint16_t *out = (uint16_t *)c->buf_att;
  const uint16_t *kl = (const uint16_t *)b->k_pool + layer_off, *vl = (const uint16_t *)b->v_pool + layer_off;
  {
    fsv_prof_scope ps(c, st, FSV_K_ATTENTION, pl.kv_tokens * d.n_kv_heads * d.head_dim * 4.0, true);
#define FSV_ATTN_LAUNCH(HDV, RTV, NBV)                                                                            \
  hipExtLaunchKernelGGL((k_attention<HDV, RTV, NBV>), dim3(pl.waves), dim3(64), 0, st, ps.start(), ps.stop(), 0,   \
                        d.n_kv_heads, group, rows_cap,                                                             \
                     (const uint4 *)c->buf_q, c->q_plane_units, c->attn_part_map, b->page_table, d.max_pages_per_req, b->num_pages,  \
                     kl, vl, layer_bytes, po, pml, out, KBq)
    const bool deep = c->attn_depth >= 3;   // tiles in flight per wave: 2 (one ahead) or 3 (two ahead)
    if (d.head_dim == 128) {
      if (pl.rt <= 1) { if (deep) FSV_ATTN_LAUNCH(128, 1, 3); else FSV_ATTN_LAUNCH(128, 1, 2); }
      else if (pl.rt == 2) { if (deep) FSV_ATTN_LAUNCH(128, 2, 3); else FSV_ATTN_LAUNCH(128, 2, 2); }
      else FSV_ATTN_LAUNCH(128, 3, 2);
    } else {
      if (pl.rt <= 1) { if (deep) FSV_ATTN_LAUNCH(64, 1, 3); else FSV_ATTN_LAUNCH(64, 1, 2); }
      else if (pl.rt == 2) { if (deep) FSV_ATTN_LAUNCH(64, 2, 3); else FSV_ATTN_LAUNCH(64, 2, 2); }
      else { if (deep) FSV_ATTN_LAUNCH(64, 3, 3); else FSV_ATTN_LAUNCH(64, 3, 2); }
    }
#undef FSV_ATTN_LAUNCH
    FSV_HIP(c, hipGetLastError());
  }
  if (pl.split) {
    fsv_prof_scope pc(c, st, FSV_K_ATTN_COMBINE, 0.0);
    const int rpb = 256 / (d.head_dim / 8);
    dim3 cg(d.n_kv_heads, b->batch, fsv_ceil_div(pl.rt * 32, rpb));
    if (d.head_dim == 128)
      hipLaunchKernelGGL((k_attn_combine<128>), cg, dim3(256), 0, st, d.n_kv_heads, group, rows_cap, b->draft_offsets,
                         c->attn_part_prefix, po, pml, out, KBq);
    else
      hipLaunchKernelGGL((k_attn_combine<64>), cg, dim3(256), 0, st, d.n_kv_heads, group, rows_cap, b->draft_offsets,
                         c->attn_part_prefix, po, pml, out, KBq);
    FSV_HIP(c, hipGetLastError());
  }
  return FSV_OK;
}

}  // namespace

int fsv_bf16_attn_plan_host(fsv_ctx *c, const fsv_batch *b, fsv_attn_plan *pl) { return plan_attention(c, b, pl); }

int fsv_bf16_attn_plan_launch(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan *pl, hipStream_t st) {
  return launch_attn_plan(c, b, *pl, st);
}

int fsv_bf16_attn_launch(fsv_ctx *c, const fsv_batch *b, const fsv_attn_plan *pl, size_t layer_off, hipStream_t st) {
  return launch_attention(c, b, *pl, layer_off, st);
}

int fsv_bf16_attn_create(fsv_ctx *c) {
  const fsv_model_desc &d = c->d;
  int wpc = kAttnWavesPerCu;
  c->attn_depth = 2;
  if (const char *e = getenv("FSV_ATTN_TUNE")) {   // "waves per CU,tiles in flight[,w2,w3[,fewest tiles per part]]": measurement knob
    int a = 0, bb = 0, w2 = c->attn_w2, w3 = c->attn_w3, mt = c->attn_min_tpw;
    const int n = sscanf(e, "%d,%d,%d,%d,%d", &a, &bb, &w2, &w3, &mt);
    if (n >= 2 && a >= 1 && a <= 8 && bb >= 2 && bb <= 3) { wpc = a; c->attn_depth = bb; }
    if (n >= 4 && w2 >= 16 && w2 <= 64 && w3 >= w2 && w3 <= 96) { c->attn_w2 = w2; c->attn_w3 = w3; }
    if (n == 5 && mt >= 2 && mt <= 64) c->attn_min_tpw = mt;
  }
  c->attn_wave_target = c->n_cus * wpc;
  c->attn_wave_cap = 4 * c->attn_wave_target + 2 * d.max_batch * d.n_kv_heads;  // multi-round schedules: see plan_attention
  const int rows_cap = c->group * (d.max_gamma + 1);
  c->attn_part_bytes = (size_t)c->attn_wave_cap * rows_cap * (d.head_dim + 2) * 4;
  auto zalloc = [&](void **p, size_t bytes) -> int {
    FSV_HIP(c, hipMalloc(p, bytes));
    FSV_HIP(c, hipMemset(*p, 0, bytes));
    return FSV_OK;
  };
  int rc;
  if ((rc = zalloc(&c->attn_part, c->attn_part_bytes))) return rc;
  if ((rc = zalloc((void **)&c->attn_part_prefix, sizeof(int32_t) * (d.max_batch + 1)))) return rc;
  if ((rc = zalloc((void **)&c->attn_part_map, sizeof(int32_t) * kDescInts * (c->attn_wave_cap / d.n_kv_heads + 1)))) return rc;
  return FSV_OK;
}
