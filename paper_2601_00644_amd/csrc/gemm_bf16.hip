// Weight-streaming 16-bit GEMM (bf16 or fp16 operands, fp32 sums) of the FSV_BF16 path: the dense projections of the target forward (Alg. 2
// step 2) for a few dozen to a few hundred rows, where streaming the weight matrix from HBM is the bound.
// Built with -mllvm -amdgpu-mfma-vgpr-form (accumulators in architectural registers, the weight chunks in
// flight in accumulation registers).
//
// A block is up to four compute waves (the host picks two to four, so that the launch fills the compute units) and NLD
// loader waves.  Compute wave w owns 32 output features (one weight
// tile row) for up to MT*32 batch rows over the block's K range and streams that strip of the re-tiled
// matrix straight from HBM into MFMA operand registers, D chunks of 128 k (D = 1) ahead of its use.  The loader waves
// copy the activation chunks of the same K range from global memory (L2) directly into a three-stage LDS
// ring, two chunks ahead; the compute waves read their B operands from the ring.  Because the activation
// loads are issued by a wave of their own, the compute waves' load counter tracks the weight stream only
// and a wait for the oldest chunk never drains the younger ones.  One barrier per chunk hands a filled
// stage to the compute waves and a consumed one back to the loader.
//
// The strips of consecutive feature tiles lie K / 16 KiB plus a padding of 8 KiB apart: all waves advance through their
// strips in step, and with the strips a power of two apart (256 KiB at K = 4096) their concurrent requests fall on
// the same memory channels; a plain reader with this access pattern gains 9 % from the padding (measured on MI355X).
//
// F16: both operands are fp16 (the projections whose input is a normalised activation or an attention output, which are
// bounded whatever the model and gain three significant bits over bf16 that way).  Their weights were converted from bf16
// at creation, times a power of two per matrix that places the largest weight near 2^13 (the conversion is then exact
// for every weight down to 2^-31 of the largest); the epilogue multiplies the fp32 sums by the inverse power.  Same
// instruction rate, same bytes.
#include <hip/hip_ext.h>
#include <math.h>
#include <stdlib.h>

#include "bf16_common.h"

using namespace fsv_bf16;

namespace {

enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_F32 = 2 };

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;

#define FSV_IN_AGPR(x) asm("" : "+a"(x))
// The barrier as an opaque statement: memory operations do not move across it, and no counter wait is attached.
#define FSV_BARRIER() asm volatile("s_barrier" ::: "memory")

constexpr int KC = 8;     // 16-wide k blocks per chunk (128 contraction elements)
constexpr int NST = 3;    // LDS stages of the activation ring
constexpr int GRAN = 2;   // chunks per 256-element granule of the K cut
constexpr int NLD = 2;    // loader waves per block: two halve the time of the first fills, which matters for the short split-K blocks

// Stores one wave's result: for row tiles mt < mtc of the block starting at tile mt0, lane holds, for batch row
// m = tile*32 + lane%32, features nt*32 + 8*(v/4) + 4*h + v%4 of strip nt.
template <int MT, int EPI, bool F16>
__device__ __forceinline__ void store_strip(f32x16_t (&acc)[MT], void *__restrict__ out, int nt, int mt0, int mtc, int lane,
                                            int h, int split, int M, int Mpad, int N, int KBo, float oscale) {
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (mt >= mtc) continue;
    if constexpr (F16) {   // undo the power of two the weights carry (exact)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mt][v] *= oscale;
    }
    const int m = (mt0 + mt) * 32 + (lane & 31);
    if constexpr (EPI == EPI_PARTIAL) {
      if (m >= M) continue;  // the consumers read rows below M only
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

// Loader wave lw of a block: activation chunk `it` -> LDS stage it % NST, one 1 KiB row of units per instruction; loader
// wave l takes the rows i with i % NLD == l.  Meets 1 + per barriers, as every compute wave of the block does.
template <int MT>
__device__ __forceinline__ void loader_wave(uint4 *lds, const uint4 *__restrict__ Ap, int lw, int lane, int mt0, int mlast,
                                            int KB, int cb0, int per) {
  constexpr int CHU = MT * KC * 64;
  constexpr int PERW = (MT * KC + NLD - 1) / NLD;  // instructions per loader wave and chunk
  auto fill = [&](int it) {
    uint4 *dst = lds + (it % NST) * CHU;
#pragma unroll
    for (int j = 0; j < PERW; ++j) {
      const int i = min(j * NLD + lw, MT * KC - 1);  // (a repeated last row when the split is uneven)
      const int mt = min(i / KC, mlast);
      const uint4 *src = Ap + ((size_t)(mt0 + mt) * KB + (size_t)(cb0 + it) * KC + i % KC) * 64 + lane;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                       (__attribute__((address_space(3))) void *)(dst + i * 64), 16, 0, 0);
    }
  };
  fill(0);
  if (per > 1) {
    fill(1);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PERW) : "memory");  // chunk 0 has landed, chunk 1 may be in flight
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  FSV_BARRIER();
  for (int it = 0; it < per; ++it) {
    // stage (it + 2) % NST was read during step it - 1, which every compute wave left at the last barrier
    if (it + 2 < per) {
      fill(it + 2);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PERW) : "memory");  // chunk it + 1 has landed
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    FSV_BARRIER();
  }
}

template <int MT, int EPI, int D, bool F16, int NCW>
__global__ __launch_bounds__(64 * (NCW + NLD)) void k_gemm(const void *__restrict__ Wp, uint32_t wbytes, const uint4 *__restrict__ Ap,
                                              void *__restrict__ out, int N, int KB, int Mt_total, int M, int Mpad,
                                              int S, int nchunks, int KBo, int NBv, int MB, float oscale, int NT, uint32_t strip_bytes) {
  // strip_bytes: distance between the weight strips of consecutive 32-feature tiles (K / 16 KiB of operands plus padding)
  // NCW: compute waves of the block (the block has NCW + NLD waves); NT: weight strips the matrix holds
  extern __shared__ uint4 lds[];
  constexpr int CHU = MT * KC * 64;  // 16-byte units of one activation chunk
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, h = lane >> 5;
  // Blocks are dealt to the eight XCDs round robin by their linear index, which is decoded as
  // (XCD, row block, split group, feature block) with the row block fastest: the row blocks that need the same
  // weight strip are then neighbours in time on ONE XCD and all but the first find the strip in that XCD's L2
  // (many rows: the weights come from HBM once, not once per row block), and with a multiple of eight splits a
  // split always lands on the same XCD, so every XCD stages only its own K slices of the activation matrix.
  int nblk, split, zb;
  {
    const int L = blockIdx.x, x = L & 7, a = L >> 3;
    zb = a % MB;
    const int a2 = a / MB;
    if ((S & 7) == 0) {
      const int s8 = S >> 3;
      split = x + 8 * (a2 % s8);
      nblk = a2 / s8;
    } else {  // the host pads the feature blocks to a multiple of eight in this case
      split = a2 % S;
      nblk = (a2 / S) * 8 + x;
    }
  }
  if (nblk >= NBv) return;  // padding block (whole block, before any barrier)
  const int mt0 = zb * MT, mtc = min(MT, Mt_total - mt0), mlast = mtc - 1;
  // K range of the split: a balanced cut of the `nchunks` granules into S parts, counted in chunks
  const int cb0 = (split * nchunks / S) * GRAN, per = ((split + 1) * nchunks / S) * GRAN - cb0;

  if (w >= NCW) {
    loader_wave<MT>(lds, Ap, w - NCW, lane, mt0, mlast, KB, cb0, per);
    return;
  }

  // ---- compute waves ----
  const int nt = nblk * NCW + w;
  if constexpr (NCW != 4) {   // (the strips are padded to a multiple of four)
    if (nt >= NT) {  // no strip left for this wave of the last feature block: it only keeps the block's barrier count
      FSV_BARRIER();
      for (int it = 0; it < per; ++it) FSV_BARRIER();
      return;
    }
  }
  const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void *)Wp, 0, wbytes, 0x00020000);
  const uint32_t wbase = (uint32_t)nt * strip_bytes + (uint32_t)lane * 16u;
  constexpr uint32_t OOB = 0xFFFF0000u;  // a chunk beyond the K range: the descriptor returns zeros, no memory traffic
  bf16x8_t wb[D + 1][KC];   // sixteen bytes of operand per lane; the element type only matters to the MFMA below
  auto issue = [&](int it, bf16x8_t(&dst)[KC]) {
    const uint32_t off = (it < per) ? wbase + (uint32_t)(cb0 + it) * (KC * 1024u) : OOB;
#pragma unroll
    for (int kb = 0; kb < KC; ++kb)
      dst[kb] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(wrs, off + kb * 1024u, 0, 2));
  };
  f32x16_t acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
#pragma unroll
  for (int j = 0; j < D; ++j) issue(j, wb[j]);
  FSV_BARRIER();

  // B operands are read from the ring DL k blocks ahead of the MFMAs that use them (a wave is alone on its SIMD,
  // so nothing else hides the LDS latency); the scheduling barriers keep that order.
  constexpr int DL = 2;
  auto consume = [&](int it, bf16x8_t(&wuse)[KC]) {
    const uint4 *stage = lds + (it % NST) * CHU + lane;
    bf16x8_t aop[DL + 1][MT];
    auto fetch = [&](int kb) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        uint4 raw = stage[(mt * KC + kb) * 64];
        aop[kb % (DL + 1)][mt] = *reinterpret_cast<bf16x8_t *>(&raw);
      }
    };
#pragma unroll
    for (int kb = 0; kb < DL; ++kb) fetch(kb);
#pragma unroll
    for (int kb = 0; kb < KC; ++kb) {
      if (kb + DL < KC) fetch(kb + DL);
      __builtin_amdgcn_sched_barrier(0);
      FSV_IN_AGPR(wuse[kb]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        if constexpr (F16)
          acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, wuse[kb]),
                                                           __builtin_bit_cast(f16x8_t, aop[kb % (DL + 1)][mt]), acc[mt], 0, 0, 0);
        else
          acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wuse[kb], aop[kb % (DL + 1)][mt], acc[mt], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Step s of an unrolled round consumes buffer s and refills the buffer consumed just before it with the chunk D
  // ahead; buffers rotate by name.  Steps past the K range are skipped whole, so that every wave of the block meets
  // exactly 1 + per barriers.
  for (int it = 0; it < per; it += D + 1) {
#pragma unroll
    for (int s = 0; s <= D; ++s) {
      issue(it + s + D, wb[(s + D) % (D + 1)]);
      __builtin_amdgcn_sched_barrier(0);
      if (it + s < per) {
        consume(it + s, wb[s]);
        FSV_BARRIER();
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  store_strip<MT, EPI, F16>(acc, out, nt, mt0, mtc, lane, h, split, M, Mpad, N, KBo, oscale);
}

template <int MT, int EPI>
int launch_t(fsv_ctx *c, int cls, dim3 grid, const void *Wp, uint32_t wbytes, const void *Ap, void *out, int N, int KB, int Mt,
             int M, int Mpad, int splits, int nchunks, int KBo, int NB, int mblocks, int f16, float oscale, int ncw, int NT,
             uint32_t strip_bytes, hipStream_t st) {
  // Weight chunks in flight per wave ahead of the one in use.  Measured on MI355X, one is best: with two to four the
  // bytes in flight across the chip approach the size of the L2s they pass through and the achieved bandwidth drops.
  constexpr int D = 1;
  const size_t ldsb = (size_t)NST * MT * KC * 64 * 16;   // fsv_bf16_gemm_init has raised the kernel's limit to this
  // the profiling events ride on the dispatch itself: they time the kernel, not the gaps around it
  fsv_prof_scope ps(c, st, cls, (double)N * KB * 32.0, true);
#define FSV_GEMM_GO(F16V, NCWV, OSC)                                                                                          \
  hipExtLaunchKernelGGL((k_gemm<MT, EPI, D, F16V, NCWV>), grid, dim3(64 * (NCWV + NLD)), ldsb, st, ps.start(), ps.stop(), 0, Wp, \
                        wbytes, (const uint4 *)Ap, out, N, KB, Mt, M, Mpad, splits, nchunks, KBo, NB, mblocks, OSC, NT, strip_bytes)
  if (f16) {
    if (ncw == 4) FSV_GEMM_GO(true, 4, oscale);
    else if (ncw == 3) FSV_GEMM_GO(true, 3, oscale);
    else FSV_GEMM_GO(true, 2, oscale);
  } else {
    if (ncw == 4) FSV_GEMM_GO(false, 4, 1.0f);
    else if (ncw == 3) FSV_GEMM_GO(false, 3, 1.0f);
    else FSV_GEMM_GO(false, 2, 1.0f);
  }
#undef FSV_GEMM_GO
  return FSV_OK;
}

template <int EPI>
int launch_e(fsv_ctx *c, int cls, const void *Wp, const void *Ap, void *out, int N, int K, int NTpad, int M, int splits,
             int KBo, int f16, float oscale, int ncw, hipStream_t st) {
  if (ncw < 2 || ncw > 4) FSV_FAIL(c, FSV_E_INVALID_ARG, "internal: %d compute waves per block", ncw);
  const int Mt = fsv_ceil_div(M, 32), Mpad = Mt * 32, nchunks = K / 256, KB = K / 16;
  // row tiles per block: the fewest row blocks of at most four tiles (more do not fit the 256 registers a wave of a
  // six-wave block may use), the tiles spread evenly over them (five tiles are taken as 3 + 2, not 4 + 1: a block
  // works on its full tile count whatever the number of real rows)
  const int mblocks = fsv_ceil_div(Mt, 4), mt_blk = fsv_ceil_div(Mt, mblocks);
  const uint32_t strip_bytes = (uint32_t)KB * 1024u + (uint32_t)c->strip_pad_bytes;
  const size_t wbytes = (size_t)NTpad * strip_bytes;
  if (wbytes > 0xFFFF0000ull) FSV_FAIL(c, FSV_E_UNSUPPORTED, "a weight matrix must stay below 4 GiB");
  if (splits < 1 || splits > nchunks) FSV_FAIL(c, FSV_E_INVALID_ARG, "bad split count %d for %d granules", splits, nchunks);
  // one-dimensional grid, decoded in the kernel; feature blocks padded to a multiple of eight when the splits are not
  const int NB = fsv_ceil_div(NTpad, ncw), NBg = (splits % 8 == 0) ? NB : (NB + 7) / 8 * 8;
  dim3 grid((unsigned)NBg * splits * mblocks, 1, 1);
#define FSV_ARGS c, cls, grid, Wp, (uint32_t)wbytes, Ap, out, N, KB, Mt, M, Mpad, splits, nchunks, KBo, NB, mblocks, f16, oscale, ncw, NTpad, strip_bytes, st
  switch (mt_blk) {
    case 1: return launch_t<1, EPI>(FSV_ARGS);
    case 2: return launch_t<2, EPI>(FSV_ARGS);
    case 3: return launch_t<3, EPI>(FSV_ARGS);
    default: return launch_t<4, EPI>(FSV_ARGS);
  }
#undef FSV_ARGS
}

template <int MT, int EPI>
int init_t(fsv_ctx *c) {
#define FSV_GEMM_ATTR(F16V, NCWV)                                                                          \
  FSV_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm<MT, EPI, 1, F16V, NCWV>),          \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, NST * MT * KC * 64 * 16))
  FSV_GEMM_ATTR(false, 4); FSV_GEMM_ATTR(false, 3); FSV_GEMM_ATTR(false, 2);
  FSV_GEMM_ATTR(true, 4); FSV_GEMM_ATTR(true, 3); FSV_GEMM_ATTR(true, 2);
#undef FSV_GEMM_ATTR
  return FSV_OK;
}

template <int EPI>
int init_e(fsv_ctx *c) {
  int rc;
  if ((rc = init_t<1, EPI>(c)) || (rc = init_t<2, EPI>(c)) || (rc = init_t<3, EPI>(c)) || (rc = init_t<4, EPI>(c))) return rc;
  return FSV_OK;
}

}  // namespace

// Raise the dynamic LDS limit of every instantiation (up to 96 KiB) on the current device; called once per context
// from its creation, with error checking, so that no launch depends on a lazily set process-wide flag.
int fsv_bf16_gemm_init(fsv_ctx *c) {
  int rc;
  if ((rc = init_e<EPI_PARTIAL>(c)) || (rc = init_e<EPI_SWIGLU>(c)) || (rc = init_e<EPI_F32>(c))) return rc;
  return FSV_OK;
}

// f16: both operands are fp16 and the sums are multiplied by oscale (see the head of this file); else bf16 operands.
// ncw: compute waves (weight strips) per block, 2..4.
int fsv_bf16_gemm(fsv_ctx *c, int cls, int epi, const void *Wp, const void *Ap, void *out, int N, int K, int NTpad, int M,
                  int splits, int KBo, int f16, float oscale, int ncw, hipStream_t st) {
  int rc;
  switch (epi) {
    case EPI_PARTIAL: rc = launch_e<EPI_PARTIAL>(c, cls, Wp, Ap, out, N, K, NTpad, M, splits, KBo, f16, oscale, ncw, st); break;
    case EPI_SWIGLU: rc = launch_e<EPI_SWIGLU>(c, cls, Wp, Ap, out, N, K, NTpad, M, splits, KBo, f16, oscale, ncw, st); break;
    default: rc = launch_e<EPI_F32>(c, cls, Wp, Ap, out, N, K, NTpad, M, splits, KBo, f16, oscale, ncw, st); break;
  }
  if (rc) return rc;
  FSV_HIP(c, hipGetLastError());
  return FSV_OK;
}
