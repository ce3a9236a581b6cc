// Device helpers shared by the translation units of the FSV_BF16 path: conversions and the operand
// orders of activations, query blocks and KV page tiles (gfx950, 32x32x16 bf16 MFMA).
#pragma once
#include "fsv_internal.h"

namespace fsv_bf16 {

constexpr int KCHUNK = 256;       // contraction elements per split / group granule (a multiple of every chunk size)
constexpr int RTMAX = 3;         // query-row tiles of 32 per (request, kv head): group * (gamma+1) <= 96
constexpr float kLog2eF = 1.4426950408889634f;

__device__ inline float bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline uint16_t f2bf(float f) {  // round to nearest even (hardware conversion)
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
// fp16 (11 significant bits) for the two tensors that are bounded whatever the model: the normalised activations entering
// a projection and the attention output.  Round to nearest even (hardware conversion), held at +-65504 beyond the range
// (a NaN stays a NaN).
__device__ inline uint16_t f2h(float f) {
  const float g = fminf(fmaxf(f, -65504.0f), 65504.0f);
  _Float16 hv = (_Float16)(f != f ? f : g);
  return __builtin_bit_cast(uint16_t, hv);
}
__device__ inline float h2f(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ inline uint32_t f2h2(float lo, float hi) { return (uint32_t)f2h(lo) | ((uint32_t)f2h(hi) << 16); }
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// offset, in 16-byte units, of the operand unit holding (row r, k .. k+7), k a multiple of 8
__device__ __host__ inline size_t tile_unit(int r, int k, int KB) {
  return ((size_t)(r >> 5) * KB + (k >> 4)) * 64 + (r & 31) + 32 * ((k >> 3) & 1);
}

// K tile: element (t, e) at ((e/16*2 + (e%16)/8)*16 + t)*8 + e%8       (operand of the score MFMA, rows = keys)
// V tile: element (t, e) at ((e/32*2 + (t%8)/4)*32 + e%32)*8 + 4*(t/8) + t%4   (operand of the P.V MFMA, rows = features,
//         contraction index ordered the way the score accumulators leave the probabilities in registers)
__device__ __host__ inline int k_tile_off(int t, int e) { return (((e >> 4) * 2 + ((e >> 3) & 1)) * 16 + t) * 8 + (e & 7); }
__device__ __host__ inline int v_tile_off(int t, int e) {
  return (((e >> 5) * 2 + ((t >> 2) & 1)) * 32 + (e & 31)) * 8 + 4 * (t >> 3) + (t & 3);
}

// query operand: row rr = i*group + g of (request, kv head), feature e:
//   (((b*RTMAX + rr/32)*Hkv + kvh)*(hd/16) + e/16)*64 + rr%32 + 32*((e%16)/8) units of 8, element e%8
__device__ inline size_t q_elem_off(int b, int kvh, int rr, int e, int Hkv, int hd) {
  return (((((size_t)b * RTMAX + (rr >> 5)) * Hkv + kvh) * (hd >> 4) + (e >> 4)) * 64 + (rr & 31) + 32 * ((e >> 3) & 1)) * 8 +
         (e & 7);
}

}  // namespace fsv_bf16
