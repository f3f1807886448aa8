// Device-side helpers shared by the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "echo_kernels.h"

namespace echo {

// MFMA operands are IEEE half precision (11-bit significand): activations, the KV cache and the attention
// probabilities are rounded to it, which keeps the logit error of a 36-layer, 151936-entry model an order of
// magnitude below what 8-bit-significand bf16 operands give.  The weights are bf16 values; they are held as
// half-precision values scaled by W_SCALE (a power of two, so exact for every bf16 weight of magnitude
// 2^-22 .. 255), and the fp32 accumulators are scaled back by W_UNSCALE in the epilogues.
typedef __attribute__((ext_vector_type(8))) _Float16 h16x8;
constexpr float W_SCALE = 256.0f, W_UNSCALE = 1.0f / 256.0f;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs; NaN keeps a quiet NaN)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// fp32 -> half bits, round to nearest even, saturating at the largest finite half
__device__ __forceinline__ uint16_t f32_to_h16_bits(float f) {
  _Float16 h = (_Float16)fminf(fmaxf(f, -65504.0f), 65504.0f);
  return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float h16_bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ f32x16 mfma_h16(h16x8 a, h16x8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }

template <bool BF16>
__device__ __forceinline__ float load_w(const void *p, int64_t i) {
  if (BF16) return bf16_bits_to_f32(((const uint16_t *)p)[i]);
  return ((const float *)p)[i];
}

// Philox-4x32 with 10 rounds (Salmon et al., SC'11): multipliers 0xD2511F53 / 0xCD9E8D57, key
// increments 0x9E3779B9 / 0xBB67AE85.
struct u32x4 { uint32_t x, y, z, w; };
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return {c0, c1, c2, c3};
}

// Four draws for vocabulary entries 4*i4 .. 4*i4+3 of sequence n at generation step s.
__device__ __forceinline__ u32x4 draw4(uint64_t seed, uint32_t n, uint32_t s, uint32_t i4) {
  return philox4x32_10(i4, s, n, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// Step and stream words of row m's draws.
__device__ __forceinline__ uint32_t draw_step(const DrawIds &d, int m) { return (uint32_t)(d.row_step ? d.row_step[m] : *d.d_step); }
__device__ __forceinline__ uint32_t draw_stream(const DrawIds &d, int m) { return (uint32_t)(d.row_stream ? d.row_stream[m] : m); }

// 23 random bits -> u = (2k+1) 2^-24, then the standard Gumbel variate -log(-log u) in fp32.
__device__ __forceinline__ float gumbel_from_bits(uint32_t bits) {
  float u = (float)(2u * (bits >> 9) + 1u) * 0x1p-24f;
  return -logf(-logf(u));
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Running Gumbel-max / log-sum-exp state for one row over a subset of the vocabulary.
struct SampleAcc {
  float zmax, zsum;   // max z and sum exp(z - zmax)
  float best, zbest;  // best perturbed score and the z at that entry
  int32_t idx;        // its vocabulary index (lowest index on exact ties)
};
__device__ __forceinline__ SampleAcc sample_acc_init() { return {-INFINITY, 0.f, -INFINITY, 0.f, 0x7fffffff}; }
__device__ __forceinline__ void sample_acc_add(SampleAcc &a, float z, float score, int32_t i) {
  if (z > a.zmax) { a.zsum = a.zsum * expf(a.zmax - z) + 1.f; a.zmax = z; }
  else a.zsum += expf(z - a.zmax);
  if (score > a.best || (score == a.best && i < a.idx)) { a.best = score; a.idx = i; a.zbest = z; }
}
__device__ __forceinline__ void sample_acc_merge(SampleAcc &a, const SampleAcc &b) {
  if (b.zmax > a.zmax) { a.zsum = a.zsum * expf(a.zmax - b.zmax) + b.zsum; a.zmax = b.zmax; }
  else if (b.zmax > -INFINITY) a.zsum += b.zsum * expf(b.zmax - a.zmax);
  if (b.best > a.best || (b.best == a.best && b.idx < a.idx)) { a.best = b.best; a.idx = b.idx; a.zbest = b.zbest; }
}
__device__ __forceinline__ SampleAcc sample_acc_shfl_xor(const SampleAcc &a, int o) {
  SampleAcc b;
  b.zmax = __shfl_xor(a.zmax, o, 64); b.zsum = __shfl_xor(a.zsum, o, 64);
  b.best = __shfl_xor(a.best, o, 64); b.zbest = __shfl_xor(a.zbest, o, 64);
  b.idx = __shfl_xor(a.idx, o, 64);
  return b;
}

}  // namespace echo
