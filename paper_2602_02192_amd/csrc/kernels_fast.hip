// MFMA path, everything that is not a dense contraction: residual + RMSNorm (with the split-K
// reduction folded in), QKV post-processing (reduction, per-head norm, rotary embedding, KV append).
#include "echo_device.h"
#include "echo_kernels.h"

namespace echo {

// grid M rows, block <= 1024 (a multiple of 64 covering d/4 or d/8 lanes).  h[m] = embed[token[m]]            (embed != null)
//                           h[m] += sum_s partials[s][..][m]  (nsplit <= REDUCE_MAX_SPLIT, summed in split order)
// then Xp[m] = half(h[m] * rsqrt(mean(h[m]^2) + eps) * gain).  d % 8 == 0, d <= 8192.
// Every load of a thread (residual, all partials) is issued before the first use, so the kernel costs
// one memory round trip whatever the split count.
constexpr int RN_THREADS = 1024;
__global__ __launch_bounds__(RN_THREADS) void resid_norm_kernel(float *h, const uint16_t *embed, const int32_t *token,
                                                                const f32x4 *partials, int nsplit, int Np, uint16_t *Xp,
                                                                const uint16_t *gain, int Mp, int d, float eps) {
  __shared__ float sh[RN_THREADS / 64];
  int m = blockIdx.x, d4 = d >> 2;
  f32x4 v[2];
  float ss = 0.f;
  int tok = embed ? token[m] : 0;
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    int n4 = threadIdx.x + c * (int)blockDim.x;
    if (n4 >= d4) break;
    f32x4 a, pp[REDUCE_MAX_SPLIT];
#pragma unroll
    for (int s = 0; s < REDUCE_MAX_SPLIT; ++s)
      pp[s] = s < nsplit ? partials[((int64_t)s * Mp + m) * (Np >> 2) + n4] : f32x4{0.f, 0.f, 0.f, 0.f};
    if (embed) {
      if (tok >= 0) {
        uint2 e = *(const uint2 *)(embed + (int64_t)tok * d + n4 * 4);
        a = {__uint_as_float(e.x << 16), __uint_as_float(e.x & 0xffff0000u), __uint_as_float(e.y << 16),
             __uint_as_float(e.y & 0xffff0000u)};
      } else a = {0.f, 0.f, 0.f, 0.f};
    } else a = *(const f32x4 *)(h + (int64_t)m * d + n4 * 4);
#pragma unroll
    for (int s = 0; s < REDUCE_MAX_SPLIT; ++s) a += pp[s];
    *(f32x4 *)(h + (int64_t)m * d + n4 * 4) = a;
    v[c] = a;
    ss += a[0] * a[0] + a[1] * a[1] + a[2] * a[2] + a[3] * a[3];
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = 0.f;
  for (int i = 0; i < (int)blockDim.x / 64; ++i) ss += sh[i];
  float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    int n4 = threadIdx.x + c * (int)blockDim.x;
    if (n4 >= d4) break;
    int n = n4 * 4;
    uint2 g = *(const uint2 *)(gain + n);
    float g0 = __uint_as_float(g.x << 16), g1 = __uint_as_float(g.x & 0xffff0000u);
    float g2 = __uint_as_float(g.y << 16), g3 = __uint_as_float(g.y & 0xffff0000u);
    uint2 o;
    o.x = (uint32_t)f32_to_h16_bits(v[c][0] * inv * g0) | ((uint32_t)f32_to_h16_bits(v[c][1] * inv * g1) << 16);
    o.y = (uint32_t)f32_to_h16_bits(v[c][2] * inv * g2) | ((uint32_t)f32_to_h16_bits(v[c][3] * inv * g3) << 16);
    *(uint2 *)(Xp + ((int64_t)(n >> 3) * Mp + m) * 8 + (n & 7)) = o;
  }
}

void fast_resid_norm(float *h, const void *embed_bf16, const int32_t *token, const float *partials, int nsplit, int Np,
                     void *Xp, const void *gain_bf16, int M, int Mp, int d, float eps, hipStream_t st) {
  if (M <= 0) return;
  int threads = ((d >> 2) + 63) / 64 * 64;   // one float4 per thread when the row fits, else two
  if (threads > RN_THREADS) threads = ((d >> 3) + 63) / 64 * 64;
  hipLaunchKernelGGL(resid_norm_kernel, dim3(M), dim3(threads), 0, st, h, (const uint16_t *)embed_bf16, token,
                     (const f32x4 *)partials, nsplit, Np, (uint16_t *)Xp, (const uint16_t *)gain_bf16, Mp, d, eps);
}

// grid (M, ceil((Hq + 2*Hkv) / QP_HEADS)), block QP_HEADS * hd/2 with hd/2 <= 64: each group of hd/2 lanes sums the
// split-K partials of one head of one row, applies the optional per-head RMSNorm and the rotary embedding, and writes
// q (half [M][Hq][hd]) or appends k / v to the half-precision cache.
constexpr int QP_HEADS = 8;
__global__ void qkv_post_kernel(const float *partials, int nsplit, int Np, int Mp, uint16_t *q_out, const uint16_t *q_gain,
                                const uint16_t *k_gain, int qk_norm, float eps, const float2 *rope_cs, RowState rows,
                                KvGeom kv, int layer, int Hq, int Hkv) {
  int hd = kv.head_dim, half = hd / 2;
  int m = blockIdx.x, j = blockIdx.y * QP_HEADS + threadIdx.x / half, i = threadIdx.x % half;
  if (j >= Hq + 2 * Hkv) return;
  bool is_q = j < Hq, is_k = !is_q && j < Hq + Hkv;
  if (!is_q && !rows.active[m]) return;
  int n0 = j * hd + i, n1 = n0 + half;
  float a = 0.f, b = 0.f, pa[REDUCE_MAX_SPLIT], pb[REDUCE_MAX_SPLIT];
#pragma unroll
  for (int s = 0; s < REDUCE_MAX_SPLIT; ++s) {   // all loads issued before the sums
    pa[s] = s < nsplit ? partials[((int64_t)s * Mp + m) * Np + n0] : 0.f;
    pb[s] = s < nsplit ? partials[((int64_t)s * Mp + m) * Np + n1] : 0.f;
  }
#pragma unroll
  for (int s = 0; s < REDUCE_MAX_SPLIT; ++s) { a += pa[s]; b += pb[s]; }
  if (is_q || is_k) {
    if (qk_norm) {
      float ss = a * a + b * b;   // the head's lanes are an aligned power-of-two group within the wave
      for (int off = half >> 1; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
      float inv = 1.0f / sqrtf(ss / (float)hd + eps);
      const uint16_t *g = is_q ? q_gain : k_gain;
      a = a * inv * bf16_bits_to_f32(g[i]);
      b = b * inv * bf16_bits_to_f32(g[i + half]);
    }
    float2 cs = rope_cs[(int64_t)m * half + i];
    float ra = a * cs.x - b * cs.y, rb = a * cs.y + b * cs.x;
    a = ra; b = rb;
  }
  if (is_q) {
    uint16_t *dst = q_out + ((int64_t)m * Hq + j) * hd;
    dst[i] = f32_to_h16_bits(a);
    dst[i + half] = f32_to_h16_bits(b);
  } else {   // append to the tiled cache
    int kvh = is_k ? j - Hq : j - Hq - Hkv, pos = rows.pos[m];
    uint16_t *head = (uint16_t *)kv.base + kv.tiled_head_off(rows.slot[m], layer, kvh);
    if (is_k) { head[kv.tiled_k_off(pos, i)] = f32_to_h16_bits(a); head[kv.tiled_k_off(pos, i + half)] = f32_to_h16_bits(b); }
    else { head[kv.tiled_v_off(pos, i)] = f32_to_h16_bits(a); head[kv.tiled_v_off(pos, i + half)] = f32_to_h16_bits(b); }
  }
}

void fast_qkv_post(const float *partials, int nsplit, int Np, int Mp, void *q_h16, const void *q_gain, const void *k_gain,
                   int qk_norm, float eps, const float *rope_cs, RowState rows, KvGeom kv, int layer, int M, int Hq, int Hkv,
                   hipStream_t st) {
  hipLaunchKernelGGL(qkv_post_kernel, dim3(M, (Hq + 2 * Hkv + QP_HEADS - 1) / QP_HEADS), dim3(QP_HEADS * kv.head_dim / 2), 0, st, partials, nsplit, Np, Mp,
                     (uint16_t *)q_h16, (const uint16_t *)q_gain, (const uint16_t *)k_gain, qk_norm, eps,
                     (const float2 *)rope_cs, rows, kv, layer, Hq, Hkv);
}

}  // namespace echo
