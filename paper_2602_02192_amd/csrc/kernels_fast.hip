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

// The same for batches of hundreds of rows and more (prefill, scoring, wide decode steps), where the kernel above is a
// launch of millions of threads that move 14 bytes each: here a thread takes four consecutive dims of the head's first half
// and their four rotation partners, with 16-byte loads of the partials and of the rotation table and 8-byte stores of q and
// of the key tile (a value tile holds eight keys of one dim per unit, so values still leave as single halves).  Same sums in
// the same order: bit-identical to the kernel above.  grid (M, ceil((Hq + 2*Hkv) / QPW_HEADS)), block QPW_HEADS * hd/8.
constexpr int QPW_HEADS = 16;
__global__ void qkv_post_wide_kernel(const float *partials, int nsplit, int Np, int Mp, uint16_t *q_out, const uint16_t *q_gain,
                                     const uint16_t *k_gain, int qk_norm, float eps, const float2 *rope_cs, RowState rows,
                                     KvGeom kv, int layer, int Hq, int Hkv) {
  const int hd = kv.head_dim, half = hd / 2, per_head = half / 4;
  const int m = blockIdx.x, j = blockIdx.y * QPW_HEADS + threadIdx.x / per_head, i = (threadIdx.x % per_head) * 4;
  if (j >= Hq + 2 * Hkv) return;
  const bool is_q = j < Hq, is_k = !is_q && j < Hq + Hkv;
  if (!is_q && !rows.active[m]) return;
  const int n0 = j * hd + i, n1 = n0 + half;
  f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f}, pa[REDUCE_MAX_SPLIT], pb[REDUCE_MAX_SPLIT];
#pragma unroll
  for (int s = 0; s < REDUCE_MAX_SPLIT; ++s) {   // all loads issued before the sums
    const float *row = partials + ((int64_t)s * Mp + m) * Np;
    pa[s] = s < nsplit ? *(const f32x4 *)(row + n0) : f32x4{0.f, 0.f, 0.f, 0.f};
    pb[s] = s < nsplit ? *(const f32x4 *)(row + n1) : f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int s = 0; s < REDUCE_MAX_SPLIT; ++s) { a += pa[s]; b += pb[s]; }
  if (is_q || is_k) {
    if (qk_norm) {
      // Summed in the order of the one-pair-per-lane kernel, whose tree adds lane i ^ off to lane i for off = half/2 .. 1:
      // its lanes 4q .. 4q+3 sit in this thread, so its offsets >= 4 are shuffles over the head's threads, element by
      // element, and its offsets 2 and 1 are the local sums at the end.
      float t[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) t[e] = a[e] * a[e] + b[e] * b[e];
      for (int off = per_head >> 1; off > 0; off >>= 1) {
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] += __shfl_xor(t[e], off);
      }
      const float ss = (t[0] + t[2]) + (t[1] + t[3]);
      float inv = 1.0f / sqrtf(ss / (float)hd + eps);
      const uint16_t *g = is_q ? q_gain : k_gain;
#pragma unroll
      for (int e = 0; e < 4; ++e) { a[e] = a[e] * inv * bf16_bits_to_f32(g[i + e]); b[e] = b[e] * inv * bf16_bits_to_f32(g[i + e + half]); }
    }
    const f32x4 *cs = (const f32x4 *)(rope_cs + (int64_t)m * half + i);
    const f32x4 c01 = cs[0], c23 = cs[1];
    const float cx[4] = {c01[0], c01[2], c23[0], c23[2]}, sy[4] = {c01[1], c01[3], c23[1], c23[3]};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float ra = a[e] * cx[e] - b[e] * sy[e], rb = a[e] * sy[e] + b[e] * cx[e];
      a[e] = ra; b[e] = rb;
    }
  }
  uint2 ha, hb;
  ha.x = (uint32_t)f32_to_h16_bits(a[0]) | ((uint32_t)f32_to_h16_bits(a[1]) << 16);
  ha.y = (uint32_t)f32_to_h16_bits(a[2]) | ((uint32_t)f32_to_h16_bits(a[3]) << 16);
  hb.x = (uint32_t)f32_to_h16_bits(b[0]) | ((uint32_t)f32_to_h16_bits(b[1]) << 16);
  hb.y = (uint32_t)f32_to_h16_bits(b[2]) | ((uint32_t)f32_to_h16_bits(b[3]) << 16);
  if (is_q) {
    uint16_t *dst = q_out + ((int64_t)m * Hq + j) * hd;
    *(uint2 *)(dst + i) = ha;
    *(uint2 *)(dst + i + half) = hb;
  } else {
    const int kvh = is_k ? j - Hq : j - Hq - Hkv, pos = rows.pos[m];
    uint16_t *head = (uint16_t *)kv.base + kv.tiled_head_off(rows.slot[m], layer, kvh);
    if (is_k) {   // four dims of one 8-dim unit of the key
      *(uint2 *)(head + kv.tiled_k_off(pos, i)) = ha;
      *(uint2 *)(head + kv.tiled_k_off(pos, i + half)) = hb;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        head[kv.tiled_v_off(pos, i + e)] = f32_to_h16_bits(a[e]);
        head[kv.tiled_v_off(pos, i + e + half)] = f32_to_h16_bits(b[e]);
      }
    }
  }
}

void fast_qkv_post(const float *partials, int nsplit, int Np, int Mp, void *q_h16, const void *q_gain, const void *k_gain,
                   int qk_norm, float eps, const float *rope_cs, RowState rows, KvGeom kv, int layer, int M, int Hq, int Hkv,
                   hipStream_t st) {
  if (M >= 256) {
    hipLaunchKernelGGL(qkv_post_wide_kernel, dim3(M, (Hq + 2 * Hkv + QPW_HEADS - 1) / QPW_HEADS), dim3(QPW_HEADS * kv.head_dim / 8), 0, st, partials,
                       nsplit, Np, Mp, (uint16_t *)q_h16, (const uint16_t *)q_gain, (const uint16_t *)k_gain, qk_norm, eps,
                       (const float2 *)rope_cs, rows, kv, layer, Hq, Hkv);
    return;
  }
  hipLaunchKernelGGL(qkv_post_kernel, dim3(M, (Hq + 2 * Hkv + QP_HEADS - 1) / QP_HEADS), dim3(QP_HEADS * kv.head_dim / 2), 0, st, partials, nsplit, Np, Mp,
                     (uint16_t *)q_h16, (const uint16_t *)q_gain, (const uint16_t *)k_gain, qk_norm, eps,
                     (const float2 *)rope_cs, rows, kv, layer, Hq, Hkv);
}

// ---- nucleus (top-p) sampling over materialised logits ---------------------------------------------------------
// With p = softmax(logits / T): keep the shortest prefix of the tokens in descending order of p (lower index first
// among equals) whose probabilities reach top_p, draw by Gumbel-max over the kept set with the usual per-index noise,
// return the log-prob renormalised over the kept set (Sec. 5.1 runs rollouts at top-p 0.95).  Three launches:
// 1. topp_cut_kernel, one workgroup per row, finds the cut without sorting: a radix select over the order-preserving
//    integer image of the logit, most significant byte first; each round histograms the probability mass of the
//    candidates by their next byte and walks the 256 bins from the top until the running mass reaches the target.
//    Mass is summed in integers, q_i = floor(exp(z_i - max) * 2^40), so the sums do not depend on the order of the
//    additions and the kept set is the same on every run.  Equal keys have equal mass; of the keys equal
//    to the cut the lowest indices are kept until the target is met, so the kernel also returns the last kept index
//    among them.  Seven passes over the row, which stays in L2.
// 2. topp_draw_kernel, TOPP_CHUNKS workgroups per row: the sampler's running (max, sum-exp, best perturbed score) over
//    the kept tokens of one slice of the vocabulary, in the partial layout of the fused sampler;
// 3. sample_combine_kernel merges the slices.
constexpr int TOPP_THREADS = 1024, TOPP_CHUNKS = TOPP_CHUNKS_PER_ROW;
__device__ __forceinline__ uint32_t float_order_key(float f) {   // a < b  <=>  key(a) < key(b)
  uint32_t u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}
__device__ __forceinline__ float order_key_float(uint32_t key) {   // the float whose key this is
  return __uint_as_float((key & 0x80000000u) ? key ^ 0x80000000u : ~key);
}
constexpr int TOPP_CAND = 1024;   // keys the last round can take from the list (more: it walks the row like the others)
__global__ __launch_bounds__(TOPP_THREADS) void topp_cut_kernel(uint32_t *cut_key, int32_t *cut_last, const float *logits, int64_t ld,
                                                                 int V, float temperature, float top_p, const int32_t *row_active) {
  __shared__ unsigned long long hist[4];        // mass of the bins of each of the first four wavefronts
  __shared__ unsigned long long sub[16][256];   // lanes that meet in one bin are spread over 16 copies of it
  __shared__ unsigned long long sh_u64[TOPP_THREADS / 64];
  __shared__ float sh_f[TOPP_THREADS / 64];
  __shared__ int sh_i[TOPP_THREADS / 64];
  __shared__ unsigned long long sel_above, sel_mass;
  __shared__ uint32_t sel_digit;
  const int m = blockIdx.x, tid = threadIdx.x, wv = tid >> 6;
  if (row_active && !row_active[m]) return;
  const float *lg = logits + (int64_t)m * ld;
  // Every pass visits the row with a stride of the block, two 16-byte loads in flight per thread (a plain loop waits out
  // one memory latency per element); an index past the end yields -inf: mass 0, no maximum, never above a cut.
  const int n4 = (ld & 3) == 0 ? V >> 2 : 0;   // 16-byte loads need aligned rows
  auto visit = [&](auto &&f) {
    const f32x4 *lg4 = (const f32x4 *)lg;
    constexpr int B = 2;   // more copies of the body than this and the kernel outgrows the instruction cache
    for (int i = tid; i < n4; i += B * TOPP_THREADS) {
      f32x4 v[B];
#pragma unroll
      for (int u = 0; u < B; ++u) { int j = i + u * TOPP_THREADS; v[u] = j < n4 ? lg4[j] : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY}; }
#pragma unroll
      for (int u = 0; u < B; ++u) { f(v[u][0]); f(v[u][1]); f(v[u][2]); f(v[u][3]); }
    }
    for (int i = n4 * 4 + tid; i < V; i += TOPP_THREADS) f(lg[i]);
  };
  // max of z and sum of exp(z - max), one pass (running maximum, the sum rescaled whenever it moves); 1/T instead of the
  // division: nothing here is returned, the kept set only needs the same arithmetic in every pass
  const float inv_t = 1.0f / temperature;
  float mx = -INFINITY, zs = 0.f;
  visit([&](float v) {
    float z = v * inv_t;
    if (z > mx) { zs = zs * __expf(mx - z) + 1.f; mx = z; }
    else zs += __expf(z - mx);
  });
  for (int o = 32; o > 0; o >>= 1) {
    float om = __shfl_xor(mx, o, 64), os = __shfl_xor(zs, o, 64), nm = fmaxf(mx, om);
    zs = (mx > -INFINITY ? zs * __expf(mx - nm) : 0.f) + (om > -INFINITY ? os * __expf(om - nm) : 0.f);
    mx = nm;
  }
  if ((tid & 63) == 0) { sh_f[wv] = mx; sh_u64[wv] = (unsigned long long)__float_as_uint(zs); }
  __syncthreads();
  mx = sh_f[0];
  for (int w = 1; w < TOPP_THREADS / 64; ++w) mx = fmaxf(mx, sh_f[w]);
  zs = 0.f;
  for (int w = 0; w < TOPP_THREADS / 64; ++w) zs += __uint_as_float((uint32_t)sh_u64[w]) * __expf(sh_f[w] - mx);
  // probability mass in units of 2^-40 of the largest one, as an integer: sums of it do not depend on the order of the
  // additions.  (Two 32-bit conversions; a float -> 64-bit integer conversion is a long instruction sequence.)
  auto mass = [&](float logit) {
    float e = __expf(logit * inv_t - mx) * 256.0f;          // <= 256
    uint32_t hi = (uint32_t)e;
    uint32_t lo = (uint32_t)((e - (float)hi) * 4294967296.0f);
    return ((unsigned long long)hi << 32) | lo;
  };
  unsigned long long target = (unsigned long long)ceil((double)zs * 1099511627776.0 * (double)top_p);
  if (target < 1) target = 1;
  // radix select of the cut key: the largest key K with mass{key >= K} >= target
  uint32_t prefix = 0;
  unsigned long long above = 0;   // mass of the keys above the current prefix range
  // The third round notes the keys it histograms (those that share the cut's upper 16 bits: a few hundred of a row of
  // N(0, 1)-like logits); if they fit the list the last round walks the list instead of the row.
  __shared__ uint32_t cand[TOPP_CAND];
  __shared__ int cand_n;
  if (tid == 0) cand_n = 0;
  for (int round = 0; round < 4; ++round) {
    const int shift = 24 - 8 * round;
    __syncthreads();
    for (int j = tid; j < 16 * 256; j += TOPP_THREADS) (&sub[0][0])[j] = 0;
    __syncthreads();
    if (round == 3 && cand_n <= TOPP_CAND) {
      for (int j = tid; j < cand_n; j += TOPP_THREADS) {
        const uint32_t key = cand[j];
        if ((key >> 8) == prefix) {
          unsigned long long q = mass(order_key_float(key));
          if (q) atomicAdd(&sub[tid & 15][key & 255u], q);
        }
      }
    } else {
      visit([&](float v) {
        uint32_t key = float_order_key(v);
        if (round == 0 || (key >> (shift + 8)) == prefix) {
          unsigned long long q = mass(v);
          if (q) atomicAdd(&sub[tid & 15][(key >> shift) & 255u], q);
          if (round == 2) {
            const int k = atomicAdd(&cand_n, 1);
            if (k < TOPP_CAND) cand[k] = key;
          }
        }
      });
    }
    __syncthreads();
    // walk the bins from the top: thread t of the first four wavefronts owns bin 255 - t, so an inclusive prefix sum
    // over t is the mass of the bins at or above its own; exactly one bin takes the running mass across the target
    unsigned long long h = 0, incl = 0;
    if (tid < 256) {
      for (int j = 0; j < 16; ++j) h += sub[j][255 - tid];
      incl = h;
      for (int o = 1; o < 64; o <<= 1) { unsigned long long v = __shfl_up(incl, o, 64); if ((tid & 63) >= o) incl += v; }
      if ((tid & 63) == 63) hist[wv] = incl;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = 0; w < wv; ++w) incl += hist[w];
      const unsigned long long at = above + incl, before = at - h;
      if ((at >= target && before < target) || (tid == 255 && at < target)) { sel_digit = (uint32_t)(255 - tid); sel_above = before; sel_mass = h; }
    }
    __syncthreads();
    prefix = (prefix << 8) | sel_digit;
    above = sel_above;
  }
  const uint32_t cut = prefix;
  // Keys equal to the cut share one mass, so the last round's bin of the cut -- whose keys are exactly those -- holds
  // their number times that mass; the first `take` of them in index order are kept.  (A mass of zero, far below the
  // maximum: every such key is kept, and their number does not matter.)
  const unsigned long long qc = mass(order_key_float(cut));
  const long long n_ties = qc ? (long long)(sel_mass / qc) : 0;
  const unsigned long long need = target - above;   // > 0: mass still missing once every key above the cut is kept
  const long long take = qc ? (long long)((need + qc - 1) / qc) : (long long)V;   // >= 1
  if (tid == 0) { cut_key[m] = cut; cut_last[m] = V; }   // V: every key equal to the cut is kept
  if (take >= n_ties) return;
  // Only some of the equal keys are kept (exact ties at the cut: rare): their indices are collected and the take-th
  // smallest one closes the kept set.  More ties than the list holds (flat logits): ranks by a scan over contiguous runs.
  __shared__ int tie_list[TOPP_THREADS];
  __shared__ int tie_n;
  if (tid == 0) tie_n = 0;
  __syncthreads();
  if (n_ties <= TOPP_THREADS) {
    for (int i = tid; i < V; i += TOPP_THREADS)
      if (float_order_key(lg[i]) == cut) tie_list[atomicAdd(&tie_n, 1)] = i;
    __syncthreads();
    if (tid < n_ties) {
      const int mine = tie_list[tid];
      int smaller = 0;
      for (int u = 0; u < n_ties; ++u) smaller += tie_list[u] < mine;
      if (smaller == take - 1) cut_last[m] = mine;
    }
    return;
  }
  const int chunk = (V + TOPP_THREADS - 1) / TOPP_THREADS, i0 = tid * chunk, i1 = min(V, i0 + chunk);
  int mine = 0;
  for (int i = i0; i < i1; ++i) mine += float_order_key(lg[i]) == cut;
  int incl = mine;
  for (int o = 1; o < 64; o <<= 1) { int v = __shfl_up(incl, o, 64); if ((tid & 63) >= o) incl += v; }
  __syncthreads();
  if ((tid & 63) == 63) sh_i[wv] = incl;
  __syncthreads();
  int rank = incl - mine;   // ties before this thread's run
  for (int w = 0; w < wv; ++w) rank += sh_i[w];
  if (rank < take && take <= rank + mine) {   // the take-th tie lies in this thread's run
    for (int i = i0; i < i1; ++i)
      if (float_order_key(lg[i]) == cut && ++rank == take) cut_last[m] = i;
  }
}

// grid (TOPP_CHUNKS, M), block 256: slice c of row m.
__global__ void topp_draw_kernel(float *part, int Mp, const uint32_t *cut_key, const int32_t *cut_last, const float *logits, int64_t ld,
                                 int V, float temperature, uint64_t seed, DrawIds ids, const int32_t *row_active) {
  __shared__ SampleAcc sh[4];
  const int c = blockIdx.x, m = blockIdx.y;
  if (row_active && !row_active[m]) return;
  const uint32_t step = draw_step(ids, m), stream = draw_stream(ids, m), cut = cut_key[m];
  const int last = cut_last[m];
  const int v4 = (V + 3) / 4, per = (v4 + TOPP_CHUNKS - 1) / TOPP_CHUNKS, b4 = c * per, e4 = min(v4, b4 + per);
  const float *lg = logits + (int64_t)m * ld;
  SampleAcc a = sample_acc_init();
  for (int i4 = b4 + threadIdx.x; i4 < e4; i4 += blockDim.x) {
    u32x4 r = draw4(seed, stream, step, (uint32_t)i4);
    uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      int i = i4 * 4 + e;
      if (i < V) {
        float v = lg[i];
        uint32_t key = float_order_key(v);
        if (key > cut || (key == cut && i <= last)) {
          float z = v / temperature;
          sample_acc_add(a, z, z + gumbel_from_bits(w[e]), i);
        }
      }
    }
  }
  for (int o = 32; o > 0; o >>= 1) { SampleAcc b = sample_acc_shfl_xor(a, o); sample_acc_merge(a, b); }
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) sample_acc_merge(a, sh[w]);
    int64_t o = (int64_t)c * Mp + m, plane = (int64_t)TOPP_CHUNKS * Mp;
    part[o] = a.zmax;
    part[plane + o] = a.zsum;
    part[2 * plane + o] = a.best;
    part[3 * plane + o] = a.zbest;
    part[4 * plane + o] = __int_as_float(a.idx);
  }
}

size_t fast_topp_scratch_floats(int Mp) { return (size_t)5 * TOPP_CHUNKS * Mp + 2 * (size_t)Mp; }

void fast_topp_cut_and_draw(float *scratch, const float *logits, int64_t ld, int M, int Mp, int V, float temperature, float top_p,
                            uint64_t seed, DrawIds ids, const int32_t *row_active, hipStream_t st) {
  if (M <= 0) return;
  uint32_t *cut_key = (uint32_t *)(scratch + (size_t)5 * TOPP_CHUNKS * Mp);
  int32_t *cut_last = (int32_t *)cut_key + Mp;
  hipLaunchKernelGGL(topp_cut_kernel, dim3(M), dim3(TOPP_THREADS), 0, st, cut_key, cut_last, logits, ld, V, temperature, top_p, row_active);
  hipLaunchKernelGGL(topp_draw_kernel, dim3(TOPP_CHUNKS, M), dim3(256), 0, st, scratch, Mp, cut_key, cut_last, logits, ld, V, temperature,
                     seed, ids, row_active);
}

}  // namespace echo
