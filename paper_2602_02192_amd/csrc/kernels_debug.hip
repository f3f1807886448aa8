// Debug path: plain fp32 kernels over row-major weights (fp32 or bf16 storage), fp32 activations and an
// fp32 KV cache.  One thread (or one small block) per output, sequential sums; no tiling.  This is the
// "fp32 debug mode" the fast kernels are cross-checked against on the GPU, and the path for fp32 models.
#include "echo_device.h"
#include "echo_kernels.h"

namespace echo {

template <bool BF>
__global__ void dbg_embed_kernel(float *h, const void *embed, const int32_t *token, int d) {
  int m = blockIdx.x, t = token[m];
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(int64_t)m * d + i] = t >= 0 ? load_w<BF>(embed, (int64_t)t * d + i) : 0.f;
}

void dbg_embed(float *h, const void *embed, int w_bf16, const int32_t *token, int M, int d, hipStream_t st) {
  if (w_bf16) hipLaunchKernelGGL(dbg_embed_kernel<true>, dim3(M), dim3(256), 0, st, h, embed, token, d);
  else hipLaunchKernelGGL(dbg_embed_kernel<false>, dim3(M), dim3(256), 0, st, h, embed, token, d);
}

__device__ float block_sum_256(float v, float *sh) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) t += sh[i];
  return t;
}

template <bool BF>
__global__ void dbg_rmsnorm_kernel(float *x, const float *h, const void *gain, int d, float eps) {
  __shared__ float sh[8];
  int m = blockIdx.x;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += blockDim.x) { float v = h[(int64_t)m * d + i]; ss += v * v; }
  ss = block_sum_256(ss, sh);
  float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += blockDim.x) x[(int64_t)m * d + i] = h[(int64_t)m * d + i] * inv * load_w<BF>(gain, i);
}

void dbg_rmsnorm(float *x, const float *h, const void *gain, int w_bf16, int M, int d, float eps, hipStream_t st) {
  if (w_bf16) hipLaunchKernelGGL(dbg_rmsnorm_kernel<true>, dim3(M), dim3(256), 0, st, x, h, gain, d, eps);
  else hipLaunchKernelGGL(dbg_rmsnorm_kernel<false>, dim3(M), dim3(256), 0, st, x, h, gain, d, eps);
}

// One wavefront per output element block: lanes stride over k, then a shuffle reduction.
template <bool BF>
__global__ void dbg_gemm_kernel(float *Y, const float *X, const void *W, int M, int N, int K, int accumulate) {
  int n = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  int m = blockIdx.y, lane = threadIdx.x & 63;
  if (n >= N) return;
  float acc = 0.f;
  for (int k = lane; k < K; k += 64) acc += load_w<BF>(W, (int64_t)n * K + k) * X[(int64_t)m * K + k];
  acc = wave_sum(acc);
  if (lane == 0) {
    int64_t o = (int64_t)m * N + n;
    Y[o] = accumulate ? Y[o] + acc : acc;
  }
}

void dbg_gemm(float *Y, const float *X, const void *W, int w_bf16, int M, int N, int K, int accumulate, hipStream_t st) {
  dim3 grid((N + 3) / 4, M), block(256);
  if (w_bf16) hipLaunchKernelGGL(dbg_gemm_kernel<true>, grid, block, 0, st, Y, X, W, M, N, K, accumulate);
  else hipLaunchKernelGGL(dbg_gemm_kernel<false>, grid, block, 0, st, Y, X, W, M, N, K, accumulate);
}

// grid (M, Hq + 2*Hkv), block hd/2 threads (<= 128): optional per-head RMSNorm, rotary embedding on q and k,
// append k and v to the fp32 cache.
template <bool BF>
__global__ void dbg_qkv_post_kernel(float *qkv, const void *q_gain, const void *k_gain, int qk_norm, float eps,
                                    const float2 *rope_cs, RowState rows, KvGeom kv, int layer, int Hq, int Hkv) {
  __shared__ float sh[8];
  int m = blockIdx.x, j = blockIdx.y, hd = kv.head_dim, half = hd / 2, i = threadIdx.x;
  int width = (Hq + 2 * Hkv) * hd;
  float *v = qkv + (int64_t)m * width + (int64_t)j * hd;
  bool is_q = j < Hq, is_k = !is_q && j < Hq + Hkv;
  float a = v[i], b = v[i + half];
  if (is_q || is_k) {
    if (qk_norm) {
      float ss = a * a + b * b;
      ss = wave_sum(ss);
      if (blockDim.x > 64) {  // hd = 256: two wavefronts
        if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
        __syncthreads();
        ss = sh[0] + sh[1];
      }
      float inv = 1.0f / sqrtf(ss / (float)hd + eps);
      const void *g = is_q ? q_gain : k_gain;
      a = a * inv * load_w<BF>(g, i);
      b = b * inv * load_w<BF>(g, i + half);
    }
    float2 cs = rope_cs[(int64_t)m * half + i];
    float ra = a * cs.x - b * cs.y, rb = a * cs.y + b * cs.x;
    a = ra; b = rb;
  }
  if (is_q) { v[i] = a; v[i + half] = b; return; }
  if (!rows.active[m]) return;
  int kvh = is_k ? j - Hq : j - Hq - Hkv;
  float *dst = (float *)kv.base + (int64_t)rows.slot[m] * kv.slot_stride() + (int64_t)layer * kv.layer_stride() +
               (is_k ? 0 : kv.kv_stride()) + (int64_t)kvh * kv.head_stride() + (int64_t)rows.pos[m] * hd;
  dst[i] = a; dst[i + half] = b;
}

void dbg_qkv_post(float *qkv, const void *q_gain, const void *k_gain, int w_bf16, int qk_norm, float eps,
                  const float *rope_cs, RowState rows, KvGeom kv, int layer, int M, int Hq, int Hkv, hipStream_t st) {
  dim3 grid(M, Hq + 2 * Hkv), block(kv.head_dim / 2);
  if (w_bf16) hipLaunchKernelGGL(dbg_qkv_post_kernel<true>, grid, block, 0, st, qkv, q_gain, k_gain, qk_norm, eps,
                                 (const float2 *)rope_cs, rows, kv, layer, Hq, Hkv);
  else hipLaunchKernelGGL(dbg_qkv_post_kernel<false>, grid, block, 0, st, qkv, q_gain, k_gain, qk_norm, eps,
                          (const float2 *)rope_cs, rows, kv, layer, Hq, Hkv);
}

// grid (M, Hq), one wavefront: scores to LDS (dynamic, max_ctx floats), max, exp/sum, weighted sum of V.
__global__ void dbg_attention_kernel(float *out, const float *qkv, RowState rows, KvGeom kv, int layer, int Hq, int Hkv) {
  extern __shared__ float sc[];
  int m = blockIdx.x, j = blockIdx.y, lane = threadIdx.x, hd = kv.head_dim;
  float *o = out + ((int64_t)m * Hq + j) * hd;
  if (!rows.active[m]) { for (int i = lane; i < hd; i += 64) o[i] = 0.f; return; }
  int width = (Hq + 2 * Hkv) * hd, n_keys = rows.pos[m] + 1, kvh = j / (Hq / Hkv);
  const float *q = qkv + (int64_t)m * width + (int64_t)j * hd;
  const float *K = (const float *)kv.base + (int64_t)rows.slot[m] * kv.slot_stride() + (int64_t)layer * kv.layer_stride() +
                   (int64_t)kvh * kv.head_stride();
  const float *V = K + kv.kv_stride();
  float scale = 1.0f / sqrtf((float)hd), mx = -INFINITY;
  for (int t = lane; t < n_keys; t += 64) {
    float s = 0.f;
    for (int i = 0; i < hd; ++i) s += q[i] * K[(int64_t)t * hd + i];
    s *= scale;
    sc[t] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float den = 0.f;
  for (int t = lane; t < n_keys; t += 64) { float e = expf(sc[t] - mx); sc[t] = e; den += e; }
  den = wave_sum(den);
  __syncthreads();
  for (int i = lane; i < hd; i += 64) {
    float acc = 0.f;
    for (int t = 0; t < n_keys; ++t) acc += sc[t] * V[(int64_t)t * hd + i];
    o[i] = acc / den;
  }
}

void dbg_attention(float *out, const float *qkv, RowState rows, KvGeom kv, int layer, int M, int Hq, int Hkv, hipStream_t st) {
  hipLaunchKernelGGL(dbg_attention_kernel, dim3(M, Hq), dim3(64), (size_t)kv.max_ctx * sizeof(float), st, out, qkv, rows,
                     kv, layer, Hq, Hkv);
}

__global__ void dbg_swiglu_kernel(float *ff, const float *gu, int M, int F) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)M * F) return;
  int64_t m = idx / F, f = idx % F;
  float g = gu[m * 2 * F + f], u = gu[m * 2 * F + F + f];
  ff[idx] = g / (1.0f + expf(-g)) * u;
}

void dbg_swiglu(float *ff, const float *gu, int M, int F, hipStream_t st) {
  int64_t n = (int64_t)M * F;
  hipLaunchKernelGGL(dbg_swiglu_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, ff, gu, M, F);
}

// One block of 256 threads per row: Gumbel-max token and log softmax(z)[token] from materialised logits.
__global__ void dbg_sample_kernel(int32_t *tok, float *lp, const float *logits, int64_t ld, int V, float temperature,
                                  uint64_t seed, DrawIds ids, const int32_t *row_active) {
  __shared__ SampleAcc sh[4];
  int m = blockIdx.x;
  if (row_active && !row_active[m]) return;
  const uint32_t s = draw_step(ids, m), stream = draw_stream(ids, m);
  SampleAcc a = sample_acc_init();
  const float *lg = logits + (int64_t)m * ld;
  for (int i4 = threadIdx.x; i4 * 4 < V; i4 += blockDim.x) {
    u32x4 r = draw4(seed, stream, s, (uint32_t)i4);
    uint32_t w[4] = {r.x, r.y, r.z, r.w};
    for (int e = 0; e < 4; ++e) {
      int i = i4 * 4 + e;
      if (i >= V) break;
      float z = lg[i] / temperature;
      sample_acc_add(a, z, z + gumbel_from_bits(w[e]), i);
    }
  }
  for (int o = 32; o > 0; o >>= 1) { SampleAcc b = sample_acc_shfl_xor(a, o); sample_acc_merge(a, b); }
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) sample_acc_merge(a, sh[w]);
    tok[m] = a.idx;
    lp[m] = a.zbest - (a.zmax + logf(a.zsum));
  }
}

void dbg_sample(int32_t *tok, float *lp, const float *logits, int64_t ld, int M, int V, float temperature, uint64_t seed,
                DrawIds ids, const int32_t *row_active, hipStream_t st) {
  hipLaunchKernelGGL(dbg_sample_kernel, dim3(M), dim3(256), 0, st, tok, lp, logits, ld, V, temperature, seed, ids,
                     row_active);
}

__global__ void dbg_target_logprob_kernel(float *lp, const float *logits, int64_t ld, int V, float temperature,
                                          const int32_t *target) {
  __shared__ float sh[8];
  int m = blockIdx.x, t = target[m];
  if (t < 0) { if (threadIdx.x == 0) lp[m] = 0.f; return; }
  const float *lg = logits + (int64_t)m * ld;
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < V; i += blockDim.x) mx = fmaxf(mx, lg[i] / temperature);
  mx = wave_max(mx);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  float den = 0.f;
  for (int i = threadIdx.x; i < V; i += blockDim.x) den += expf(lg[i] / temperature - mx);
  den = block_sum_256(den, sh + 4);
  if (threadIdx.x == 0) lp[m] = lg[t] / temperature - (mx + logf(den));
}

void dbg_target_logprob(float *lp, const float *logits, int64_t ld, int M, int V, float temperature,
                        const int32_t *target, hipStream_t st) {
  hipLaunchKernelGGL(dbg_target_logprob_kernel, dim3(M), dim3(256), 0, st, lp, logits, ld, V, temperature, target);
}

}  // namespace echo
