// bf16 path: grouped-query decode attention over the contiguous per-sequence KV cache.
//
// attn_simple_kernel: one wavefront per (row, query head), two passes, no split -- the plain form, kept as
//   the on-GPU cross-check of the split-K kernel.
// attn_splitk_kernel: one workgroup per (row, KV head, chunk of keys); the group's query heads share every
//   K/V tile; tiles are staged in LDS from fully coalesced 16-byte loads; QK^T and PV run on MFMA with an
//   online softmax per wavefront; partial (max, sum, acc) per chunk are merged by attn_combine_kernel in
//   chunk order (deterministic, no atomics).
#include "echo_device.h"
#include "echo_kernels.h"

namespace echo {

__device__ __forceinline__ const uint16_t *kv_head_ptr(const KvGeom &kv, int slot, int layer, int kvh) {
  return (const uint16_t *)kv.base + (int64_t)slot * kv.slot_stride() + (int64_t)layer * kv.layer_stride() +
         (int64_t)kvh * kv.head_stride();
}

// Xp (bf16 K8 [Mp][Hq*hd]) element (m, n)
__device__ __forceinline__ int64_t k8_index(int m, int n, int Mp) { return ((int64_t)(n >> 3) * Mp + m) * 8 + (n & 7); }

// grid (M, Hq), block 64, dynamic LDS max_ctx floats; hd <= 256, hd % 64 == 0.
__global__ void attn_simple_kernel(uint16_t *Xp, const uint16_t *q_bf16, RowState rows, KvGeom kv, int layer, int Mp, int Hq,
                                   int Hkv) {
  extern __shared__ float sc[];
  int m = blockIdx.x, j = blockIdx.y, lane = threadIdx.x, hd = kv.head_dim;
  if (!rows.active[m]) {
    for (int i = lane; i < hd; i += 64) Xp[k8_index(m, j * hd + i, Mp)] = 0;
    return;
  }
  int n_keys = rows.pos[m] + 1, kvh = j / (Hq / Hkv);
  const uint16_t *K = kv_head_ptr(kv, rows.slot[m], layer, kvh), *V = K + kv.kv_stride();
  const uint16_t *q = q_bf16 + ((int64_t)m * Hq + j) * hd;
  float scale = 1.0f / sqrtf((float)hd), mx = -INFINITY;
  for (int t = lane; t < n_keys; t += 64) {
    float s = 0.f;
    for (int i = 0; i < hd; ++i) s += bf16_bits_to_f32(q[i]) * bf16_bits_to_f32(K[(int64_t)t * hd + i]);
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
    for (int t = 0; t < n_keys; ++t) acc += sc[t] * bf16_bits_to_f32(V[(int64_t)t * hd + i]);
    Xp[k8_index(m, j * hd + i, Mp)] = f32_to_bf16_bits(acc / den);
  }
}

void fast_attention_simple(void *Xp_out, const void *q_bf16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq,
                           int Hkv, hipStream_t st) {
  hipLaunchKernelGGL(attn_simple_kernel, dim3(M, Hq), dim3(64), (size_t)kv.max_ctx * sizeof(float), st, (uint16_t *)Xp_out,
                     (const uint16_t *)q_bf16, rows, kv, layer, Mp, Hq, Hkv);
}

void fast_attention(void *Xp_out, const void *q_bf16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq, int Hkv,
                    int chunk_keys, int max_splits, float *part_o, float *part_ml, hipStream_t st) {
  fast_attention_simple(Xp_out, q_bf16, rows, kv, layer, M, Mp, Hq, Hkv, st);
}

}  // namespace echo
