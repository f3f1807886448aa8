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

// ---- split-K MFMA kernel -----------------------------------------------------------------------------
// MFMA roles.  QK^T: A = Q (row = query head of the group, zero beyond the group), B = K^T (column = key);
// lane l receives, in accumulator registers 0..3, the scores of key l%32 for query rows 4*(l/32)+i.
// PV: A = P (bf16, through LDS), B = V with column c of MFMA e standing for head dimension (HD/32)*c + e,
// so that a lane's B operand is built from 8-byte (HD=128) or 4-byte (HD=64) LDS reads of 8 keys.
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));
constexpr int ATT_TILE = 32;     // keys per tile
constexpr int ATT_WAVES = 4;

template <int HD> struct AttLds {
  static constexpr int ROW = HD * 2 + 16;                  // padded K/V row in bytes
  static constexpr int PROW = ATT_TILE * 2 + 16;            // padded P row in bytes
  static constexpr int PER_WAVE = 2 * ATT_TILE * ROW + 8 * PROW;
  static constexpr int MERGE_PER_WAVE = 8 * HD * 4 + 64;    // O rows + (m, l)
  static constexpr int TOTAL = ATT_WAVES * PER_WAVE;
};

template <int HD>
__device__ __forceinline__ void att_issue_loads(v4u (&rk)[HD / 16], v4u (&rv)[HD / 16], const uint16_t *__restrict__ Kg,
                                                const uint16_t *__restrict__ Vg, int tk0, int n_keys, int lane) {
#pragma unroll
  for (int i = 0; i < HD / 16; ++i) {
    int u = i * 64 + lane, key = tk0 + u / (HD / 8);
    key = min(key, n_keys - 1);               // tail keys re-read the last valid row (masked by the caller)
    int64_t off = (int64_t)key * HD + (u % (HD / 8)) * 8;
    rk[i] = *(const v4u *)(Kg + off);
    rv[i] = *(const v4u *)(Vg + off);
  }
}

// Keys per split of a row with n_keys keys cut into nsplit equal parts (whole tiles).
__device__ __forceinline__ int att_split_len(int n_keys, int nsplit) {
  return ((n_keys + nsplit - 1) / nsplit + ATT_TILE - 1) & ~(ATT_TILE - 1);
}

// grid (nsplit, Hkv, M).  Every row's keys are cut into nsplit equal chunks of that row's own length.  DIRECT
// (nsplit == 1): the workgroup normalises and writes the bf16 output itself and no partials exist.
template <int HD, bool DIRECT>
__global__ __launch_bounds__(256, 2) void attn_splitk_kernel(float *__restrict__ part_o, float *__restrict__ part_ml,
                                                             uint16_t *__restrict__ Xp, int Mp,
                                                             const uint16_t *__restrict__ q_bf16, RowState rows, KvGeom kv,
                                                             int layer, int Hq, int Hkv, int nsplit) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  using L = AttLds<HD>;
  constexpr int KS = HD / 16;          // k-steps of QK^T
  constexpr int NE = HD / 32;          // PV MFMAs per 16 keys; also head dims per lane column
  constexpr int LD = HD / 16;          // 16-byte loads per lane per K (or V) tile
  const int c = blockIdx.x, kvh = blockIdx.y, m = blockIdx.z;
  const int grp = Hq / Hkv;
  if (!rows.active[m]) {
    if (DIRECT)
      for (int idx = threadIdx.x; idx < grp * HD; idx += 256) Xp[k8_index(m, kvh * grp * HD + idx, Mp)] = 0;
    return;
  }
  const int n_keys = rows.pos[m] + 1, chunk_keys = att_split_len(n_keys, nsplit), key0 = c * chunk_keys;
  if (key0 >= n_keys) return;
  const int key1 = min(n_keys, key0 + chunk_keys), ntiles = (key1 - key0 + ATT_TILE - 1) / ATT_TILE;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  char *Ks = lds + w * L::PER_WAVE, *Vs = Ks + ATT_TILE * L::ROW, *Ps = Vs + ATT_TILE * L::ROW;
  const uint16_t *Kg = kv_head_ptr(kv, rows.slot[m], layer, kvh), *Vg = Kg + kv.kv_stride();

  // Q as MFMA A operand: row = col (query head within the group), dims ks*16 + half*8 .. +8
  bf16x8 qa[KS];
  {
    const uint16_t *qrow = q_bf16 + ((int64_t)m * Hq + kvh * grp + (col < grp ? col : 0)) * HD;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      v4u v = *(const v4u *)(qrow + ks * 16 + half * 8);
      if (col >= grp) v = v4u{0u, 0u, 0u, 0u};
      qa[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }
  const float scale = 1.0f / sqrtf((float)HD);
  float m_run[4], l_run[4];
  f32x16 o[NE];
#pragma unroll
  for (int i = 0; i < 4; ++i) { m_run[i] = -INFINITY; l_run[i] = 0.f; }
#pragma unroll
  for (int e = 0; e < NE; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[e][r] = 0.f;

  // global -> register staging of one tile: 16-byte unit u = i*64 + lane covers key u/(HD/8), byte (u%(HD/8))*16
  v4u rk[LD], rv[LD];
  int tile = w;
  if (tile < ntiles) att_issue_loads<HD>(rk, rv, Kg, Vg, key0 + tile * ATT_TILE, n_keys, lane);
  for (; tile < ntiles; tile += ATT_WAVES) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // earlier LDS reads of this wavefront are done
#pragma unroll
    for (int i = 0; i < LD; ++i) {
      int u = i * 64 + lane, key = u / (HD / 8), b = (u % (HD / 8)) * 16;
      *(v4u *)(Ks + key * L::ROW + b) = rk[i];
      *(v4u *)(Vs + key * L::ROW + b) = rv[i];
    }
    if (tile + ATT_WAVES < ntiles) att_issue_loads<HD>(rk, rv, Kg, Vg, key0 + (tile + ATT_WAVES) * ATT_TILE, n_keys, lane);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    // ---- S = Q K^T
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      v4u kb = *(const v4u *)(Ks + col * L::ROW + (ks * 16 + half * 8) * 2);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ks], __builtin_bit_cast(bf16x8, kb), sacc, 0, 0, 0);
    }
    // ---- online softmax over this tile's 32 keys (rows 4*half + i, key = col)
    bool kvalid = key0 + tile * ATT_TILE + col < key1;
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float sv = kvalid ? sacc[i] * scale : -INFINITY;
      float tm = sv;
#pragma unroll
      for (int x = 16; x > 0; x >>= 1) tm = fmaxf(tm, __shfl_xor(tm, x, 64));
      float mn = fmaxf(m_run[i], tm);
      float alpha = __expf(m_run[i] - mn);
      p[i] = __expf(sv - mn);
      l_run[i] = l_run[i] * alpha + p[i];
      m_run[i] = mn;
#pragma unroll
      for (int e = 0; e < NE; ++e) o[e][i] *= alpha;
    }
    // ---- P (bf16) through LDS into A-operand layout
    {
      int r0 = half * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) *(uint16_t *)(Ps + (r0 + i) * L::PROW + col * 2) = f32_to_bf16_bits(p[i]);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      v4u pa = v4u{0u, 0u, 0u, 0u};
      if (col < 8) pa = *(const v4u *)(Ps + col * L::PROW + (k2 * 16 + half * 8) * 2);
      bf16x8 pA = __builtin_bit_cast(bf16x8, pa);
      if (HD == 128) {
        v2u vr[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) vr[j] = *(const v2u *)(Vs + (k2 * 16 + half * 8 + j) * L::ROW + col * 8);
#pragma unroll
        for (int e = 0; e < NE; ++e) {
          uint32_t d[4];
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            uint32_t a = (e < 2) ? vr[2 * jj].x : vr[2 * jj].y, b = (e < 2) ? vr[2 * jj + 1].x : vr[2 * jj + 1].y;
            d[jj] = (e & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
          }
          v4u vb = v4u{d[0], d[1], d[2], d[3]};
          o[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pA, __builtin_bit_cast(bf16x8, vb), o[e], 0, 0, 0);
        }
      } else {  // HD == 64: two dims per column
        uint32_t vr[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) vr[j] = *(const uint32_t *)(Vs + (k2 * 16 + half * 8 + j) * L::ROW + col * 4);
#pragma unroll
        for (int e = 0; e < NE; ++e) {
          uint32_t d[4];
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            uint32_t a = vr[2 * jj], b = vr[2 * jj + 1];
            d[jj] = (e & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
          }
          v4u vb = v4u{d[0], d[1], d[2], d[3]};
          o[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pA, __builtin_bit_cast(bf16x8, vb), o[e], 0, 0, 0);
        }
      }
    }
  }
  // ---- fold the wavefront's lanes (l), then the four wavefronts, in wavefront order
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int x = 16; x > 0; x >>= 1) l_run[i] += __shfl_xor(l_run[i], x, 64);
  __syncthreads();   // every wavefront is past its last LDS tile; the staging area is reused for the merge
  {
    float *mo = (float *)(lds + w * L::MERGE_PER_WAVE);      // [8][HD] then m[8], l[8]
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
      for (int i = 0; i < 4; ++i) mo[(half * 4 + i) * HD + NE * col + e] = o[e][i];
    if (col == 0)
#pragma unroll
      for (int i = 0; i < 4; ++i) { mo[8 * HD + half * 4 + i] = m_run[i]; mo[8 * HD + 8 + half * 4 + i] = l_run[i]; }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < grp * HD; idx += 256) {
    int r = idx / HD, dd = idx % HD;
    float mw[ATT_WAVES], M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < ATT_WAVES; ++ww) { mw[ww] = ((float *)(lds + ww * L::MERGE_PER_WAVE))[8 * HD + r]; M = fmaxf(M, mw[ww]); }
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int ww = 0; ww < ATT_WAVES; ++ww) {
      const float *mo = (const float *)(lds + ww * L::MERGE_PER_WAVE);
      float f = __expf(mw[ww] - M);
      acc += mo[r * HD + dd] * f;
      lsum += mo[8 * HD + 8 + r] * f;
    }
    if (DIRECT) {
      Xp[k8_index(m, (kvh * grp + r) * HD + dd, Mp)] = f32_to_bf16_bits(acc / lsum);
    } else {
      int64_t pi = ((int64_t)m * Hq + kvh * grp + r) * nsplit + c;
      part_o[pi * HD + dd] = acc;
      if (dd == 0) { part_ml[pi * 2] = M; part_ml[pi * 2 + 1] = lsum; }
    }
  }
}

// grid (M, Hq), block HD: merge the chunk partials of one (row, head) in chunk order, normalise, write bf16 K8.
template <int HD>
__global__ void attn_combine_kernel(uint16_t *Xp, const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                    RowState rows, int Mp, int Hq, int nsplit) {
  int m = blockIdx.x, j = blockIdx.y, dd = threadIdx.x;
  int64_t xi = k8_index(m, j * HD + dd, Mp);
  if (!rows.active[m]) { Xp[xi] = 0; return; }
  int n_keys = rows.pos[m] + 1, per = att_split_len(n_keys, nsplit), ns = (n_keys + per - 1) / per;
  int64_t pi = ((int64_t)m * Hq + j) * nsplit;
  float M = -INFINITY;
  for (int c = 0; c < ns; ++c) M = fmaxf(M, part_ml[(pi + c) * 2]);
  float acc = 0.f, lsum = 0.f;
  for (int c = 0; c < ns; ++c) {
    float f = __expf(part_ml[(pi + c) * 2] - M);
    acc += part_o[(pi + c) * HD + dd] * f;
    lsum += part_ml[(pi + c) * 2 + 1] * f;
  }
  Xp[xi] = f32_to_bf16_bits(acc / lsum);
}

// Splits per row: enough workgroups (rows x KV heads x splits) to put two on every compute unit, never more
// than max_splits (the capacity of the partial buffers).  One split needs no partials and no combine launch.
int fast_attention_splits(int M, int Hkv, int max_splits) {
  int ns = 640 / (M * Hkv);
  if (ns < 1) ns = 1;
  return ns < max_splits ? ns : max_splits;
}

template <int HD>
static void attention_launch(void *Xp_out, const void *q_bf16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq, int Hkv,
                             int nsplit, float *part_o, float *part_ml, hipStream_t st) {
  dim3 grid(nsplit, Hkv, M);
  if (nsplit == 1) {
    hipLaunchKernelGGL((attn_splitk_kernel<HD, true>), grid, dim3(256), AttLds<HD>::TOTAL, st, part_o, part_ml, (uint16_t *)Xp_out,
                       Mp, (const uint16_t *)q_bf16, rows, kv, layer, Hq, Hkv, nsplit);
  } else {
    hipLaunchKernelGGL((attn_splitk_kernel<HD, false>), grid, dim3(256), AttLds<HD>::TOTAL, st, part_o, part_ml, (uint16_t *)Xp_out,
                       Mp, (const uint16_t *)q_bf16, rows, kv, layer, Hq, Hkv, nsplit);
    hipLaunchKernelGGL(attn_combine_kernel<HD>, dim3(M, Hq), dim3(HD), 0, st, (uint16_t *)Xp_out, part_o, part_ml, rows, Mp, Hq,
                       nsplit);
  }
}

void fast_attention(void *Xp_out, const void *q_bf16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq, int Hkv,
                    int nsplit, float *part_o, float *part_ml, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)attn_splitk_kernel<128, true>, hipFuncAttributeMaxDynamicSharedMemorySize, AttLds<128>::TOTAL);
    (void)hipFuncSetAttribute((const void *)attn_splitk_kernel<128, false>, hipFuncAttributeMaxDynamicSharedMemorySize, AttLds<128>::TOTAL);
    (void)hipFuncSetAttribute((const void *)attn_splitk_kernel<64, true>, hipFuncAttributeMaxDynamicSharedMemorySize, AttLds<64>::TOTAL);
    (void)hipFuncSetAttribute((const void *)attn_splitk_kernel<64, false>, hipFuncAttributeMaxDynamicSharedMemorySize, AttLds<64>::TOTAL);
    attr_set = true;
  }
  if (kv.head_dim == 128) attention_launch<128>(Xp_out, q_bf16, rows, kv, layer, M, Mp, Hq, Hkv, nsplit, part_o, part_ml, st);
  else attention_launch<64>(Xp_out, q_bf16, rows, kv, layer, M, Mp, Hq, Hkv, nsplit, part_o, part_ml, st);
}

}  // namespace echo
