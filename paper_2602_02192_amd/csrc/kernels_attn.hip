// MFMA path: grouped-query decode attention over the tiled per-sequence KV cache.
//
// attn_simple_kernel: one wavefront per (row, query head), two passes, no split -- the plain form, kept as
//   the on-GPU cross-check of the split-K kernel.
// attn_splitk_kernel: one workgroup per (row, KV head, split of the keys).  Its wavefronts take tiles of 32 keys
//   in turn.  A tile's K and V are stored in MFMA operand order (see KvGeom), so a wavefront streams them from
//   HBM straight into operand registers with contiguous 1 KiB loads, one tile ahead of the one being computed; the
//   loop touches no LDS.  The group's query heads share every tile.  S^T = K Q^T and O^T = V^T P^T run on MFMA
//   (keys and head dims on the 32-row side, the group's query heads on the column side), with an online softmax
//   whose state lives in the lanes of each query-head column.  Per-wavefront and per-split partial (max, sum,
//   acc) are merged in a fixed order (no atomics): by the workgroup through LDS, by attn_combine_kernel across
//   splits.
// attn_rows_kernel: the same loop with several rows of the batch per workgroup, for batches that give every compute unit
//   two rows and more: the prompt tiles that neighbouring rows of one group share are loaded and multiplied once.
// attn_prefix_kernel: a group's shared prompt tiles once for all its rows, as partials that attn_splitk_kernel folds in.
// attn_prefill_kernel: causal attention over runs of consecutive positions (prefill, teacher-forced scoring).
#include <type_traits>

#include "echo_device.h"
#include "echo_kernels.h"

namespace echo {

// Xp (half K8 [Mp][Hq*hd]) element (m, n)
__device__ __forceinline__ int64_t k8_index(int m, int n, int Mp) { return ((int64_t)(n >> 3) * Mp + m) * 8 + (n & 7); }

// grid (M, Hq), block 64, dynamic LDS max_ctx floats; hd <= 256, hd % 64 == 0.
__global__ void attn_simple_kernel(uint16_t *Xp, const uint16_t *q_h16, RowState rows, KvGeom kv, int layer, int Mp, int Hq,
                                   int Hkv) {
  extern __shared__ float sc[];
  int m = blockIdx.x, j = blockIdx.y, lane = threadIdx.x, hd = kv.head_dim;
  if (!rows.active[m]) {
    for (int i = lane; i < hd; i += 64) Xp[k8_index(m, j * hd + i, Mp)] = 0;
    return;
  }
  int n_keys = rows.pos[m] + 1, kvh = j / (Hq / Hkv);
  const uint16_t *head = (const uint16_t *)kv.base + kv.tiled_head_off(rows.slot[m], layer, kvh);
  const uint16_t *q = q_h16 + ((int64_t)m * Hq + j) * hd;
  float scale = 1.0f / sqrtf((float)hd), mx = -INFINITY;
  for (int t = lane; t < n_keys; t += 64) {
    float s = 0.f;
    for (int i = 0; i < hd; ++i) s += h16_bits_to_f32(q[i]) * h16_bits_to_f32(head[kv.tiled_k_off(t, i)]);
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
    for (int t = 0; t < n_keys; ++t) acc += sc[t] * h16_bits_to_f32(head[kv.tiled_v_off(t, i)]);
    Xp[k8_index(m, j * hd + i, Mp)] = f32_to_h16_bits(acc / den);
  }
}

void fast_attention_simple(void *Xp_out, const void *q_h16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq,
                           int Hkv, hipStream_t st) {
  hipLaunchKernelGGL(attn_simple_kernel, dim3(M, Hq), dim3(64), (size_t)kv.max_ctx * sizeof(float), st, (uint16_t *)Xp_out,
                     (const uint16_t *)q_h16, rows, kv, layer, Mp, Hq, Hkv);
}

// ---- split-K MFMA kernel -----------------------------------------------------------------------------
// MFMA roles (v_mfma_f32_32x32x16_f16; lane l: half = l/32, col = l%32).
// S^T = K Q^T: A = K tile (row = key of the tile, k = 16 head dims), B = Q^T (column = query head of the group, zero
//   beyond the group); accumulator register 4g+i of a lane holds the score of key 8g + 4*half + i for head `col`.
// O^T = V^T P^T: A = V tile (row = head dim 32e + row, k = 16 keys), B = P^T (column = query head); register 4g+i
//   of accumulator e holds head dim 32e + 8g + 4*half + i for head `col`.
// So everything a query head needs (running max, running sum, its column of O^T) sits in the two lanes of its column,
// and rescaling is lane-local.
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
constexpr int ATT_TILE = 32;     // keys per tile
constexpr int ATT_WAVES = 4;

template <int HD> struct AttLds {
  static constexpr int MERGE_PER_WAVE = 8 * HD * 4 + 64;    // O rows of up to 8 query heads + (m, l)
  static constexpr int Q_BYTES = 8 * HD * 2;                // the group's queries (B operands are re-read per tile)
  static constexpr int TOTAL = ATT_WAVES * MERGE_PER_WAVE + Q_BYTES;
};

// Keys per split of a row with n_keys keys cut into nsplit equal parts (whole tiles).
__device__ __forceinline__ int att_split_len(int n_keys, int nsplit) {
  return ((n_keys + nsplit - 1) / nsplit + ATT_TILE - 1) & ~(ATT_TILE - 1);
}

// A tile is 64*HD halves = HD*8 units of 16 bytes: the K tile, then the V tile; lane l of load i reads unit i*64 + l.
// STREAM: the tile is read once (decode) and should not displace anything in the caches; the causal block kernel
// reads every tile from many wavefronts and wants it cached.
template <int HD, bool STREAM = true>
__device__ __forceinline__ void att_issue_k(v4u (&rk)[HD / 16], const v4u *__restrict__ head, int tile, int lane) {
  const v4u *t = head + (int64_t)tile * (HD * 8) + lane;
#pragma unroll
  for (int i = 0; i < HD / 16; ++i) rk[i] = STREAM ? __builtin_nontemporal_load(t + i * 64) : t[i * 64];
}
template <int HD, bool STREAM = true>
__device__ __forceinline__ void att_issue_v(v4u (&rv)[HD / 16], const v4u *__restrict__ head, int tile, int lane) {
  const v4u *t = head + (int64_t)tile * (HD * 8) + HD * 4 + lane;
#pragma unroll
  for (int i = 0; i < HD / 16; ++i) rv[i] = STREAM ? __builtin_nontemporal_load(t + i * 64) : t[i * 64];
}

// grid (nsplit, Hkv, M).  Every row's keys are cut into nsplit equal chunks of that row's own length.  DIRECT
// (nsplit == 1): the workgroup normalises and writes the half-precision output itself and no partials exist.
// DIRECT with np > 0: rows whose ptiles carry ATT_PREFIX_DONE skip their group's shared prompt tiles and fold in the
// partials attn_prefix_kernel left for them (np chunk slots per (row, head), prefix_tpc tiles per chunk).
template <int HD, bool DIRECT>
__global__ __launch_bounds__(256, 2) void attn_splitk_kernel(float *__restrict__ part_o, float *__restrict__ part_ml,
                                                          uint16_t *__restrict__ Xp, int Mp, const uint16_t *__restrict__ q_h16,
                                                          RowState rows, KvGeom kv, int layer, int Hq, int Hkv, int nsplit,
                                                          int np, int prefix_tpc) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  using L = AttLds<HD>;
  constexpr int KS = HD / 16;          // k-steps of K Q^T; also 1 KiB loads per K (or V) tile
  constexpr int NE = HD / 32;          // 32-dim blocks of the head
  const int c = blockIdx.x, kvh = blockIdx.y, m = blockIdx.z;
  const int grp = Hq / Hkv;
  if (!rows.active[m]) {
    if (DIRECT)
      for (int idx = threadIdx.x; idx < grp * HD; idx += 256) Xp[k8_index(m, kvh * grp * HD + idx, Mp)] = 0;
    return;
  }
  const int n_keys = rows.pos[m] + 1, chunk_keys = att_split_len(n_keys, nsplit), key0 = c * chunk_keys;
  if (key0 >= n_keys) return;
  const int key1 = min(n_keys, key0 + chunk_keys), ntiles = (key1 - key0 + ATT_TILE - 1) / ATT_TILE, tile0 = key0 / ATT_TILE;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const v4u *head = (const v4u *)((const uint16_t *)kv.base + kv.tiled_head_off(rows.slot[m], layer, kvh));
  // The whole tiles of the group's prompt are identical in every sequence of the group; all of them read the copy of
  // one slot, so the tiles reach HBM once per group and the other sequences find them in L2 (workgroups of one KV head
  // land on one XCD, i.e. behind one L2).
  const v4u *head_sh = (const v4u *)((const uint16_t *)kv.base + kv.tiled_head_off(rows.pslot[m], layer, kvh));
  const int ptiles_raw = rows.ptiles[m], ptiles = ptiles_raw & ~ATT_PREFIX_DONE;
  const bool pre = DIRECT && np > 0 && (ptiles_raw & ATT_PREFIX_DONE);

  // One K and one V register tile per wavefront.  The next tile's K is requested as soon as K Q^T has consumed the
  // current one, the next V as soon as V^T P^T has; loads return in order, so waiting for V leaves the next K in flight.
  v4u rk[KS], rv[KS];
  // (streaming loads for the shared tiles too: measured faster than cached loads, the concurrent misses of a group merge)
  auto issue_k = [&](int t) { att_issue_k<HD, true>(rk, t < ptiles ? head_sh : head, t, lane); };
  auto issue_v = [&](int t) { att_issue_v<HD, true>(rv, t < ptiles ? head_sh : head, t, lane); };
  int tile = (pre ? ptiles : 0) + w;
  if (tile < ntiles) { issue_k(tile0 + tile); issue_v(tile0 + tile); }

  // the group's queries as B operands in LDS: unit (ks*2 + half)*8 + head holds dims ks*16 + half*8 .. +8 of one head
  v4u *qs = (v4u *)(lds + ATT_WAVES * L::MERGE_PER_WAVE);
  for (int idx = threadIdx.x; idx < 8 * (HD / 8); idx += 256) {
    int hq = idx & 7, d8 = idx >> 3;
    v4u v = v4u{0u, 0u, 0u, 0u};
    if (hq < grp) v = *(const v4u *)(q_h16 + ((int64_t)m * Hq + kvh * grp + hq) * HD + d8 * 8);
    qs[idx] = v;
  }
  __syncthreads();

  const float scale = 1.0f / sqrtf((float)HD);
  float m_run = -INFINITY, l_run = 0.f;   // of query head `col` (lanes of one column agree on m_run; l_run is per half)
  f32x16 o[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[e][r] = 0.f;

  auto step = [&](auto more_tag) {
    constexpr bool more = decltype(more_tag)::value;
    // ---- S^T = K Q^T
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      v4u qb = v4u{0u, 0u, 0u, 0u};
      if (col < 8) qb = qs[(ks * 2 + half) * 8 + col];
      s = mfma_h16(__builtin_bit_cast(h16x8, rk[ks]), __builtin_bit_cast(h16x8, qb), s);
    }
    // the MFMAs above read rk when they issue; the loads below write rk when the data arrives, after them
    if (more) issue_k(tile0 + tile + ATT_WAVES);
    // ---- online softmax for head `col` over the tile's keys (register 4g+i: key 8g + 4*half + i)
    const int kbase = key0 + tile * ATT_TILE + 4 * half;
    float tm = -INFINITY;
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float sv = (kbase + 8 * g + i < key1) ? s[4 * g + i] * scale : -INFINITY;
        s[4 * g + i] = sv;
        tm = fmaxf(tm, sv);
      }
    tm = fmaxf(tm, __shfl_xor(tm, 32, 64));
    const float mn = fmaxf(m_run, tm);
    const float alpha = __expf(m_run - mn);
    m_run = mn;
    float ls = 0.f;
    uint32_t pk[8];   // bf16 pairs: pk[2g + i/2] = keys 8g + 4*half + {i, i+1}
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int i = 0; i < 4; i += 2) {
        float p0 = __expf(s[4 * g + i] - mn), p1 = __expf(s[4 * g + i + 1] - mn);
        ls += p0 + p1;
        pk[2 * g + (i >> 1)] = (uint32_t)f32_to_h16_bits(p0) | ((uint32_t)f32_to_h16_bits(p1) << 16);
      }
    l_run = l_run * alpha + ls;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int e = 0; e < NE; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[e][r] *= alpha;
    }
    // ---- O^T += V^T P^T.  The B operand of k-step ks2 wants keys 16*ks2 + 8*half + 0..7 of head `col`: the first
    // four sit in the half-0 lane of the column (its registers of group g = 2*ks2 + half), the last four in the half-1 lane.
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const int ga = 2 * ks2, gb = 2 * ks2 + 1;   // half-0 lanes keep group ga and send gb; half-1 lanes the reverse
      uint32_t s0 = half ? pk[2 * ga] : pk[2 * gb], s1 = half ? pk[2 * ga + 1] : pk[2 * gb + 1];
      uint32_t r0 = __shfl_xor(s0, 32, 64), r1 = __shfl_xor(s1, 32, 64);
      uint32_t m0 = half ? pk[2 * gb] : pk[2 * ga], m1 = half ? pk[2 * gb + 1] : pk[2 * ga + 1];
      v4u pb = half ? v4u{r0, r1, m0, m1} : v4u{m0, m1, r0, r1};
#pragma unroll
      for (int e = 0; e < NE; ++e)
        o[e] = mfma_h16(__builtin_bit_cast(h16x8, rv[ks2 * NE + e]), __builtin_bit_cast(h16x8, pb), o[e]);
    }
    if (more) issue_v(tile0 + tile + ATT_WAVES);
  };
  // every tile but the wavefront's last requests its successor unconditionally: a load behind a condition would make
  // the compiler's wait counts assume it was not issued, and the waits that follow would drain the queue
  for (; tile + ATT_WAVES < ntiles; tile += ATT_WAVES) step(std::true_type{});
  if (tile < ntiles) step(std::false_type{});
  // ---- the two lanes of a column add their sums; then the four wavefronts are folded in wavefront order
  l_run += __shfl_xor(l_run, 32, 64);
  {
    float *mo = (float *)(lds + w * L::MERGE_PER_WAVE);      // [8][HD] then m[8], l[8]
    if (col < grp) {
#pragma unroll
      for (int e = 0; e < NE; ++e)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int i = 0; i < 4; ++i) mo[col * HD + 32 * e + 8 * g + 4 * half + i] = o[e][4 * g + i];
      if (half == 0) { mo[8 * HD + col] = m_run; mo[8 * HD + 8 + col] = l_run; }
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < grp * HD; idx += 256) {
    int r = idx / HD, dd = idx % HD;
    float mw[ATT_WAVES], M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < ATT_WAVES; ++ww) { mw[ww] = ((float *)(lds + ww * L::MERGE_PER_WAVE))[8 * HD + r]; M = fmaxf(M, mw[ww]); }
    // the chunks of the shared prompt, computed once for the whole group
    const int npc = pre ? (ptiles + prefix_tpc - 1) / prefix_tpc : 0;
    const int64_t ppi = ((int64_t)m * Hq + kvh * grp + r) * np;
    for (int pc = 0; pc < npc; ++pc) M = fmaxf(M, part_ml[(ppi + pc) * 2]);
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int ww = 0; ww < ATT_WAVES; ++ww) {
      const float *mo = (const float *)(lds + ww * L::MERGE_PER_WAVE);
      float f = __expf(mw[ww] - M);   // a wavefront that saw no tile has max -inf and weight 0
      acc += mo[r * HD + dd] * f;
      lsum += mo[8 * HD + 8 + r] * f;
    }
    for (int pc = 0; pc < npc; ++pc) {
      float f = __expf(part_ml[(ppi + pc) * 2] - M);
      acc += part_o[(ppi + pc) * HD + dd] * f;
      lsum += part_ml[(ppi + pc) * 2 + 1] * f;
    }
    if (DIRECT) {
      Xp[k8_index(m, (kvh * grp + r) * HD + dd, Mp)] = f32_to_h16_bits(acc / lsum);
    } else {
      int64_t pi = ((int64_t)m * Hq + kvh * grp + r) * nsplit + c;
      part_o[pi * HD + dd] = acc;
      if (dd == 0) { part_ml[pi * 2] = M; part_ml[pi * 2 + 1] = lsum; }
    }
  }
}

// ---- the shared prompt of a group, once for all its sequences ---------------------------------------------------
// grid (chunks, Hkv, jobs).  A job is up to 32 / grp sequences of one group: the MFMA column side, which the kernel above
// fills with one sequence's grp query heads, here carries (sequence, head) pairs of the whole job, so a prompt tile is
// loaded and multiplied once per job instead of once per sequence.  Chunk c covers the whole prompt tiles
// c * tiles_per_chunk .. of the job's prompt slot (no masking: every key of a whole tile is a prompt key).  The result is
// the partial (max, sum, acc) of every (row, head) for that chunk, in slot c of the row's np chunk slots.
template <int HD> struct AttPxLds {
  static constexpr int MERGE_PER_WAVE = 32 * HD * 4 + 256;   // O columns of 32 (sequence, head) pairs + m[32], l[32]
  static constexpr int Q_BYTES = 32 * HD * 2;
  static constexpr int TOTAL = ATT_WAVES * MERGE_PER_WAVE + Q_BYTES;
};

template <int HD>
__global__ __launch_bounds__(256, 2) void attn_prefix_kernel(float *__restrict__ part_o, float *__restrict__ part_ml,
                                                          const uint16_t *__restrict__ q_h16, const PrefixJob *__restrict__ jobs,
                                                          KvGeom kv, int layer, int Hq, int Hkv, int tiles_per_chunk, int np) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  using L = AttPxLds<HD>;
  constexpr int KS = HD / 16, NE = HD / 32;
  const int c = blockIdx.x, kvh = blockIdx.y;
  const PrefixJob *job = jobs + blockIdx.z;
  const int nrows = job->nrows, t0 = c * tiles_per_chunk, t1 = min(job->ptiles, t0 + tiles_per_chunk);
  if (nrows <= 0 || t0 >= t1) return;
  const int grp = Hq / Hkv;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const v4u *head = (const v4u *)((const uint16_t *)kv.base + kv.tiled_head_off(job->pslot, layer, kvh));
  v4u rk[KS], rv[KS];
  // cached loads: the jobs of a large group (more than 32 / grp sequences) read the same tiles
  auto issue_k = [&](int t) { att_issue_k<HD, false>(rk, head, t, lane); };
  auto issue_v = [&](int t) { att_issue_v<HD, false>(rv, head, t, lane); };
  int tile = t0 + w;
  if (tile < t1) { issue_k(tile); issue_v(tile); }

  // queries as B operands: unit (ks*2 + half)*32 + column holds dims ks*16 + half*8 .. +8 of column = sequence*grp + head
  v4u *qs = (v4u *)(lds + ATT_WAVES * L::MERGE_PER_WAVE);
  for (int idx = threadIdx.x; idx < 32 * (HD / 8); idx += 256) {
    int cc = idx & 31, d8 = idx >> 5, si = cc / grp, hq = cc - si * grp;
    v4u v = v4u{0u, 0u, 0u, 0u};
    if (si < nrows) v = *(const v4u *)(q_h16 + ((int64_t)job->rows[si] * Hq + kvh * grp + hq) * HD + d8 * 8);
    qs[idx] = v;
  }
  __syncthreads();

  const float scale = 1.0f / sqrtf((float)HD);
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 o[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[e][r] = 0.f;

  auto step = [&](auto more_tag) {
    constexpr bool more = decltype(more_tag)::value;
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      s = mfma_h16(__builtin_bit_cast(h16x8, rk[ks]), __builtin_bit_cast(h16x8, qs[(ks * 2 + half) * 32 + col]), s);
    if (more) issue_k(tile + ATT_WAVES);
    float tm = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] *= scale; tm = fmaxf(tm, s[r]); }
    tm = fmaxf(tm, __shfl_xor(tm, 32, 64));
    const float mn = fmaxf(m_run, tm);
    const float alpha = __expf(m_run - mn);
    m_run = mn;
    float ls = 0.f;
    uint32_t pk[8];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int i = 0; i < 4; i += 2) {
        float p0 = __expf(s[4 * g + i] - mn), p1 = __expf(s[4 * g + i + 1] - mn);
        ls += p0 + p1;
        pk[2 * g + (i >> 1)] = (uint32_t)f32_to_h16_bits(p0) | ((uint32_t)f32_to_h16_bits(p1) << 16);
      }
    l_run = l_run * alpha + ls;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int e = 0; e < NE; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[e][r] *= alpha;
    }
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {   // the P^T hand-over between the two lanes of a column, as in the kernel above
      const int ga = 2 * ks2, gb = 2 * ks2 + 1;
      uint32_t s0 = half ? pk[2 * ga] : pk[2 * gb], s1 = half ? pk[2 * ga + 1] : pk[2 * gb + 1];
      uint32_t r0 = __shfl_xor(s0, 32, 64), r1 = __shfl_xor(s1, 32, 64);
      uint32_t m0 = half ? pk[2 * gb] : pk[2 * ga], m1 = half ? pk[2 * gb + 1] : pk[2 * ga + 1];
      v4u pb = half ? v4u{r0, r1, m0, m1} : v4u{m0, m1, r0, r1};
#pragma unroll
      for (int e = 0; e < NE; ++e)
        o[e] = mfma_h16(__builtin_bit_cast(h16x8, rv[ks2 * NE + e]), __builtin_bit_cast(h16x8, pb), o[e]);
    }
    if (more) issue_v(tile + ATT_WAVES);
  };
  for (; tile + ATT_WAVES < t1; tile += ATT_WAVES) step(std::true_type{});
  if (tile < t1) step(std::false_type{});
  l_run += __shfl_xor(l_run, 32, 64);
  {
    float *mo = (float *)(lds + w * L::MERGE_PER_WAVE);      // [32][HD] then m[32], l[32]
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) mo[col * HD + 32 * e + 8 * g + 4 * half + i] = o[e][4 * g + i];
    if (half == 0) { mo[32 * HD + col] = m_run; mo[32 * HD + 32 + col] = l_run; }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < nrows * grp * HD; idx += 256) {
    int cc = idx / HD, dd = idx % HD, si = cc / grp, hq = cc - si * grp;
    float mw[ATT_WAVES], M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < ATT_WAVES; ++ww) { mw[ww] = ((float *)(lds + ww * L::MERGE_PER_WAVE))[32 * HD + cc]; M = fmaxf(M, mw[ww]); }
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int ww = 0; ww < ATT_WAVES; ++ww) {
      const float *mo = (const float *)(lds + ww * L::MERGE_PER_WAVE);
      float f = __expf(mw[ww] - M);
      acc += mo[cc * HD + dd] * f;
      lsum += mo[32 * HD + 32 + cc] * f;
    }
    int64_t pi = ((int64_t)job->rows[si] * Hq + kvh * grp + hq) * np + c;
    part_o[pi * HD + dd] = acc;
    if (dd == 0) { part_ml[pi * 2] = M; part_ml[pi * 2 + 1] = lsum; }
  }
}

// grid (M, Hq), block HD: merge the chunk partials of one (row, head) in chunk order, normalise, write half K8.
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
  Xp[xi] = f32_to_h16_bits(acc / lsum);
}

// Splits per row: enough workgroups (rows x KV heads x splits) to put two on every compute unit, never more
// than max_splits (the capacity of the partial buffers).  One split needs no partials and no combine launch.
int fast_attention_splits(int M, int Hkv, int max_splits) {
  int ns = 640 / (M * Hkv);
  if (ns < 1) ns = 1;
  return ns < max_splits ? ns : max_splits;
}

template <int HD>
static void attention_launch(void *Xp_out, const void *q_h16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq, int Hkv,
                             int nsplit, float *part_o, float *part_ml, PrefixPlan px, hipStream_t st) {
  dim3 grid(nsplit, Hkv, M);
  if (nsplit == 1) {
    const bool pre = px.n_jobs > 0 && px.np > 0;
    hipLaunchKernelGGL((attn_splitk_kernel<HD, true>), grid, dim3(256), AttLds<HD>::TOTAL, st, part_o, part_ml, (uint16_t *)Xp_out,
                       Mp, (const uint16_t *)q_h16, rows, kv, layer, Hq, Hkv, nsplit, pre ? px.np : 0, px.tiles_per_chunk);
  } else {
    hipLaunchKernelGGL((attn_splitk_kernel<HD, false>), grid, dim3(256), AttLds<HD>::TOTAL, st, part_o, part_ml, (uint16_t *)Xp_out,
                       Mp, (const uint16_t *)q_h16, rows, kv, layer, Hq, Hkv, nsplit, 0, 1);
    hipLaunchKernelGGL(attn_combine_kernel<HD>, dim3(M, Hq), dim3(HD), 0, st, (uint16_t *)Xp_out, part_o, part_ml, rows, Mp, Hq,
                       nsplit);
  }
}

// ---- several rows of the batch per workgroup ---------------------------------------------------------------------
// A decode batch with more (row, KV head) pairs than the chip has room for at once gives every compute unit several of them
// anyway; a workgroup of eight wavefronts that takes up to R rows (R * grp <= 32 MFMA columns, column = row * grp + head)
// can then take the whole prompt tiles that rows of one group have in common once for all of them: the tile is loaded
// and multiplied once, every column keeps its own softmax state.  A row's remaining tiles follow with the other rows'
// columns masked.  attn_rows_plan_kernel, once per decode step, deals the rows that are still generating to the launch's
// NG row sets in order and evenly (so a batch that has partly drained still gives every workgroup the same number of rows,
// to within one), and writes for every set its rows and a list of segments of whole tiles (cache slot, first tile,
// columns, number of valid keys) -- the same for every layer and KV head.  Lane i of every wavefront holds segment i, so
// finding the segment of a tile is a ballot and a few lane reads, with no memory access on the way to the tile's
// address.  The wavefronts take the workgroup's tiles in turn, one K and one V register tile each, exactly as in
// attn_splitk_kernel.
constexpr int ATT_ROWS_MAX = 8;            // rows per workgroup at most
constexpr int ATT_ROWS_WAVES = 8;
constexpr int ATT_ROWS_BATCH_MAX = 1024;   // rows of a batch that the plan kernel (one workgroup) deals
constexpr int ATT_SEG_MAX = 24;            // runs of rows with a common prompt (<= R/2) + two segments per row
constexpr int ATT_SEG_INTS = 8;            // cache slot, first tile, first and end position in the workgroup's tile list, first and end column, valid keys
constexpr int ATT_HDR_INTS = 16;           // number of rows, tiles in all, the rows
constexpr int ATT_PLAN_INTS = ATT_HDR_INTS + ATT_SEG_MAX * ATT_SEG_INTS;

// One workgroup of ATT_ROWS_BATCH_MAX threads, thread m for row m; NG row sets, each of at most R rows (NG * R >= M).
__global__ __launch_bounds__(ATT_ROWS_BATCH_MAX) void attn_rows_plan_kernel(int32_t *__restrict__ plan, RowState rows, int M, int grp, int NG, int R) {
  __shared__ int32_t f[ATT_ROWS_BATCH_MAX][4];   // prompt slot, whole prompt tiles, keys, slot
  __shared__ int32_t order[ATT_ROWS_BATCH_MAX];  // the rows that are generating, in row order
  __shared__ int32_t wtot[ATT_ROWS_BATCH_MAX / 64 + 1];
  const int t = threadIdx.x, w = t >> 6, lane = t & 63;
  const bool val = t < M && rows.active[t] != 0;
  if (val) { f[t][0] = rows.pslot[t]; f[t][1] = rows.ptiles[t] & ~ATT_PREFIX_DONE; f[t][2] = rows.pos[t] + 1; f[t][3] = rows.slot[t]; }
  const uint64_t bal = __ballot(val);
  if (lane == 0) wtot[w] = __popcll(bal);
  __syncthreads();
  int rank = __popcll(bal & ((1ull << lane) - 1)), n_act = 0;
  for (int i = 0; i < ATT_ROWS_BATCH_MAX / 64; ++i) { if (i < w) rank += wtot[i]; n_act += wtot[i]; }
  if (val) order[rank] = t;
  __syncthreads();
  // set t takes the generating rows of rank ceil(t n / NG) .. ceil((t + 1) n / NG) - 1: at most ceil(n / NG) <= R of them
  const int first = (int)(((int64_t)t * n_act + NG - 1) / NG), end = (int)(((int64_t)(t + 1) * n_act + NG - 1) / NG), nr = t < NG ? end - first : 0;
  // The sets go into the list longest first (by tiles, shared ones counted per row): workgroups start in list order, so
  // when a launch has more workgroups than the chip holds at once the short ones fill in behind the long ones.
  int mine = 0;
  for (int r = 0; r < nr; ++r) mine += (f[order[first + r]][2] + ATT_TILE - 1) / ATT_TILE;
  __shared__ int32_t tot[ATT_ROWS_BATCH_MAX];
  if (t < NG) tot[t] = mine;
  __syncthreads();
  if (t >= NG) return;
  int place = 0;
  for (int u = 0; u < NG; ++u) place += tot[u] > mine || (tot[u] == mine && u < t);
  int32_t *hdr = plan + (int64_t)place * ATT_PLAN_INTS, *seg = hdr + ATT_HDR_INTS;
  int ns = 0, v = 0;
  auto emit = [&](int slot, int tile0, int n, int c0, int c1, int keys) {
    int32_t *s = seg + ns * ATT_SEG_INTS;
    s[0] = slot; s[1] = tile0; s[2] = v; s[3] = v + n; s[4] = c0; s[5] = c1; s[6] = keys; s[7] = 0;
    v += n;
    ++ns;
  };
  for (int r = 0; r < nr;) {
    const int32_t *a = f[order[first + r]];
    const int ps = a[0], pt = a[1];
    int r2 = r + 1, full = a[2] / ATT_TILE;
    while (r2 < nr) {
      const int32_t *b = f[order[first + r2]];
      if (b[0] != ps || b[1] != pt) break;
      full = min(full, b[2] / ATT_TILE);
      ++r2;
    }
    const int sh = r2 - r >= 2 ? min(pt, full) : 0;   // whole tiles that every row of the run reads from the same slot
    if (sh > 0) emit(ps, 0, sh, r * grp, r2 * grp, 0x7fffffff);
    for (int rr = r; rr < r2; ++rr) {
      const int32_t *b = f[order[first + rr]];
      const int nk = b[2], nt = (nk + ATT_TILE - 1) / ATT_TILE;
      int a0 = sh;
      const int e0 = min(pt, nt);
      if (e0 > a0) { emit(ps, a0, e0 - a0, rr * grp, (rr + 1) * grp, nk); a0 = e0; }   // prompt tiles the row reads alone
      if (nt > a0) emit(b[3], a0, nt - a0, rr * grp, (rr + 1) * grp, nk);
    }
    r = r2;
  }
  for (int i = ns; i < ATT_SEG_MAX; ++i) {   // unused entries lie beyond every tile
    int32_t *s = seg + i * ATT_SEG_INTS;
    s[0] = 0; s[1] = 0; s[2] = 0x7fffffff; s[3] = 0x7fffffff; s[4] = 0; s[5] = 0; s[6] = 0; s[7] = 0;
  }
  hdr[0] = nr; hdr[1] = v;
  for (int r = 0; r < ATT_ROWS_MAX; ++r) hdr[2 + r] = r < nr ? order[first + r] : -1;
}

template <int HD> struct AttRowsLds {
  static constexpr int Q_BYTES = 32 * HD * 2;
  // per wavefront: O^T of its columns as [head dim][ncols + 1] floats (the odd stride spreads a store over the banks), then m[32], l[32]
  __host__ __device__ static int merge_per_wave(int ncols) { return HD * (ncols + 1) * 4 + 256; }
  __host__ __device__ static int total(int ncols) { return Q_BYTES + ATT_ROWS_WAVES * merge_per_wave(ncols); }
};

// grid (1, Hkv, NG), block 512; R = the most rows a set can hold (NG * R >= M).
template <int HD>
__global__ __launch_bounds__(ATT_ROWS_WAVES * 64) void attn_rows_kernel(uint16_t *__restrict__ Xp, int Mp, const uint16_t *__restrict__ q_h16,
                                                                       const int32_t *__restrict__ plan, const int32_t *__restrict__ row_active,
                                                                       KvGeom kv, int layer, int Hq, int Hkv, int M, int R) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  using L = AttRowsLds<HD>;
  constexpr int KS = HD / 16, NE = HD / 32, NW = ATT_ROWS_WAVES;
  const int kvh = blockIdx.y, gi = blockIdx.z, NG = gridDim.z, grp = Hq / Hkv, ncols = R * grp;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int32_t *hdr = plan + (int64_t)gi * ATT_PLAN_INTS;

  // lane i holds segment i of the workgroup's list; lanes 32 .. 47 the header (number of rows, tiles in all, the rows)
  int sg_slot = 0, sg_tile0 = 0, sg_v0 = 0x7fffffff, sg_v1 = 0x7fffffff, sg_c0 = 0, sg_c1 = 0, sg_keys = 0, hd_word = 0;
  if (lane < ATT_SEG_MAX) {
    const int4 *sp = (const int4 *)(hdr + ATT_HDR_INTS + lane * ATT_SEG_INTS);
    const int4 a = sp[0], b = sp[1];
    sg_slot = a.x; sg_tile0 = a.y; sg_v0 = a.z; sg_v1 = a.w; sg_c0 = b.x; sg_c1 = b.y; sg_keys = b.z;
  } else if (lane >= 32 && lane < 32 + ATT_HDR_INTS) {
    hd_word = hdr[lane - 32];
  }
  const int nrows = __builtin_amdgcn_readlane(hd_word, 32), V = __builtin_amdgcn_readlane(hd_word, 33);
  const int64_t head_units = (int64_t)HD * 8;   // 16-byte units per tile (K then V)
  const v4u *cache = (const v4u *)kv.base;
  const int64_t lk_off = ((int64_t)layer * kv.layer_stride() + (int64_t)kvh * 2 * kv.head_stride()) / 8;   // in 16-byte units
  const int64_t slot_units = kv.slot_stride() / 8;

  struct Loc { const v4u *tile; int tile_idx, c0, c1, keys; };
  auto locate = [&](int v) {
    const int s = __popcll(__ballot(sg_v1 <= v));   // segments that end at or before v: the index of v's segment
    Loc l;
    const int slot = __builtin_amdgcn_readlane(sg_slot, s);
    l.tile_idx = __builtin_amdgcn_readlane(sg_tile0, s) + v - __builtin_amdgcn_readlane(sg_v0, s);
    l.c0 = __builtin_amdgcn_readlane(sg_c0, s);
    l.c1 = __builtin_amdgcn_readlane(sg_c1, s);
    l.keys = __builtin_amdgcn_readlane(sg_keys, s);
    l.tile = cache + (int64_t)slot * slot_units + lk_off + (int64_t)l.tile_idx * head_units + lane;
    return l;
  };
  v4u rk[KS], rv[KS];
  auto issue_k = [&](const Loc &l) {
#pragma unroll
    for (int i = 0; i < KS; ++i) rk[i] = __builtin_nontemporal_load(l.tile + i * 64);
  };
  auto issue_v = [&](const Loc &l) {
#pragma unroll
    for (int i = 0; i < KS; ++i) rv[i] = __builtin_nontemporal_load(l.tile + HD * 4 + i * 64);
  };
  int v = w;
  Loc cur = locate(v < V ? v : 0), nxt = cur;
  if (v < V) {
    // in the order the loop issues them (K then V, each in k-step order): the wait counts of the loop are the merge of
    // this path and the loop's own, and a first tile requested in another order would make every trip wait for more
#pragma unroll
    for (int i = 0; i < KS; ++i) { rk[i] = __builtin_nontemporal_load(cur.tile + i * 64); __builtin_amdgcn_sched_barrier(0); }
#pragma unroll
    for (int i = 0; i < KS; ++i) { rv[i] = __builtin_nontemporal_load(cur.tile + HD * 4 + i * 64); __builtin_amdgcn_sched_barrier(0); }
  }

  // the queries of all columns as B operands: unit (ks*2 + half)*32 + column holds dims ks*16 + half*8 .. +8
  v4u *qs = (v4u *)lds;
  for (int idx = threadIdx.x; idx < 32 * (HD / 8); idx += NW * 64) {
    const int cc = idx & 31, d8 = idx >> 5, r = cc / grp, hq = cc - r * grp;
    v4u q = v4u{0u, 0u, 0u, 0u};
    if (r < nrows) q = *(const v4u *)(q_h16 + ((int64_t)hdr[2 + r] * Hq + kvh * grp + hq) * HD + d8 * 8);
    qs[idx] = q;
  }
  __syncthreads();

  const float scale = 1.0f / sqrtf((float)HD);
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 o[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[e][r] = 0.f;

  auto step = [&](auto more_tag) {
    constexpr bool more = decltype(more_tag)::value;
    if (more) nxt = locate(v + NW);
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      s = mfma_h16(__builtin_bit_cast(h16x8, rk[ks]), __builtin_bit_cast(h16x8, qs[(ks * 2 + half) * 32 + col]), s);
    if (more) issue_k(nxt);
    // a column outside the segment's rows sees no key of this tile
    const int klim = (col >= cur.c0 && col < cur.c1) ? cur.keys : 0;
    const int kbase = cur.tile_idx * ATT_TILE + 4 * half;
    float tm = -INFINITY;
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float sv = (kbase + 8 * g + i < klim) ? s[4 * g + i] * scale : -INFINITY;
        s[4 * g + i] = sv;
        tm = fmaxf(tm, sv);
      }
    tm = fmaxf(tm, __shfl_xor(tm, 32, 64));
    const float mn = fmaxf(m_run, tm);
    const float mref = mn == -INFINITY ? 0.f : mn;             // a column that has seen no key yet: every p is exp(-inf) = 0
    const float alpha = m_run == mn ? 1.0f : __expf(m_run - mref);
    m_run = mn;
    float ls = 0.f;
    uint32_t pk[8];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int i = 0; i < 4; i += 2) {
        float p0 = __expf(s[4 * g + i] - mref), p1 = __expf(s[4 * g + i + 1] - mref);
        ls += p0 + p1;
        pk[2 * g + (i >> 1)] = (uint32_t)f32_to_h16_bits(p0) | ((uint32_t)f32_to_h16_bits(p1) << 16);
      }
    l_run = l_run * alpha + ls;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int e = 0; e < NE; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[e][r] *= alpha;
    }
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {   // the P^T hand-over between the two lanes of a column, as in attn_splitk_kernel
      const int ga = 2 * ks2, gb = 2 * ks2 + 1;
      uint32_t s0 = half ? pk[2 * ga] : pk[2 * gb], s1 = half ? pk[2 * ga + 1] : pk[2 * gb + 1];
      uint32_t r0 = __shfl_xor(s0, 32, 64), r1 = __shfl_xor(s1, 32, 64);
      uint32_t m0_ = half ? pk[2 * gb] : pk[2 * ga], m1_ = half ? pk[2 * gb + 1] : pk[2 * ga + 1];
      v4u pb = half ? v4u{r0, r1, m0_, m1_} : v4u{m0_, m1_, r0, r1};
#pragma unroll
      for (int e = 0; e < NE; ++e)
        o[e] = mfma_h16(__builtin_bit_cast(h16x8, rv[ks2 * NE + e]), __builtin_bit_cast(h16x8, pb), o[e]);
    }
    if (more) { issue_v(nxt); cur = nxt; }
  };
  for (; v + NW < V; v += NW) step(std::true_type{});
  if (v < V) step(std::false_type{});

  // ---- the two lanes of a column add their sums; then the wavefronts are folded in wavefront order
  l_run += __shfl_xor(l_run, 32, 64);
  const int ncp = ncols + 1, mpw = L::merge_per_wave(ncols);
  char *mg = lds + L::Q_BYTES;
  if (col < ncols) {
    float *mo = (float *)(mg + w * mpw);
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) mo[(32 * e + 8 * g + 4 * half + i) * ncp + col] = o[e][4 * g + i];
    if (half == 0) { mo[HD * ncp + col] = m_run; mo[HD * ncp + 32 + col] = l_run; }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < nrows * grp * HD; idx += NW * 64) {
    const int cc = idx / HD, dd = idx % HD, r = cc / grp, hq = cc - r * grp;
    float mw[NW], Mx = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) { mw[ww] = ((const float *)(mg + ww * mpw))[HD * ncp + cc]; Mx = fmaxf(Mx, mw[ww]); }
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      const float *mo = (const float *)(mg + ww * mpw);
      const float f = mw[ww] == -INFINITY ? 0.f : __expf(mw[ww] - Mx);   // a wavefront that saw no key of the column
      acc += mo[dd * ncp + cc] * f;
      lsum += mo[HD * ncp + 32 + cc] * f;
    }
    Xp[k8_index(hdr[2 + r], (kvh * grp + hq) * HD + dd, Mp)] = f32_to_h16_bits(acc / lsum);
  }
  // rows that are not generating belong to no set: their outputs are zero; workgroup gi clears rows gi, gi + NG, ..
  for (int m = gi; m < M; m += NG) {
    if (row_active[m]) continue;
    for (int idx = threadIdx.x; idx < grp * HD; idx += NW * 64) Xp[k8_index(m, kvh * grp * HD + idx, Mp)] = 0;
  }
}

// Row sets of a launch over M rows: one workgroup per compute unit where the batch allows (sets x KV heads >= 256), more
// when a set would otherwise need more rows than the MFMA columns hold.  mode 3: as few sets as the columns allow.
static int attention_row_sets(int M, int Hq, int Hkv, int mode) {
  const int grp = Hq / Hkv, rmax = 32 / grp < ATT_ROWS_MAX ? 32 / grp : ATT_ROWS_MAX;
  const int need = (M + rmax - 1) / rmax, fill = mode == 3 ? 1 : (256 + Hkv - 1) / Hkv;
  return need > fill ? need : fill;
}

int fast_attention_rows_per_group(int M, int Hq, int Hkv, int mode) {
  const int grp = Hq / Hkv;
  if (mode == 1 || mode == 2 || 32 / grp < 2 || M < 2 || M > ATT_ROWS_BATCH_MAX) return 1;
  const int NG = attention_row_sets(M, Hq, Hkv, mode);
  if (mode != 3 && M < 2 * NG) return 1;   // fewer than two rows per compute unit: one row per workgroup, keys split where it pays
  return (M + NG - 1) / NG;
}

size_t fast_attention_plan_ints(int max_rows) { return (size_t)(max_rows < ATT_ROWS_BATCH_MAX ? max_rows : ATT_ROWS_BATCH_MAX) * ATT_PLAN_INTS; }

void fast_attention_rows_plan(int32_t *plan, RowState rows, int M, int Hq, int Hkv, int mode, hipStream_t st) {
  const int NG = attention_row_sets(M, Hq, Hkv, mode);
  hipLaunchKernelGGL(attn_rows_plan_kernel, dim3(1), dim3(ATT_ROWS_BATCH_MAX), 0, st, plan, rows, M, Hq / Hkv, NG, (M + NG - 1) / NG);
}

template <int HD>
static void attention_rows_launch(void *Xp_out, const void *q_h16, const int32_t *plan, RowState rows, KvGeom kv, int layer, int M, int Mp,
                                  int Hq, int Hkv, int mode, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)attn_rows_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, AttRowsLds<HD>::total(32));
    attr_set = true;
  }
  const int NG = attention_row_sets(M, Hq, Hkv, mode), R = (M + NG - 1) / NG;
  hipLaunchKernelGGL(attn_rows_kernel<HD>, dim3(1, Hkv, NG), dim3(ATT_ROWS_WAVES * 64), AttRowsLds<HD>::total(R * (Hq / Hkv)), st,
                     (uint16_t *)Xp_out, Mp, (const uint16_t *)q_h16, plan, rows.active, kv, layer, Hq, Hkv, M, R);
}

void fast_attention_rows(void *Xp_out, const void *q_h16, const int32_t *plan, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq,
                         int Hkv, int mode, hipStream_t st) {
  if (kv.head_dim == 128) attention_rows_launch<128>(Xp_out, q_h16, plan, rows, kv, layer, M, Mp, Hq, Hkv, mode, st);
  else attention_rows_launch<64>(Xp_out, q_h16, plan, rows, kv, layer, M, Mp, Hq, Hkv, mode, st);
}

// ---- causal kernel for runs of consecutive positions ---------------------------------------------------
// grid (blocks, Hkv), eight wavefronts per workgroup (two per SIMD, so one's MFMAs run under the other's softmax).
// A block is up to 8 * 32 / grp consecutive rows of one cache slot; wavefront w carries rows w * 32/grp .. as one tile
// of 32 columns, a column being a (row, query head of the KV head's group) pair: column index = row_in_wavefront * grp
// + head.  The wavefronts need the same K / V tiles, so the workgroup fetches every tile once: all threads load it
// two tiles ahead into staging
// registers, store it one tile ahead into an LDS double buffer, and the wavefronts read their MFMA A operands from
// there (same MFMA roles as the split-K kernel: S^T = K Q^T, O^T = V^T P^T).  The queries stay in registers as B
// operands.  Keys after a column's own position are masked; only the tiles
// that reach past a wavefront's first position need the mask, and a wavefront skips the tiles past its last row.
// Blocks are taken longest first (the builder emits them by ascending position).
constexpr int ATT_PF_NQ = ATT_PREFILL_COLS / 32;
constexpr float ATT_PF_SLACK = 8.0f;
template <int HD> struct AttPfLds {
  static constexpr int TILE_UNITS = HD * 8;                     // 16-byte units: K tile then V tile
  static constexpr int BYTES = 2 * TILE_UNITS * 16;
};

template <int HD>
__global__ __launch_bounds__(ATT_PREFILL_WAVES * 64) void attn_prefill_kernel(uint16_t *__restrict__ Xp, int Mp, const uint16_t *__restrict__ q_h16,
                                                           const PrefillBlock *__restrict__ blocks, int nblocks, KvGeom kv, int layer,
                                                           int Hq, int Hkv) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  using L = AttPfLds<HD>;
  constexpr int KS = HD / 16, NE = HD / 32, NQ = ATT_PF_NQ, TU = L::TILE_UNITS, NT = ATT_PREFILL_WAVES * 64, PER_T = TU / NT;
  const PrefillBlock b = blocks[nblocks - 1 - blockIdx.x];
  const int kvh = blockIdx.y, grp = Hq / Hkv, rb = ATT_PREFILL_COLS / grp;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, half = lane >> 5, col = lane & 31;
  const int r0 = w * rb, rows_w = max(0, min(rb, b.nrows - r0));   // this wavefront's rows: r0 .. r0 + rows_w - 1 of the block
  const int ntiles = (b.pos0 + b.nrows + ATT_TILE - 1) / ATT_TILE;            // of the workgroup
  const int ntiles_w = rows_w > 0 ? (b.pos0 + r0 + rows_w + ATT_TILE - 1) / ATT_TILE : 0;
  const int nfull_w = rows_w > 0 ? min((b.pos0 + r0 + 1) / ATT_TILE, ntiles_w - 1) : 0;   // tiles that need no mask
  const v4u *head = (const v4u *)((const uint16_t *)kv.base + kv.tiled_head_off(b.slot, layer, kvh));
  v4u *ring = (v4u *)lds;

  v4u stg[2][PER_T];
  auto gload = [&](int st, int tile) {
    const v4u *t = head + (int64_t)min(tile, ntiles - 1) * TU + tid;   // past the end: the last tile again, never used
#pragma unroll
    for (int j = 0; j < PER_T; ++j) stg[st][j] = t[j * NT];
  };
  auto lstore = [&](int st, int buf) {
#pragma unroll
    for (int j = 0; j < PER_T; ++j) ring[buf * TU + j * NT + tid] = stg[st][j];
  };
  gload(0, 0);
  gload(1, 1);

  int pcol[NQ];   // the column's position; a column beyond the wavefront's rows is all zero and unmasked
#pragma unroll
  for (int t = 0; t < NQ; ++t) pcol[t] = (t * 32 + col) / grp < rows_w ? b.pos0 + r0 + (t * 32 + col) / grp : 0x7fffffff;
  v4u qs[NQ * KS];   // qs[t*KS + ks]: dims ks*16 + half*8 .. +8 of column t*32 + col
#pragma unroll
  for (int t = 0; t < NQ; ++t) {
    const int idx = t * 32 + col, r = idx / grp, hh = idx % grp;
    const bool valid = r < rows_w;
    const uint16_t *src = q_h16 + ((int64_t)(b.m0 + r0 + (valid ? r : 0)) * Hq + kvh * grp + hh) * HD + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qs[t * KS + ks] = valid ? *(const v4u *)(src + ks * 16) : v4u{0u, 0u, 0u, 0u};
  }
  lstore(0, 0);
  gload(0, 2);
  __syncthreads();

  // scores are kept in units of log2(e) / sqrt(HD), so the exponentials are bare v_exp_f32 (2^x) instructions
  const float scale2 = 1.44269504088896f / sqrtf((float)HD);
  float m_run[NQ], l_run[NQ];
  f32x16 o[NQ][NE];
#pragma unroll
  for (int t = 0; t < NQ; ++t) {
    m_run[t] = -INFINITY; l_run[t] = 0.f;
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[t][e][r] = 0.f;
  }
  typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));

  auto compute = [&](int tile, int buf, auto mask_tag) {
    constexpr bool mask = decltype(mask_tag)::value;
    const v4u *kt = ring + buf * TU + lane, *vt = kt + HD * 4;
    const int kbase = tile * ATT_TILE + 4 * half;
    v4u rk[KS], rv[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) rk[i] = kt[i * 64];
#pragma unroll
    for (int i = 0; i < KS; ++i) rv[i] = vt[i * 64];
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
      f32x16 sa, sb;   // two chains of HD/32 dependent MFMAs instead of one of HD/16
#pragma unroll
      for (int r = 0; r < 16; ++r) { sa[r] = 0.f; sb[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ks += 2) {
        sa = mfma_h16(__builtin_bit_cast(h16x8, rk[ks]), __builtin_bit_cast(h16x8, qs[t * KS + ks]), sa);
        sb = mfma_h16(__builtin_bit_cast(h16x8, rk[ks + 1]), __builtin_bit_cast(h16x8, qs[t * KS + ks + 1]), sb);
      }
      float tm = -INFINITY;
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float sv = (sa[4 * g + i] + sb[4 * g + i]) * scale2;
          if (mask && kbase + 8 * g + i > pcol[t]) sv = -INFINITY;
          sa[4 * g + i] = sv;
          tm = fmaxf(tm, sv);
        }
      tm = fmaxf(tm, __shfl_xor(tm, 32, 64));
      // The reference exponent only follows the running maximum when that has grown by more than ATT_PF_SLACK (in
      // powers of two): softmax does not depend on the reference, p stays below 2^ATT_PF_SLACK (exact in fp32 sums
      // and well inside the half range), and the accumulators are rescaled a few times per row instead of at almost
      // every tile.  Finite from the first tile on: key 0 is visible to every column.
      const float mn = tm > m_run[t] + ATT_PF_SLACK ? tm : m_run[t];
      const float alpha = __builtin_amdgcn_exp2f(m_run[t] - mn);
      m_run[t] = mn;
      float ls = 0.f;
      uint32_t pk[8];   // half pairs: pk[2g + i/2] = keys 8g + 4*half + {i, i+1}; p <= 1, so the conversion cannot overflow
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < 4; i += 2) {
          float p0 = __builtin_amdgcn_exp2f(sa[4 * g + i] - mn), p1 = __builtin_amdgcn_exp2f(sa[4 * g + i + 1] - mn);
          ls += p0 + p1;
          pk[2 * g + (i >> 1)] = __builtin_bit_cast(uint32_t, h16x2{(_Float16)p0, (_Float16)p1});
        }
      l_run[t] = l_run[t] * alpha + ls;
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int e = 0; e < NE; ++e)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[t][e][r] *= alpha;
      }
      // P^T as B operand of k-step ks2: keys 16*ks2 + 8*half + 0..7 of the column.  Register group 2*ks2 of the half-0
      // lane and group 2*ks2+1 of the half-1 lane stay; the other two cross to the partner lane: v_permlane32_swap
      // exchanges the upper half of its first operand with the lower half of its second, which is exactly that.
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2) {
        const int ga = 2 * ks2, gb = 2 * ks2 + 1;
        auto x0 = __builtin_amdgcn_permlane32_swap(pk[2 * ga], pk[2 * gb], false, false);
        auto x1 = __builtin_amdgcn_permlane32_swap(pk[2 * ga + 1], pk[2 * gb + 1], false, false);
        v4u pb = v4u{x0[0], x1[0], x0[1], x1[1]};
#pragma unroll
        for (int e = 0; e < NE; ++e)
          o[t][e] = mfma_h16(__builtin_bit_cast(h16x8, rv[ks2 * NE + e]), __builtin_bit_cast(h16x8, pb), o[t][e]);
      }
    }
  };
  // Trip i: tile i+1 (loaded two trips ago) goes to the LDS buffer that tile i-1 occupied, its staging registers are
  // refilled with tile i+3, tile i is consumed, and the barrier both publishes tile i+1 and retires tile i.  Loads,
  // stores and barriers are unconditional and the same for every wavefront; only the arithmetic is skipped.
  for (int i0 = 0; i0 < ntiles; i0 += 2) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int i = i0 + s;
      lstore((s + 1) & 1, (s + 1) & 1);
      gload((s + 1) & 1, i + 3);
      if (i < nfull_w) compute(i, s, std::false_type{});
      else if (i < ntiles_w) compute(i, s, std::true_type{});
      __syncthreads();
    }
  }

#pragma unroll
  for (int t = 0; t < NQ; ++t) {
    const float l = l_run[t] + __shfl_xor(l_run[t], 32, 64);
    const int idx = t * 32 + col, r = idx / grp, hh = idx % grp;
    if (r < rows_w) {
      const float inv = 1.0f / l;
#pragma unroll
      for (int e = 0; e < NE; ++e)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 wv;
          wv.x = (uint32_t)f32_to_h16_bits(o[t][e][4 * g] * inv) | ((uint32_t)f32_to_h16_bits(o[t][e][4 * g + 1] * inv) << 16);
          wv.y = (uint32_t)f32_to_h16_bits(o[t][e][4 * g + 2] * inv) | ((uint32_t)f32_to_h16_bits(o[t][e][4 * g + 3] * inv) << 16);
          *(uint2 *)(Xp + k8_index(b.m0 + r0 + r, (kvh * grp + hh) * HD + 32 * e + 8 * g + 4 * half, Mp)) = wv;
        }
    }
  }
}

template <int HD>
static void attention_prefill_launch(void *Xp_out, const void *q_h16, const PrefillBlock *blocks, int nblocks, KvGeom kv, int layer,
                                     int Mp, int Hq, int Hkv, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)attn_prefill_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, AttPfLds<HD>::BYTES);
    attr_set = true;
  }
  hipLaunchKernelGGL(attn_prefill_kernel<HD>, dim3(nblocks, Hkv), dim3(ATT_PREFILL_WAVES * 64), AttPfLds<HD>::BYTES, st, (uint16_t *)Xp_out, Mp,
                     (const uint16_t *)q_h16, blocks, nblocks, kv, layer, Hq, Hkv);
}

void fast_attention_prefill(void *Xp_out, const void *q_h16, const PrefillBlock *blocks, int nblocks, KvGeom kv, int layer, int Mp,
                            int Hq, int Hkv, hipStream_t st) {
  if (nblocks <= 0) return;
  if (kv.head_dim == 128) attention_prefill_launch<128>(Xp_out, q_h16, blocks, nblocks, kv, layer, Mp, Hq, Hkv, st);
  else attention_prefill_launch<64>(Xp_out, q_h16, blocks, nblocks, kv, layer, Mp, Hq, Hkv, st);
}

template <int HD>
static void prefix_launch(const void *q_h16, KvGeom kv, int layer, int Hq, int Hkv, float *part_o, float *part_ml, PrefixPlan px,
                          hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)attn_prefix_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, AttPxLds<HD>::TOTAL);
    attr_set = true;
  }
  hipLaunchKernelGGL(attn_prefix_kernel<HD>, dim3(px.np, Hkv, px.n_jobs), dim3(256), AttPxLds<HD>::TOTAL, st, part_o, part_ml,
                     (const uint16_t *)q_h16, px.jobs, kv, layer, Hq, Hkv, px.tiles_per_chunk, px.np);
}

void fast_attention_prefix(const void *q_h16, KvGeom kv, int layer, int Hq, int Hkv, float *part_o, float *part_ml, PrefixPlan px,
                           hipStream_t st) {
  if (px.n_jobs <= 0 || px.np <= 0) return;
  if (kv.head_dim == 128) prefix_launch<128>(q_h16, kv, layer, Hq, Hkv, part_o, part_ml, px, st);
  else prefix_launch<64>(q_h16, kv, layer, Hq, Hkv, part_o, part_ml, px, st);
}

void fast_attention(void *Xp_out, const void *q_h16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq, int Hkv,
                    int nsplit, float *part_o, float *part_ml, PrefixPlan px, hipStream_t st) {
  if (kv.head_dim == 128) attention_launch<128>(Xp_out, q_h16, rows, kv, layer, M, Mp, Hq, Hkv, nsplit, part_o, part_ml, px, st);
  else attention_launch<64>(Xp_out, q_h16, rows, kv, layer, M, Mp, Hq, Hkv, nsplit, part_o, part_ml, px, st);
}

}  // namespace echo
