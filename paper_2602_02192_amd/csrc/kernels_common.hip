// Small kernels used by both the debug (fp32) and the MFMA (bf16) path: rotary table, per-step
// bookkeeping, KV replication across a group, generator read-out, fills and row gathers.
#include "echo_device.h"
#include "echo_kernels.h"

namespace echo {

// cos/sin of pos * base^(-2i/hd), evaluated in double and stored as fp32: cs[m][i] = (cos, sin).
__global__ void rope_table_kernel(float2 *cs, const int32_t *pos, int M, int half, int hd, float base) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= M * half) return;
  int m = idx / half, i = idx % half;
  int p = pos[m];
  if (p < 0) p = 0;
  double theta = pow((double)base, -2.0 * (double)i / (double)hd);
  double ang = (double)p * theta, s, c;
  sincos(ang, &s, &c);
  cs[idx] = make_float2((float)c, (float)s);
}

void launch_rope_table(float *cs, const int32_t *pos, int M, int hd, float base, hipStream_t st) {
  int half = hd / 2, n = M * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, (float2 *)cs, pos, M, half, hd, base);
}

// One block.  Records the token sampled at generation step *d_step for every active sequence, chooses the
// token fed back (forced or sampled), applies the stop rules and prepares the rows of the next decode pass.
// per_row: the sequences of the batch did not start together, a row's generation step is its gen_len.
__global__ void bookkeeping_kernel(int N, int max_new, int per_row, int32_t *d_step, const int32_t *samp_tok, const float *samp_lp,
                                   const int32_t *forced, const int32_t *limit, int eos, int64_t version,
                                   const int32_t *prompt_len, int32_t *gen_len, RowState rows, int32_t *out_tok,
                                   float *out_lp, int64_t *out_ver, int32_t *n_active) {
  __shared__ int cnt;
  if (threadIdx.x == 0) cnt = 0;
  __syncthreads();
  const int s0 = *d_step;
  int mine = 0;
  for (int n = threadIdx.x; n < N; n += blockDim.x) {
    if (!rows.active[n]) continue;
    const int s = per_row ? gen_len[n] : s0;
    int tok = samp_tok[n];
    int64_t o = (int64_t)rows.slot[n] * max_new + s;   // records are kept per cache slot (= row unless rows were compacted)
    out_tok[o] = tok;
    out_lp[o] = samp_lp[n];
    out_ver[o] = version;
    int fed = forced ? forced[o] : tok;
    int len = s + 1;
    gen_len[n] = len;
    bool done = (len >= limit[n]) || (eos >= 0 && fed == eos);
    rows.token[n] = fed;
    rows.pos[n] = prompt_len[n] + s;
    rows.active[n] = done ? 0 : 1;
    mine += done ? 0 : 1;
  }
  if (mine) atomicAdd(&cnt, mine);
  __syncthreads();
  if (threadIdx.x == 0) { *d_step = s0 + 1; *n_active = cnt; }
}

void launch_bookkeeping(int N, int max_new, int per_row, int32_t *d_step, const int32_t *samp_tok, const float *samp_lp,
                        const int32_t *forced, const int32_t *limit, int eos, int64_t version,
                        const int32_t *prompt_len, int32_t *gen_len, RowState rows, int32_t *out_tok, float *out_lp,
                        int64_t *out_ver, int32_t *n_active, hipStream_t st) {
  hipLaunchKernelGGL(bookkeeping_kernel, dim3(1), dim3(256), 0, st, N, max_new, per_row, d_step, samp_tok, samp_lp, forced,
                     limit, eos, version, prompt_len, gen_len, rows, out_tok, out_lp, out_ver, n_active);
}

// Copy the prompt part of slot p*G into slots p*G+1 .. p*G+G-1.  grid = (chunks, regions per slot, P*(G-1)).
// Plain form: a region is one head's K or V plane and the prompt is its first prompt_len rows.  Tiled form: a region
// is one head's K and V tiles and the prompt is its first ceil(prompt_len/32) tiles.
__global__ void kv_replicate_kernel(KvGeom kv, const int32_t *prompt_len, int G) {
  int p = blockIdx.z / (G - 1), g = blockIdx.z % (G - 1) + 1;
  int64_t region_bytes = kv.head_stride() * kv.elt_bytes * (kv.tiled ? 2 : 1);
  int64_t bytes = kv.tiled ? (int64_t)((prompt_len[p] + 31) / 32) * 64 * kv.head_dim * kv.elt_bytes
                           : (int64_t)prompt_len[p] * kv.head_dim * kv.elt_bytes;
  const char *src = (const char *)kv.base + ((int64_t)p * G) * kv.slot_stride() * kv.elt_bytes + blockIdx.y * region_bytes;
  char *dst = (char *)kv.base + ((int64_t)p * G + g) * kv.slot_stride() * kv.elt_bytes + blockIdx.y * region_bytes;
  int64_t n16 = bytes / 16;  // head_dim * elt_bytes is a multiple of 16
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x)
    ((uint4 *)dst)[i] = ((const uint4 *)src)[i];
}

void launch_kv_replicate(KvGeom kv, const int32_t *prompt_len, int P, int G, hipStream_t st) {
  if (G <= 1 || P <= 0) return;
  int regions = kv.n_layers * kv.n_kv_heads * (kv.tiled ? 1 : 2);
  hipLaunchKernelGGL(kv_replicate_kernel, dim3(8, regions, P * (G - 1)), dim3(256), 0, st, kv, prompt_len, G);
}

// Copy part of one cache slot's prompt into another slot, for a list of (src slot, dst slot, begin, end) quadruples.
// grid = (chunks, regions per slot, pairs).  Plain form: a region is one head's K or V plane and [begin, end) are rows
// (keys); tiled form: a region is one head's K and V tiles and [begin, end) are tiles of 32 keys.
__global__ void kv_copy_range_kernel(KvGeom kv, const int32_t *quads) {
  const int32_t *q = quads + 4 * blockIdx.z;
  int64_t unit_bytes = (kv.tiled ? 64 : 1) * (int64_t)kv.head_dim * kv.elt_bytes;
  int64_t region_bytes = kv.head_stride() * kv.elt_bytes * (kv.tiled ? 2 : 1);
  int64_t off = (int64_t)q[2] * unit_bytes, bytes = (int64_t)(q[3] - q[2]) * unit_bytes;
  if (bytes <= 0) return;
  const char *src = (const char *)kv.base + (int64_t)q[0] * kv.slot_stride() * kv.elt_bytes + blockIdx.y * region_bytes + off;
  char *dst = (char *)kv.base + (int64_t)q[1] * kv.slot_stride() * kv.elt_bytes + blockIdx.y * region_bytes + off;
  int64_t n16 = bytes / 16;  // head_dim * elt_bytes is a multiple of 16
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x)
    ((uint4 *)dst)[i] = ((const uint4 *)src)[i];
}

void launch_kv_copy_ranges(KvGeom kv, const int32_t *quads, int n_quads, hipStream_t st) {
  if (n_quads <= 0) return;
  int regions = kv.n_layers * kv.n_kv_heads * (kv.tiled ? 1 : 2);
  hipLaunchKernelGGL(kv_copy_range_kernel, dim3(8, regions, n_quads), dim3(256), 0, st, kv, quads);
}

__global__ void draw_bits_kernel(uint32_t *out, uint64_t seed, uint32_t n, uint32_t s, uint32_t i0, int count) {
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= count) return;
  uint32_t i = i0 + (uint32_t)j;
  u32x4 r = draw4(seed, n, s, i >> 2);
  uint32_t w[4] = {r.x, r.y, r.z, r.w};
  out[j] = w[i & 3u];
}

void launch_draw_bits(uint32_t *out, uint64_t seed, uint32_t n, uint32_t s, uint32_t i0, int count, hipStream_t st) {
  hipLaunchKernelGGL(draw_bits_kernel, dim3((count + 255) / 256), dim3(256), 0, st, out, seed, n, s, i0, count);
}

__global__ void fill_i32_kernel(int32_t *p, int32_t v, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

void launch_fill_i32(int32_t *p, int32_t v, int64_t n, hipStream_t st) {
  if (n <= 0) return;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, v, n);
}

__global__ void gather_rows_kernel(float *dst, const float *src, const int32_t *src_row, int width) {
  int r = src_row[blockIdx.x];
  if (r < 0) return;
  for (int i = threadIdx.x; i < width; i += blockDim.x) dst[(int64_t)blockIdx.x * width + i] = src[(int64_t)r * width + i];
}

void launch_gather_rows_f32(float *dst, const float *src, const int32_t *src_row, int n_dst, int width, hipStream_t st) {
  if (n_dst <= 0) return;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(n_dst), dim3(256), 0, st, dst, src, src_row, width);
}

// Group-wise normalised advantages (App. "Outcome-Based Returns and Group-wise Normalization"): one wave per group of
// G consecutive returns; mean and sample standard deviation (divisor G - 1) in double, A = (R - mean) / (std + eps).
__global__ void grpo_advantage_kernel(float *adv, const float *rewards, int G, float eps) {
  const float *r = rewards + (int64_t)blockIdx.x * G;
  int lane = threadIdx.x;
  double sum = 0;
  for (int j = lane; j < G; j += 64) sum += (double)r[j];
  for (int o = 32; o; o >>= 1) sum += __shfl_xor(sum, o);
  double mean = sum / G, ss = 0;
  for (int j = lane; j < G; j += 64) {
    double dv = (double)r[j] - mean;
    ss += dv * dv;
  }
  for (int o = 32; o; o >>= 1) ss += __shfl_xor(ss, o);
  double den = sqrt(ss / (G - 1)) + (double)eps;
  for (int j = lane; j < G; j += 64) adv[(int64_t)blockIdx.x * G + j] = (float)(((double)r[j] - mean) / den);
}

// Turn-aware response mask (App. "Turn-Aware Masking") and per-token advantages: one workgroup of 1024 threads per
// sequence walks the row in tiles of 4096 tokens, 4 consecutive tokens per thread; the turn index of a token is the
// carried count of turn starts plus a prefix sum over the tile (shuffles within a wave, LDS across the 16 waves).
// VEC: rows start 16-byte aligned (stride % 4 == 0), so the 4 tokens travel as one vector.
template <bool VEC>
__global__ void __launch_bounds__(1024) grpo_mask_kernel(uint8_t *mask, float *adv_tok, const int32_t *tokens, const int32_t *lens,
                                                        const float *adv, int stride, int32_t turn_start) {
  __shared__ int wave_tot[16];
  int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int32_t *row = tokens + (int64_t)n * stride;
  uint8_t *mrow = mask + (int64_t)n * stride;
  float *arow = adv_tok ? adv_tok + (int64_t)n * stride : nullptr;
  int len = lens[n];
  float a = adv[n];
  int carry = 0;
  for (int base = 0; base < stride; base += 4096) {
    int t0 = base + 4 * tid;
    int32_t tk[4];
    if (VEC && t0 + 3 < stride) {
      int4 v = *(const int4 *)(row + t0);
      tk[0] = v.x, tk[1] = v.y, tk[2] = v.z, tk[3] = v.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) tk[j] = t0 + j < stride ? row[t0 + j] : turn_start - 1;
    }
    int hit[4], cnt = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      hit[j] = (t0 + j < len && tk[j] == turn_start) ? 1 : 0;
      cnt += hit[j];
    }
    int inc = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      int up = __shfl_up(inc, o);
      if (lane >= o) inc += up;
    }
    if (lane == 63) wave_tot[w] = inc;
    __syncthreads();
    int before = carry + inc - cnt, total = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      if (k < w) before += wave_tot[k];
      total += wave_tot[k];
    }
    carry += total;
    __syncthreads();
    int c = before;
    uint8_t m[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      c += hit[j];
      m[j] = (t0 + j < len && c > 1 && (c & 1)) ? 1 : 0;
    }
    if (VEC && t0 + 3 < stride) {
      *(uchar4 *)(mrow + t0) = make_uchar4(m[0], m[1], m[2], m[3]);
      if (arow) *(float4 *)(arow + t0) = make_float4(m[0] ? a : 0.f, m[1] ? a : 0.f, m[2] ? a : 0.f, m[3] ? a : 0.f);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (t0 + j < stride) {
          mrow[t0 + j] = m[j];
          if (arow) arow[t0 + j] = m[j] ? a : 0.f;
        }
    }
  }
}

void launch_grpo_tensors(uint8_t *mask, float *adv, float *adv_tok, const int32_t *tokens, const int32_t *lens, const float *rewards,
                         int n_seqs, int G, int stride, int32_t turn_start, float eps, hipStream_t st) {
  if (n_seqs <= 0) return;
  hipLaunchKernelGGL(grpo_advantage_kernel, dim3(n_seqs / G), dim3(64), 0, st, adv, rewards, G, eps);
  if (stride % 4 == 0)
    hipLaunchKernelGGL(grpo_mask_kernel<true>, dim3(n_seqs), dim3(1024), 0, st, mask, adv_tok, tokens, lens, adv, stride, turn_start);
  else
    hipLaunchKernelGGL(grpo_mask_kernel<false>, dim3(n_seqs), dim3(1024), 0, st, mask, adv_tok, tokens, lens, adv, stride, turn_start);
}

}  // namespace echo
