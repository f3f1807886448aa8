// MFMA path, dense contractions: weight repacking, the weight-streaming GEMM (split-K over the
// wavefronts of a workgroup and over the grid) with its epilogues, and the lm_head GEMM whose epilogue
// is the sampler (temperature, Gumbel-max, running log-sum-exp), so logits never reach HBM.
//
// Operand roles of v_mfma_f32_32x32x16_f16 here: A = 32 weight rows x 16 k, B = 16 k x 32 batch rows.
// Lane l supplies A[row l%32][k 8*(l/32) .. +8] and B[k 8*(l/32) .. +8][col l%32]; it receives
// D[row 8*g + 4*(l/32) + i][col l%32] in accumulator register 4*g + i (g, i in 0..3).
#include <type_traits>

#include "echo_device.h"
#include "echo_kernels.h"

namespace echo {

// Packed weight addressing, in units of 16 bytes (8 halves): one 32-row block is contiguous over K, a k-step of it is 64 units.
__host__ __device__ __forceinline__ int64_t w_block_base(int nb, int Kp) { return (int64_t)nb * (Kp >> 3) * 32; }
__host__ __device__ __forceinline__ int64_t w_kstep_stride(int) { return 64; }

// ---- weight repacking --------------------------------------------------------------------------------
// src: row-major bf16 [n_rows][K]; destination row of source row i is dst_row0 + i*dst_row_stride.
__global__ void pack_weight_kernel(uint4 *dst, const uint4 *src, int64_t dst_row0, int dst_row_stride, int64_t n_rows,
                                   int K8, int Kp8, int Np) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_rows * K8) return;
  int64_t i = idx / K8;
  int k8 = (int)(idx % K8);
  int64_t r = dst_row0 + i * dst_row_stride;
  uint4 v = src[idx];
  uint32_t w[4] = {v.x, v.y, v.z, v.w}, o[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)   // bf16 pair -> half pair, scaled by W_SCALE (exact)
    o[q] = (uint32_t)f32_to_h16_bits(__uint_as_float(w[q] << 16) * W_SCALE) |
           ((uint32_t)f32_to_h16_bits(__uint_as_float(w[q] & 0xffff0000u) * W_SCALE) << 16);
  dst[w_block_base((int)(r >> 5), Kp8 * 8) + (k8 >> 1) * w_kstep_stride(Np) + (k8 & 1) * 32 + (r & 31)] = make_uint4(o[0], o[1], o[2], o[3]);
}

void fast_pack_weight(void *dst, const void *src, int64_t dst_row0, int dst_row_stride, int64_t n_rows, int K, int Kp,
                      int Np, hipStream_t st) {
  int64_t n = n_rows * (K / 8);
  if (n <= 0) return;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint4 *)dst,
                     (const uint4 *)src, dst_row0, dst_row_stride, n_rows, K / 8, Kp / 8, Np);
}

// Re-pack a span of a matrix: elements [e0, e0 + n) of the row-major bf16 matrix [rows][K] (src holds just those n
// values) replace their places in the packed weight; source row i lives in destination row dst_row0 + i * stride.
// One thread per destination unit of 8 k that the span touches; a unit covered only in part keeps its other values.
__global__ void pack_span_kernel(uint16_t *dst, const uint16_t *src, int64_t e0, int64_t n, int64_t dst_row0, int dst_row_stride, int K,
                                 int Kp8, int Np) {
  const int64_t u0 = e0 >> 3, u = u0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // K % 8 == 0: units never straddle rows
  if (u * 8 >= e0 + n) return;
  const int K8 = K >> 3;
  const int64_t i = u / K8, r = dst_row0 + i * dst_row_stride;
  const int k8 = (int)(u % K8);
  uint16_t *d = dst + (w_block_base((int)(r >> 5), Kp8 * 8) + (k8 >> 1) * w_kstep_stride(Np) + (k8 & 1) * 32 + (r & 31)) * 8;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int64_t e = u * 8 + q;
    if (e >= e0 && e < e0 + n) d[q] = f32_to_h16_bits(bf16_bits_to_f32(src[e - e0]) * W_SCALE);
  }
}

void fast_pack_span(void *dst, const void *src, int64_t e0, int64_t n, int64_t dst_row0, int dst_row_stride, int K, int Kp, int Np,
                    hipStream_t st) {
  if (n <= 0) return;
  const int64_t units = ((e0 + n + 7) >> 3) - (e0 >> 3);
  hipLaunchKernelGGL(pack_span_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, st, (uint16_t *)dst, (const uint16_t *)src, e0, n,
                     dst_row0, dst_row_stride, K, Kp / 8, Np);
}

// A quantised matrix (per-row fp32 scale, int8 codes) back to row-major bf16: the bf16 value nearest to float(code) * scale,
// computed as one fp32 product, ties to even.  One thread per code.
__global__ void dequant_q8_kernel(uint16_t *__restrict__ out, const int8_t *__restrict__ codes, const float *__restrict__ scales,
                                  int64_t n, int K) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  out[i] = f32_to_bf16_bits(__fmul_rn((float)codes[i], scales[i / K]));
}

void fast_dequant_q8(void *out_bf16, const void *codes, const void *scales, int64_t rows, int K, hipStream_t st) {
  const int64_t n = rows * K;
  if (n <= 0) return;
  hipLaunchKernelGGL(dequant_q8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint16_t *)out_bf16, (const int8_t *)codes,
                     (const float *)scales, n, K);
}

// ---- the MFMA inner loop -------------------------------------------------------------------------------
// A wavefront owns NBW consecutive 32-row weight blocks and all MB 32-row batch blocks of its launch slice:
// per k-step it reads NBW KiB of weights and MB KiB of activations, so activation traffic from L2 per weight
// byte falls with NBW.  Loads run two groups of U k-steps ahead of the MFMAs (register double buffer).
template <int MB, int NBW, int U>
struct KGroup {
  h16x8 a[U][NBW];
  h16x8 b[U][MB];
};

template <int MB, int NBW, int U>
__device__ __forceinline__ void load_group(KGroup<MB, NBW, U> &g, const h16x8 *__restrict__ a_ptr, int64_t a_blk,
                                           const h16x8 *__restrict__ b_ptr, int Mp, int ks, int64_t a_step) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int n = 0; n < NBW; ++n) g.a[u][n] = __builtin_nontemporal_load(a_ptr + n * a_blk + (int64_t)(ks + u) * a_step);
    const h16x8 *bp = b_ptr + (int64_t)(ks + u) * 2 * Mp;
#pragma unroll
    for (int j = 0; j < MB; ++j) g.b[u][j] = bp[j * 32];
  }
}

template <int MB, int NBW, int U>
__device__ __forceinline__ void mma_group(f32x16 (&acc)[NBW][MB], const KGroup<MB, NBW, U> &g) {
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int n = 0; n < NBW; ++n)
#pragma unroll
      for (int j = 0; j < MB; ++j)
        acc[n][j] = mfma_h16(g.a[u][n], g.b[u][j], acc[n][j]);
}

// Wnb: first weight block of the wavefront; a_blk: distance between consecutive weight blocks (16-byte units).
template <int MB, int NBW>
__device__ __forceinline__ void mma_range(f32x16 (&acc)[NBW][MB], const h16x8 *__restrict__ Wnb, int64_t a_blk,
                                          const h16x8 *__restrict__ Xp, int Mp, int ks0, int ks1, int lane,
                                          int64_t a_step) {
  constexpr int U0 = 12 / (MB + NBW), U = U0 < 1 ? 1 : (U0 > 4 ? 4 : U0);
  const h16x8 *a_ptr = Wnb + (lane >> 5) * 32 + (lane & 31);
  const h16x8 *b_ptr = Xp + (int64_t)(lane >> 5) * Mp + (lane & 31);
  int ng = (ks1 - ks0) / U;
  KGroup<MB, NBW, U> g0, g1;
  if (ng > 0) load_group<MB, NBW, U>(g0, a_ptr, a_blk, b_ptr, Mp, ks0, a_step);
  for (int g = 0; g < ng; g += 2) {
    if (g + 1 < ng) load_group<MB, NBW, U>(g1, a_ptr, a_blk, b_ptr, Mp, ks0 + (g + 1) * U, a_step);
    mma_group<MB, NBW, U>(acc, g0);
    if (g + 2 < ng) load_group<MB, NBW, U>(g0, a_ptr, a_blk, b_ptr, Mp, ks0 + (g + 2) * U, a_step);
    if (g + 1 < ng) mma_group<MB, NBW, U>(acc, g1);
  }
  for (int ks = ks0 + ng * U; ks < ks1; ++ks) {   // remainder
    KGroup<MB, NBW, 1> r;
    load_group<MB, NBW, 1>(r, a_ptr, a_blk, b_ptr, Mp, ks, a_step);
    mma_group<MB, NBW, 1>(acc, r);
  }
}

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }

// grid (ceil(Np/32 / (NBW*waves_n)), nsplit, Mp/(32*MB)); block 64 * waves_n * waves_k.
// Wavefront w = wk*waves_n + wn: the waves_n wavefronts of one wk share a k-range (their activation reads hit
// L1 together) and own different weight blocks; the waves_k k-ranges of a grid split are summed in LDS in wk order.
template <int MB, int NBW, int EPI>
__global__ __launch_bounds__(512) void gemm_kernel(void *out, const h16x8 *__restrict__ Xp, const h16x8 *__restrict__ Wp,
                                                   int Mp, int Np, int Kp, int ksteps_per_split, int waves_n) {
  extern __shared__ float red[];
  const int waves = blockDim.x >> 6, w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wn = w % waves_n, wk = w / waves_n, nwk = waves / waves_n;
  const int nblocks = Np >> 5, split = blockIdx.y, mblk0 = blockIdx.z * MB;
  const int nb0 = (blockIdx.x * waves_n + wn) * NBW;
  const int ksteps = Kp >> 4;
  const int s0 = split * ksteps_per_split, s1 = min(ksteps, s0 + ksteps_per_split);
  const int per_wave = (s1 - s0 + nwk - 1) / nwk;
  const int k0 = min(s1, s0 + wk * per_wave), k1 = min(s1, k0 + per_wave);
  f32x16 acc[NBW][MB];
#pragma unroll
  for (int n = 0; n < NBW; ++n)
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[n][j][r] = 0.f;
  // blocks past the end re-read the last block (their results are dropped)
  const int nb_ld = min(nb0, nblocks - NBW);
  if (nb0 < nblocks)
    mma_range<MB, NBW>(acc, Wp + w_block_base(nb_ld, Kp), w_block_base(1, Kp), Xp + mblk0 * 32, Mp, k0, k1, lane,
                       w_kstep_stride(Np));
  if (nwk > 1) {
    float *mine = red + (int64_t)((wk - 1) * waves_n + wn) * (NBW * MB * 16 * 64);
    if (wk > 0) {
#pragma unroll
      for (int n = 0; n < NBW; ++n)
#pragma unroll
        for (int j = 0; j < MB; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) mine[((n * MB + j) * 16 + r) * 64 + lane] = acc[n][j][r];
    }
    __syncthreads();
    if (wk == 0) {
      for (int ww = 1; ww < nwk; ++ww) {
        const float *src = red + (int64_t)((ww - 1) * waves_n + wn) * (NBW * MB * 16 * 64);
#pragma unroll
        for (int n = 0; n < NBW; ++n)
#pragma unroll
          for (int j = 0; j < MB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[n][j][r] += src[((n * MB + j) * 16 + r) * 64 + lane];
      }
    }
  }
  if (wk != 0) return;
  const int half = lane >> 5, col = lane & 31;
#pragma unroll
  for (int n = 0; n < NBW; ++n) {
    const int nb = nb0 + n;
    if (nb >= nblocks) continue;
    if (EPI == EPI_PARTIAL) {
      f32x4 *P = (f32x4 *)out;
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        int m = (mblk0 + j) * 32 + col;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          int n4 = nb * 8 + half + 2 * g;
          f32x4 v = {acc[n][j][4 * g], acc[n][j][4 * g + 1], acc[n][j][4 * g + 2], acc[n][j][4 * g + 3]};
          P[((int64_t)split * Mp + m) * (Np >> 2) + n4] = v * W_UNSCALE;
        }
      }
    } else {  // EPI_SWIGLU: rows alternate gate_f, up_f
      uint32_t *O = (uint32_t *)out;
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        int m = (mblk0 + j) * 32 + col;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          int f = nb * 16 + half * 2 + 4 * g;
          float v0 = silu_f(acc[n][j][4 * g] * W_UNSCALE) * (acc[n][j][4 * g + 1] * W_UNSCALE);
          float v1 = silu_f(acc[n][j][4 * g + 2] * W_UNSCALE) * (acc[n][j][4 * g + 3] * W_UNSCALE);
          uint32_t pk = (uint32_t)f32_to_h16_bits(v0) | ((uint32_t)f32_to_h16_bits(v1) << 16);
          O[(((int64_t)(f >> 3) * Mp + m) * 8 + (f & 7)) >> 1] = pk;
        }
      }
    }
  }
}

// ---- weight-streaming GEMM with the activations staged through LDS -----------------------------------------
// Measured on MI355X: a compute unit sustains about 48 GB/s of vector-memory reads whether they come from HBM
// (weights) or from L2 (activations), so activation re-reads cost as much as weight bytes.  Here the WN wavefronts
// of a workgroup own WN consecutive 32-row weight blocks and walk the same k-range in chunks of KC k-steps; a
// chunk of activations (KC x MB KiB) is fetched once per workgroup, coalesced, and shared through LDS, which cuts
// the activation traffic per weight byte to MB/WN.  Weight loads run NSTAGE-1 chunks ahead in registers.  The
// activation loads of a chunk are issued before the weight loads of the same chunk: the memory counter retires in
// order, so waiting for them (to copy them into LDS) leaves every younger weight load in flight.
// grid (ceil(Np/32 / WN), nsplit, Mp/(32*MB)); block 64*WN; chunks_per_split chunks of KC k-steps per grid split.
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));

constexpr int GEMM_KC_SMALL = 8, GEMM_KC_WIDE = 4;   // k-steps per chunk for up to 128 / for 256 batch rows per workgroup
template <int MB, int WN> struct GemmLds {
  static constexpr int KC = MB >= 8 ? GEMM_KC_WIDE : GEMM_KC_SMALL;
  static constexpr int CHUNK_UNITS = KC * 2 * 32 * MB;                  // 16-byte units of one activation chunk
  static constexpr int X_BYTES = 2 * CHUNK_UNITS * 16;                   // double buffer
  static constexpr int TILE_STRIDE = 33;                                 // floats per row of the transposed output tile
  static constexpr int EPI_BYTES = WN * 32 * TILE_STRIDE * 4;            // one 32 x 32 tile per wavefront at a time
  static constexpr int BYTES = X_BYTES > EPI_BYTES ? X_BYTES : EPI_BYTES;
};

// The GEMM kernel's main loop as a function, for the lm_head (the GEMM kernel keeps its own inline copy: hipcc
// schedules the inlined function measurably worse there): accumulates, for weight block `nb` and the 32*MB batch rows from
// mrow0, the k-range of `nchunks` chunks starting at chunk c_begin.  Ends with a workgroup barrier, after which the
// LDS buffers are free for the epilogue.
template <int MB, int WN, int NSTAGE>
__device__ __forceinline__ void gemm_lds_mainloop(f32x16 (&acc)[MB], char *lds_raw, const u32x4v *__restrict__ Xp,
                                                  const h16x8 *__restrict__ Wp, int Mp, int Np, int Kp, int nb, int c_begin,
                                                  int nchunks, int mrow0) {
  using L = GemmLds<MB, WN>;
  constexpr int KC = L::KC, T = WN * 64, XU = L::CHUNK_UNITS, XL = (XU + T - 1) / T, ROWS = 32 * MB;
  u32x4v *xs = (u32x4v *)lds_raw;
  const int lane = threadIdx.x & 63, tid = threadIdx.x;
  const h16x8 *a_ptr = Wp + w_block_base(nb, Kp) + (int64_t)c_begin * KC * w_kstep_stride(Np) + (lane >> 5) * 32 + (lane & 31);
  const int64_t a_step = w_kstep_stride(Np);
#pragma unroll
  for (int j = 0; j < MB; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  h16x8 a[NSTAGE][KC];
  u32x4v xr[NSTAGE][XL];
  auto load_a = [&](int st, int c) {
#pragma unroll
    for (int u = 0; u < KC; ++u) a[st][u] = __builtin_nontemporal_load(a_ptr + (int64_t)(c * KC + u) * a_step);
  };
  // unit i of a chunk: k8 group i / ROWS (two per k-step), batch row i % ROWS
  auto load_x = [&](int st, int c) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      int idx = min(i * T + tid, XU - 1);   // surplus threads repeat the last unit: no divergent branch around a load
      xr[st][i] = Xp[(int64_t)((c_begin + c) * KC * 2 + idx / ROWS) * Mp + mrow0 + idx % ROWS];
    }
  };
  auto store_x = [&](int st, int buf) {
#pragma unroll
    for (int i = 0; i < XL; ++i) xs[buf * XU + min(i * T + tid, XU - 1)] = xr[st][i];
  };
  // The B operands of GU k-steps are read from LDS in one batch ahead of their MFMAs: with one wavefront per SIMD
  // nothing else hides the LDS latency, and a read issued right before each MFMA would expose it every time.
  auto compute = [&](int st, int buf) {
    constexpr int GU = MB >= 8 ? 2 : (MB == 4 ? 4 : KC);
    const u32x4v *bp = xs + buf * XU + (lane >> 5) * ROWS + (lane & 31);
#pragma unroll
    for (int u0 = 0; u0 < KC; u0 += GU) {
      u32x4v b[GU][MB];
#pragma unroll
      for (int u = 0; u < GU; ++u)
#pragma unroll
        for (int j = 0; j < MB; ++j) b[u][j] = bp[(u0 + u) * 2 * ROWS + j * 32];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < GU; ++u)
#pragma unroll
        for (int j = 0; j < MB; ++j) acc[j] = mfma_h16(a[st][u0 + u], __builtin_bit_cast(h16x8, b[u][j]), acc[j]);
    }
  };
  // Every load that the compiler sees behind a condition makes its wait counts assume the load was not issued, and
  // the waits that follow drain the queue.  So the pipeline is written without conditions around loads: prologue,
  // steady trips of NSTAGE chunks, and one straight-line tail per possible number of remaining chunks.
  auto tail = [&](auto r_tag) {
    constexpr int R = decltype(r_tag)::value;   // chunks left; chunk i of them sits in register stage i % NSTAGE
    const int cb = nchunks - R;
#pragma unroll
    for (int i = 0; i < R; ++i) {
      if (i + NSTAGE - 1 < R) { load_x((i + NSTAGE - 1) % NSTAGE, cb + i + NSTAGE - 1); load_a((i + NSTAGE - 1) % NSTAGE, cb + i + NSTAGE - 1); }
      compute(i % NSTAGE, (cb + i) & 1);
      if (i + 1 < R) store_x((i + 1) % NSTAGE, (cb + i + 1) & 1);
      __syncthreads();
    }
  };
  if (nchunks >= NSTAGE - 1) {
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) { load_x(s, s); load_a(s, s); }
    store_x(0, 0);
    __syncthreads();
    int c0 = 0;
    for (; c0 + 2 * NSTAGE - 2 < nchunks; c0 += NSTAGE) {
#pragma unroll
      for (int s = 0; s < NSTAGE; ++s) {
        const int c = c0 + s;
        load_x((s + NSTAGE - 1) % NSTAGE, c + NSTAGE - 1);
        load_a((s + NSTAGE - 1) % NSTAGE, c + NSTAGE - 1);
        compute(s, c & 1);
        store_x((s + 1) % NSTAGE, (c + 1) & 1);
        __syncthreads();
      }
    }
    // NSTAGE-1 .. 2*NSTAGE-2 chunks are left and c0 is a multiple of NSTAGE, so their register stages are static
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "one tail per remaining count");
    switch (nchunks - c0) {
      case 1: if (NSTAGE == 2) tail(std::integral_constant<int, 1>{}); break;
      case 2: if (NSTAGE <= 3) tail(std::integral_constant<int, 2>{}); break;
      case 3: if (NSTAGE >= 3) tail(std::integral_constant<int, 3>{}); break;
      case 4: if (NSTAGE >= 3) tail(std::integral_constant<int, 4>{}); break;
      case 5: if (NSTAGE == 4) tail(std::integral_constant<int, 5>{}); break;
      case 6: if (NSTAGE == 4) tail(std::integral_constant<int, 6>{}); break;
      default: break;
    }
  } else if (nchunks > 0) {   // a K range shorter than the pipeline: guarded loads
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
      if (s < nchunks) { load_x(s, s); load_a(s, s); }
    store_x(0, 0);
    __syncthreads();
    for (int c0 = 0; c0 < nchunks; c0 += NSTAGE) {
#pragma unroll
      for (int s = 0; s < NSTAGE; ++s) {
        const int c = c0 + s;
        if (c < nchunks) {
          if (c + NSTAGE - 1 < nchunks) { load_x((s + NSTAGE - 1) % NSTAGE, c + NSTAGE - 1); load_a((s + NSTAGE - 1) % NSTAGE, c + NSTAGE - 1); }
          compute(s, c & 1);
          if (c + 1 < nchunks) store_x((s + 1) % NSTAGE, (c + 1) & 1);
          __syncthreads();
        }
      }
    }
  }
}

// The 64-row forms with the two-chunk weight pipeline are held to 256 registers per lane (the bound that would let two
// workgroups share a compute unit; these launches have at most one per unit): the code the compiler makes under that
// bound parks nothing in the accumulation half of the register file and measured 0.9 % faster per decode step of the 4B
// model, level on the 32B model.  At 32 rows the bound changes nothing, at 128 rows it forces spills.
template <int MB, int WN, int NSTAGE> constexpr int gemm_lds_min_wgs() { return MB == 2 && NSTAGE == 2 && WN <= 4 ? 2 : 1; }

template <int MB, int WN, int NSTAGE, int EPI>
__global__ __launch_bounds__(WN * 64, (gemm_lds_min_wgs<MB, WN, NSTAGE>())) void gemm_lds_kernel(void *out, const u32x4v *__restrict__ Xp, const h16x8 *__restrict__ Wp,
                                                           int Mp, int Np, int Kp, int chunks_per_split) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  using L = GemmLds<MB, WN>;
  constexpr int KC = L::KC, T = WN * 64, XU = L::CHUNK_UNITS, XL = (XU + T - 1) / T, ROWS = 32 * MB;
  u32x4v *xs = (u32x4v *)lds_raw;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, tid = threadIdx.x;
  const int nblocks = Np >> 5, total_chunks = (Kp >> 4) / KC;
  const int nb_own = blockIdx.x * WN + w, nb = min(nb_own, nblocks - 1);   // wavefronts past the end re-read the last block
  const int c_begin = blockIdx.y * chunks_per_split, nchunks = min(chunks_per_split, total_chunks - c_begin);
  const int mrow0 = blockIdx.z * ROWS;
  const h16x8 *a_ptr = Wp + w_block_base(nb, Kp) + (int64_t)c_begin * KC * w_kstep_stride(Np) + (lane >> 5) * 32 + (lane & 31);
  const int64_t a_step = w_kstep_stride(Np);
  f32x16 acc[MB];
#pragma unroll
  for (int j = 0; j < MB; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  h16x8 a[NSTAGE][KC];
  u32x4v xr[NSTAGE][XL];
  auto load_a = [&](int st, int c) {
#pragma unroll
    for (int u = 0; u < KC; ++u) a[st][u] = __builtin_nontemporal_load(a_ptr + (int64_t)(c * KC + u) * a_step);
  };
  // unit i of a chunk: k8 group i / ROWS (two per k-step), batch row i % ROWS
  auto load_x = [&](int st, int c) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      int idx = min(i * T + tid, XU - 1);   // surplus threads repeat the last unit: no divergent branch around a load
      xr[st][i] = Xp[(int64_t)((c_begin + c) * KC * 2 + idx / ROWS) * Mp + mrow0 + idx % ROWS];
    }
  };
  auto store_x = [&](int st, int buf) {
#pragma unroll
    for (int i = 0; i < XL; ++i) xs[buf * XU + min(i * T + tid, XU - 1)] = xr[st][i];
  };
  // The B operands of GU k-steps are read from LDS in one batch ahead of their MFMAs: with one wavefront per SIMD
  // nothing else hides the LDS latency, and a read issued right before each MFMA would expose it every time.
  auto compute = [&](int st, int buf) {
    constexpr int GU = MB >= 8 ? 2 : (MB == 4 ? 4 : KC);
    const u32x4v *bp = xs + buf * XU + (lane >> 5) * ROWS + (lane & 31);
#pragma unroll
    for (int u0 = 0; u0 < KC; u0 += GU) {
      u32x4v b[GU][MB];
#pragma unroll
      for (int u = 0; u < GU; ++u)
#pragma unroll
        for (int j = 0; j < MB; ++j) b[u][j] = bp[(u0 + u) * 2 * ROWS + j * 32];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < GU; ++u)
#pragma unroll
        for (int j = 0; j < MB; ++j) acc[j] = mfma_h16(a[st][u0 + u], __builtin_bit_cast(h16x8, b[u][j]), acc[j]);
    }
  };
  // Every load that the compiler sees behind a condition makes its wait counts assume the load was not issued, and
  // the waits that follow drain the queue.  So the pipeline is written without conditions around loads: prologue,
  // steady trips of NSTAGE chunks, and one straight-line tail per possible number of remaining chunks.
  auto tail = [&](auto r_tag) {
    constexpr int R = decltype(r_tag)::value;   // chunks left; chunk i of them sits in register stage i % NSTAGE
    const int cb = nchunks - R;
#pragma unroll
    for (int i = 0; i < R; ++i) {
      if (i + NSTAGE - 1 < R) { load_x((i + NSTAGE - 1) % NSTAGE, cb + i + NSTAGE - 1); load_a((i + NSTAGE - 1) % NSTAGE, cb + i + NSTAGE - 1); }
      compute(i % NSTAGE, (cb + i) & 1);
      if (i + 1 < R) store_x((i + 1) % NSTAGE, (cb + i + 1) & 1);
      __syncthreads();
    }
  };
  if (nchunks >= NSTAGE - 1) {
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) { load_x(s, s); load_a(s, s); }
    store_x(0, 0);
    __syncthreads();
    int c0 = 0;
    for (; c0 + 2 * NSTAGE - 2 < nchunks; c0 += NSTAGE) {
#pragma unroll
      for (int s = 0; s < NSTAGE; ++s) {
        const int c = c0 + s;
        load_x((s + NSTAGE - 1) % NSTAGE, c + NSTAGE - 1);
        load_a((s + NSTAGE - 1) % NSTAGE, c + NSTAGE - 1);
        compute(s, c & 1);
        store_x((s + 1) % NSTAGE, (c + 1) & 1);
        __syncthreads();
      }
    }
    // NSTAGE-1 .. 2*NSTAGE-2 chunks are left and c0 is a multiple of NSTAGE, so their register stages are static
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "one tail per remaining count");
    switch (nchunks - c0) {
      case 1: if (NSTAGE == 2) tail(std::integral_constant<int, 1>{}); break;
      case 2: if (NSTAGE <= 3) tail(std::integral_constant<int, 2>{}); break;
      case 3: if (NSTAGE >= 3) tail(std::integral_constant<int, 3>{}); break;
      case 4: if (NSTAGE >= 3) tail(std::integral_constant<int, 4>{}); break;
      case 5: if (NSTAGE == 4) tail(std::integral_constant<int, 5>{}); break;
      case 6: if (NSTAGE == 4) tail(std::integral_constant<int, 6>{}); break;
      default: break;
    }
  } else if (nchunks > 0) {   // a K range shorter than the pipeline: guarded loads
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
      if (s < nchunks) { load_x(s, s); load_a(s, s); }
    store_x(0, 0);
    __syncthreads();
    for (int c0 = 0; c0 < nchunks; c0 += NSTAGE) {
#pragma unroll
      for (int s = 0; s < NSTAGE; ++s) {
        const int c = c0 + s;
        if (c < nchunks) {
          if (c + NSTAGE - 1 < nchunks) { load_x((s + NSTAGE - 1) % NSTAGE, c + NSTAGE - 1); load_a((s + NSTAGE - 1) % NSTAGE, c + NSTAGE - 1); }
          compute(s, c & 1);
          if (c + 1 < nchunks) store_x((s + 1) % NSTAGE, (c + 1) & 1);
          __syncthreads();
        }
      }
    }
  }
  const int half = lane >> 5, col = lane & 31;
  if (EPI == EPI_PARTIAL) {
    // transpose the wavefront's tile through LDS, 32 batch rows at a time, so that every store is a whole 128-byte
    // row segment (the LDS tile is private to the wavefront: only its own LDS traffic has to be waited for)
    float *tile = (float *)lds_raw + (size_t)w * 32 * L::TILE_STRIDE;
    float *P = (float *)out + ((int64_t)blockIdx.y * Mp + mrow0) * Np + nb * 32;
#pragma unroll
    for (int j = 0; j < MB; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[col * L::TILE_STRIDE + 8 * g + 4 * half + i] = acc[j][4 * g + i] * W_UNSCALE;
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (nb_own < nblocks) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          int r = q * 8 + (lane >> 3), n4 = (lane & 7) * 4;
          const float *t = tile + r * L::TILE_STRIDE + n4;
          f32x4 v = {t[0], t[1], t[2], t[3]};
          *(f32x4 *)(P + (int64_t)(j * 32 + r) * Np + n4) = v;
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the reads are done before the next pass overwrites the tile
    }
  } else {  // EPI_SWIGLU: weight rows alternate gate_f, up_f; a block of 32 rows yields 16 features = two K8 groups
    if (nb_own >= nblocks) return;
    uint32_t *O = (uint32_t *)out;
#pragma unroll
    for (int j = 0; j < MB; ++j) {
      uint32_t pk[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {   // features 4g + 2*half + {0,1} of the block
        float v0 = silu_f(acc[j][4 * g] * W_UNSCALE) * (acc[j][4 * g + 1] * W_UNSCALE);
        float v1 = silu_f(acc[j][4 * g + 2] * W_UNSCALE) * (acc[j][4 * g + 3] * W_UNSCALE);
        pk[g] = (uint32_t)f32_to_h16_bits(v0) | ((uint32_t)f32_to_h16_bits(v1) << 16);
      }
      // lane (half 0) assembles K8 group 0 (features 0..7), its partner (half 1) group 1 (features 8..15)
      uint32_t give0 = half ? pk[0] : pk[2], give1 = half ? pk[1] : pk[3];
      uint32_t got0 = __shfl_xor(give0, 32, 64), got1 = __shfl_xor(give1, 32, 64);
      u32x4v o = half ? u32x4v{got0, pk[2], got1, pk[3]} : u32x4v{pk[0], got0, pk[1], got1};
      int m = mrow0 + j * 32 + col;
      *(u32x4v *)(O + (((int64_t)(nb * 2 + half) * Mp + m) * 4)) = o;
    }
  }
}

// ---- the 256 x 256 register-streaming tile of the wide lm_head kernel ----------------------------------------------
// Four wavefronts in a row; every wavefront owns two weight blocks (64 output columns), streamed from global memory
// straight into A-operand registers, against eight blocks of 32 batch rows whose operands come through LDS; every
// activation operand read from LDS feeds two MFMAs.  (The projections used this form too, also as two row halves x two
// column pairs on a 256 x 128 tile, until gemm_ring_kernel below replaced it there.)
struct GemmWide {
  static constexpr int MB = 8, WN = 4, NBW = 2, ROWS = 256, T = WN * 64;
  static constexpr int CK = 1, NSTAGE = 8 / CK;   // k-steps per chunk (one barrier each), chunks in flight; CK = 2 measured 1-2 % slower
  static constexpr int CHUNK_UNITS = CK * 2 * ROWS, XL = CHUNK_UNITS / T;
  static constexpr int X_BYTES = 2 * CHUNK_UNITS * 16, TILE_STRIDE = 33, EPI_BYTES = WN * 32 * TILE_STRIDE * 4;
  static constexpr int BYTES = X_BYTES > EPI_BYTES ? X_BYTES : EPI_BYTES;
};

// ---- 256-row tiles with both operands in an LDS ring: batches of 256 rows and more ------------------------------
// What caps a large-tile GEMM here is what a compute unit can take in per cycle through its vector memory path, so a
// workgroup must fetch every operand byte once: 256 weight columns and 256 batch rows per k-step are 16 KB for 2 MFLOP.
// (A register-streaming form with two row halves fetched every weight block once per row half, 24 KB per k-step, and
// measured 12 - 25 % slower at 4096 rows.)  Eight wavefronts, two per SIMD, as two row halves x four column pairs; wavefront w
// fetches weight block w of the tile's eight and its share of the activation chunk, each as one 1 KB load that lands
// in LDS without passing through registers (global_load_lds, the data of lane l at 16 l); a stage of the ring is one
// k-step: [8 blocks x 64 units of A operands][2 k8 groups x 256 rows of B operands], 16 KB, eight stages.  Step c
// issues the loads of k-step c + LA, reads its two A and four B operands from stage c and runs eight MFMAs; before the
// barrier that ends the step a wavefront waits until its own loads of k-step c + 1 have landed (loads retire in
// order: all but the youngest LA - 1 k-steps' worth), so after the barrier the whole stage c + 1 is there.  The stage that
// step c's loads overwrite held k-step c + LA - 8, whose readers passed the barrier of step c + LA - 8 <= c - 1.
// The wait is written by hand, together with the barrier: the compiler's own barrier sequence would wait for every
// outstanding load and empty the ring.  Sums run in the same order as in the other kernels (k ascending in one
// accumulator), so results are bit-identical.  With WC = 2 the same kernel runs four wavefronts (two row halves x two
// column pairs) on a 256 x 128 tile, 12 KB per k-step: batches of a few hundred rows, where 256 x 256 tiles are too few
// to fill the chip (4 - 15 % faster there than the register-streaming form it replaced).
template <int WCv> struct GemmRingT {   // WC = 4: 256 x 256 tile, eight wavefronts; WC = 2: 256 x 128 tile, four wavefronts
  static constexpr int WR = 2, WC = WCv, WN = WR * WC, MB = 4, NBW = 2, ROWS = 256, T = WN * 64;
  static constexpr int AU = WC * NBW * 64, XU = 2 * ROWS, SU = AU + XU;   // 16-byte units of a stage: A operands, B operands
  static constexpr int XLW = XU / T, LPS = 1 + XLW;                       // activation loads, all loads per wavefront and k-step
  static constexpr int NS = 8, LA = 6;                                    // stages, k-steps ahead (< NS)
  static constexpr int TILE_STRIDE = 33, BYTES = NS * SU * 16;            // 128 KB / 96 KB; the epilogue's WN x 32 x 33 floats reuse it
};

__device__ __forceinline__ void load_to_lds(const void *g, void *l) {   // 16 bytes per lane; l is the wavefront's base, lane l lands at l + 16 l
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g, (__attribute__((address_space(3))) void *)l, 16, 0, 0);
}

template <int EPI, bool ZFAST, int WCv>
__global__ __launch_bounds__(GemmRingT<WCv>::T) void gemm_ring_kernel(void *out, const u32x4v *__restrict__ Xp, const h16x8 *__restrict__ Wp, int Mp,
                                                                int Np, int Kp, int groups_per_split) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  using L = GemmRingT<WCv>;
  constexpr int MB = L::MB, NBW = L::NBW, ROWS = L::ROWS, NS = L::NS, LA = L::LA, SU = L::SU, WC = L::WC, AU = L::AU, WN = L::WN, LPS = L::LPS;
  static_assert((GEMM_K_PAD / 16) % NS == 0 && LA < NS && LA >= 1, "a run of k-steps is a whole number of trips round the ring");
  u32x4v *ring = (u32x4v *)lds_raw;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nblocks = Np >> 5, nz = Mp / ROWS;
  const int c_lo = blockIdx.y * groups_per_split * NS;
  const int nchunks = min(Kp >> 4, c_lo + groups_per_split * NS), last = nchunks - 1;
  const int plane = blockIdx.y;
  const int bx = ZFAST ? blockIdx.x / nz : blockIdx.x, bz = ZFAST ? blockIdx.x % nz : blockIdx.z;
  const int nbw = bx * WC * NBW, nb0 = nbw + (w % WC) * NBW, mrow0 = bz * ROWS, wrow = (w / WC) * 32 * MB;
  const int64_t a_step = w_kstep_stride(Np);
  // what this wavefront fetches: weight block nbw + w (past the end: the last one again, never stored) and the
  // runs of 64 units i WN + w of the activation chunk (unit u: k8 group u / ROWS of the k-step, batch row u % ROWS)
  const h16x8 *a_src = Wp + w_block_base(min(nbw + w, nblocks - 1), Kp) + (lane >> 5) * 32 + (lane & 31);
  const u32x4v *x_src[L::XLW];
#pragma unroll
  for (int i = 0; i < L::XLW; ++i) {
    int xi = (i * WN + w) * 64 + lane;
    x_src[i] = Xp + (int64_t)(xi / ROWS) * Mp + mrow0 + xi % ROWS;
  }
  auto fetch = [&](int st, int c) {
#pragma unroll
    for (int i = 0; i < L::XLW; ++i) load_to_lds(x_src[i] + (int64_t)(c * 2) * Mp, ring + st * SU + AU + (i * WN + w) * 64);
    load_to_lds(a_src + (int64_t)c * a_step, ring + st * SU + w * 64);
  };
  // what it reads: its two weight blocks, and the rows of its row half
  const u32x4v *a_lds = ring + (w % WC) * NBW * 64 + lane;
  const u32x4v *b_lds = ring + AU + (lane >> 5) * ROWS + wrow + (lane & 31);
  f32x16 acc[NBW][MB];
#pragma unroll
  for (int n = 0; n < NBW; ++n)
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[n][j][r] = 0.f;
#pragma unroll
  for (int j = 0; j < LA; ++j) fetch(j, min(c_lo + j, last));   // a run has at least NS k-steps
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS * (LA - 1)) : "memory");
  __syncthreads();
  for (int c0 = c_lo; c0 < nchunks; c0 += NS) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      fetch((s + LA) % NS, min(c0 + s + LA, last));   // past the end: the last k-step again, never read
      u32x4v a[NBW], b[MB];
#pragma unroll
      for (int n = 0; n < NBW; ++n) a[n] = a_lds[s * SU + n * 64];
#pragma unroll
      for (int j = 0; j < MB; ++j) b[j] = b_lds[s * SU + j * 32];
#pragma unroll
      for (int j = 0; j < MB; ++j)
#pragma unroll
        for (int n = 0; n < NBW; ++n) acc[n][j] = mfma_h16(__builtin_bit_cast(h16x8, a[n]), __builtin_bit_cast(h16x8, b[j]), acc[n][j]);
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(LPS * (LA - 1)) : "memory");
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the loads past the end have landed before the ring is reused
  __syncthreads();
  const int half = lane >> 5, col = lane & 31;
  if (EPI == EPI_PARTIAL) {   // 32 x 32 tiles transposed through LDS so that every store is a whole 128-byte row segment
    float *tile = (float *)lds_raw + (size_t)w * 32 * L::TILE_STRIDE;
#pragma unroll
    for (int n = 0; n < NBW; ++n) {
      float *P = (float *)out + ((int64_t)plane * Mp + mrow0 + wrow) * Np + (nb0 + n) * 32;
#pragma unroll
      for (int j = 0; j < MB; ++j) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int i = 0; i < 4; ++i) tile[col * L::TILE_STRIDE + 8 * g + 4 * half + i] = acc[n][j][4 * g + i] * W_UNSCALE;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (nb0 + n < nblocks) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            int r = q * 8 + (lane >> 3), n4 = (lane & 7) * 4;
            const float *t = tile + r * L::TILE_STRIDE + n4;
            f32x4 v = {t[0], t[1], t[2], t[3]};
            *(f32x4 *)(P + (int64_t)(j * 32 + r) * Np + n4) = v;
          }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      }
    }
  } else {  // EPI_SWIGLU, as in the kernels above
    uint32_t *O = (uint32_t *)out;
#pragma unroll
    for (int n = 0; n < NBW; ++n) {
      if (nb0 + n >= nblocks) break;
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        uint32_t pk[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v0 = silu_f(acc[n][j][4 * g] * W_UNSCALE) * (acc[n][j][4 * g + 1] * W_UNSCALE);
          float v1 = silu_f(acc[n][j][4 * g + 2] * W_UNSCALE) * (acc[n][j][4 * g + 3] * W_UNSCALE);
          pk[g] = (uint32_t)f32_to_h16_bits(v0) | ((uint32_t)f32_to_h16_bits(v1) << 16);
        }
        uint32_t give0 = half ? pk[0] : pk[2], give1 = half ? pk[1] : pk[3];
        uint32_t got0 = __shfl_xor(give0, 32, 64), got1 = __shfl_xor(give1, 32, 64);
        u32x4v o = half ? u32x4v{got0, pk[2], got1, pk[3]} : u32x4v{pk[0], got0, pk[1], got1};
        int m = mrow0 + wrow + j * 32 + col;
        *(u32x4v *)(O + (((int64_t)((nb0 + n) * 2 + half) * Mp + m) * 4)) = o;
      }
    }
  }
}

template <int EPI, bool ZFAST, int WC = 4>
static void gemm_ring_launch(void *out, const void *Xp, const void *Wp, int Mp, int Np, int Kp, hipStream_t st, int nsplit = 1) {
  using L = GemmRingT<WC>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)gemm_ring_kernel<EPI, ZFAST, WC>, hipFuncAttributeMaxDynamicSharedMemorySize, L::BYTES);
    attr_set = true;
  }
  int nblocks = Np / 32, per_wg = L::WC * L::NBW, strips = (nblocks + per_wg - 1) / per_wg, nz = Mp / L::ROWS;
  int groups = (Kp / 16) / L::NS, gps = (groups + nsplit - 1) / nsplit, ny = (groups + gps - 1) / gps;
  dim3 grid = ZFAST ? dim3(strips * nz, ny, 1) : dim3(strips, ny, nz);
  hipLaunchKernelGGL((gemm_ring_kernel<EPI, ZFAST, WC>), grid, dim3(L::T), L::BYTES, st, out, (const u32x4v *)Xp, (const h16x8 *)Wp, Mp, Np, Kp, gps);
}

// Launch shape.  Up to 128 batch rows the LDS-staged kernel runs: three or four weight blocks per workgroup, and a
// grid split over K that brings the launch to about one workgroup per compute unit (partials cost HBM writes, so
// no more than that); a GEMM whose epilogue needs the whole K (SwiGLU) is not split and takes the workgroup width
// (three to eight blocks) that needs the fewest rounds of the chip.  Batches that are a multiple of 256 rows take the
// LDS-ring kernel (256 x 256 tiles when those fill the chip, 256 x 128 tiles with a split over K otherwise).  Shapes
// that fit neither (K not padded, odd row counts) keep the plain register-streaming kernel: waves_k wavefronts of a
// workgroup share a block's k-steps and are summed in LDS.
// The largest split count <= nsplit that the 256 x 128-tile kernel realises exactly: it cuts K into runs of
// ceil(groups / nsplit) groups of eight k-steps, which may come to fewer runs than asked for.
int fast_gemm_even_split(int Kp, int nsplit) {
  int groups = Kp / 16 / 8;
  for (;;) {
    int gps = (groups + nsplit - 1) / nsplit, ny = (groups + gps - 1) / gps;
    if (ny == nsplit) return nsplit;
    nsplit = ny;
  }
}

void fast_gemm_pick(int Np, int Kp, int Mp, int full_k, GemmShape *g) {
  int nblocks = Np / 32, ksteps = Kp / 16, mb = Mp / 32 > 8 ? 8 : Mp / 32;
  int zblocks = Mp / (32 * mb);
  g->lds = 0; g->stages = 0;
  if (Kp % GEMM_K_PAD == 0 && Mp % 256 == 0 && (nblocks + 7) / 8 * (Mp / 256) >= 128) {   // 256 x 256 tiles fill the chip
    g->lds = 2; g->nbw = 2; g->waves_k = 1; g->waves_n = 4; g->stages = 8; g->nsplit = 1;
    // One tile per compute unit at a time, so a tile count just above a multiple of 256 leaves most of the chip idle in
    // the last round (320 tiles take two rounds).  Splitting K in two runs makes the units of work half as long and the
    // rounds fill up (320 tiles: 1.5 rounds' worth), at the price of a second plane of fp32 partials written and read
    // again -- which pays once K is long (measured at 4096 rows: N 5120, K 8192: 411 -> 340 us, K 25600: 1228 -> 1011 us,
    // for about 34 us of extra plane traffic; at K 4096 the plane costs more than the split saves).
    if (!full_k && Kp >= 6144) {
      const int tiles = (nblocks + 7) / 8 * (Mp / 256);
      if ((2 * tiles + 255) / 256 * 0.5 <= 0.8 * ((tiles + 255) / 256)) g->nsplit = 2;
    }
    return;
  }
  if (Kp % GEMM_K_PAD == 0 && Mp % 256 == 0) {
    // 256 x 128 tiles (two row halves x two column pairs of wavefronts), K split until the launch has about one
    // workgroup per compute unit; a split keeps at least four groups of eight k-steps
    int strips = (nblocks + 3) / 4 * (Mp / 256), groups = ksteps / 8;
    int ns = full_k ? 1 : (240 + strips / 2) / strips;
    if (ns > groups / 4) ns = groups / 4;
    if (ns > 12) ns = 12;
    if (ns < 1) ns = 1;
    g->lds = 3; g->nbw = 2; g->waves_k = 1; g->waves_n = 4; g->stages = 8; g->nsplit = fast_gemm_even_split(Kp, ns);
    return;
  }
  if (Kp % (16 * GEMM_KC_SMALL) == 0 && (Mp <= 128 || Mp % 256 == 0)) {
    const bool wide = Mp > 128;   // 256 batch rows per workgroup, Mp/256 workgroups per weight strip
    int total_chunks = ksteps / (wide ? GEMM_KC_WIDE : GEMM_KC_SMALL);
    g->lds = 1; g->nbw = 1; g->waves_k = 1;
    if (full_k && !wide) {
      // No split over K (the SwiGLU epilogue needs whole sums), one workgroup per compute unit at a time: the launch takes
      // rounds x width, rounds = ceil(workgroups / 256).  The width with the smallest product wins, the wider one on a
      // tie (fewer rounds, fewer re-reads of the activations).  Measured at 64 rows: 608 blocks (4B) width 3, 203
      // workgroups, 21 us (width 4: 23); 768 blocks (8B) width 3, 256 workgroups, 34 us; 1600 blocks (32B) width 7,
      // 229 workgroups, 81 us -- width 3 (534 workgroups, three rounds) took 109 us there, width 4 (two rounds) 90.
      int best = 3, best_cost = 1 << 30;
      const int wn_max = Mp <= 64 ? 8 : 4;   // 128 rows: more than four wavefronts would not fit their registers
      for (int wn = 3; wn <= wn_max; ++wn) {
        int wgs = (nblocks + wn - 1) / wn, cost = (wgs + 255) / 256 * wn;
        if (cost <= best_cost) { best = wn; best_cost = cost; }
      }
      g->waves_n = best; g->stages = best == 3 && Mp != 64 ? 3 : 2; g->nsplit = 1;   // 64 rows: see gemm_lds_min_wgs
      return;
    }
    g->stages = 2;   // deeper register pipelines measured no faster once the wait counts are exact
    // workgroups of a launch with wn weight blocks per workgroup once K is split to about one workgroup per compute unit
    auto split_for = [&](int wn, int *wgs) {
      int strips = (nblocks + wn - 1) / wn * (wide ? Mp / 256 : 1);
      int ns = full_k ? 1 : (240 + strips / 2) / strips;
      if (ns > total_chunks / 2) ns = total_chunks / 2;
      if (ns > 10) ns = 10;
      if (ns < 1) ns = 1;
      int cps = (total_chunks + ns - 1) / ns;
      ns = (total_chunks + cps - 1) / cps;
      *wgs = strips * ns;
      return ns;
    };
    g->waves_n = wide || nblocks % 4 == 0 || nblocks > 96 ? 4 : 3;
    int wgs = 0;
    g->nsplit = split_for(g->waves_n, &wgs);
    // A narrow output with four blocks per workgroup can leave a third of the chip without a workgroup however K is split
    // (2560 columns: 20 strips x 8 runs = 160); three blocks give 27 strips and 216 workgroups (measured at 64 rows on the
    // 4B shape, output and down projection together: decode step 3.764 -> 3.741 ms; where the gain in workgroups is small --
    // 6144 columns, 240 -> 256 -- nothing moves).  Never past one workgroup per compute unit.
    if (!full_k && !wide && Mp <= 64 && g->waves_n == 4) {
      int wgs3 = 0, ns3 = split_for(3, &wgs3);
      if (wgs3 <= 256 && wgs3 * 20 >= wgs * 23) { g->waves_n = 3; g->nsplit = ns3; }
    }
    return;
  }
  g->nbw = 1;
  g->waves_n = 1;
  int tiles = nblocks / g->nbw * zblocks;
  int wk = 2;
  while (wk > 1 && (ksteps / wk < 8 || (size_t)(wk - 1) * g->nbw * mb * 4096 > 65536)) --wk;
  if (full_k && tiles >= 256) wk = tiles >= 512 ? 1 : 2;
  int ns = full_k ? 1 : (1536 + tiles * wk / 2) / (tiles * wk);
  if (ns > 8) ns = 8;
  while (ns > 1 && ksteps / (ns * wk) < 8) --ns;
  if (ns < 1) ns = 1;
  g->nsplit = ns;
  g->waves_k = wk;
}

template <int MB, int WN, int NSTAGE, int EPI>
static void gemm_lds_launch(void *out, const void *Xp, const void *Wp, int Mp, int Np, int Kp, int nsplit, hipStream_t st) {
  using L = GemmLds<MB, WN>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)gemm_lds_kernel<MB, WN, NSTAGE, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, L::BYTES);
    attr_set = true;
  }
  int nblocks = Np / 32, total_chunks = (Kp / 16) / L::KC, cps = (total_chunks + nsplit - 1) / nsplit;
  dim3 grid((nblocks + WN - 1) / WN, nsplit, Mp / (32 * MB)), block(64 * WN);
  hipLaunchKernelGGL((gemm_lds_kernel<MB, WN, NSTAGE, EPI>), grid, block, L::BYTES, st, out, (const u32x4v *)Xp, (const h16x8 *)Wp, Mp,
                     Np, Kp, cps);
}

// The instantiated forms: three blocks with the three-chunk weight pipeline (two chunks at 64 rows), four blocks with two
// chunks, and for the full-K projection at up to 64 rows five to eight blocks with two chunks (see fast_gemm_pick).
template <int MB, int EPI>
static void gemm_lds_dispatch_rows(void *out, const void *Xp, const void *Wp, int Mp, int Np, int Kp, GemmShape g, hipStream_t st) {
  if (g.waves_n == 3 && g.stages == 2) { gemm_lds_launch<MB, 3, 2, EPI>(out, Xp, Wp, Mp, Np, Kp, g.nsplit, st); return; }
  if (g.waves_n == 3) { gemm_lds_launch<MB, 3, 3, EPI>(out, Xp, Wp, Mp, Np, Kp, g.nsplit, st); return; }
  if constexpr (EPI == EPI_SWIGLU && MB <= 2) {
    switch (g.waves_n) {
      case 5: gemm_lds_launch<MB, 5, 2, EPI>(out, Xp, Wp, Mp, Np, Kp, g.nsplit, st); return;
      case 6: gemm_lds_launch<MB, 6, 2, EPI>(out, Xp, Wp, Mp, Np, Kp, g.nsplit, st); return;
      case 7: gemm_lds_launch<MB, 7, 2, EPI>(out, Xp, Wp, Mp, Np, Kp, g.nsplit, st); return;
      case 8: gemm_lds_launch<MB, 8, 2, EPI>(out, Xp, Wp, Mp, Np, Kp, g.nsplit, st); return;
      default: break;
    }
  }
  gemm_lds_launch<MB, 4, 2, EPI>(out, Xp, Wp, Mp, Np, Kp, g.nsplit, st);
}

template <int EPI>
static void gemm_lds_dispatch(void *out, const void *Xp, const void *Wp, int Mp, int Np, int Kp, GemmShape g, hipStream_t st) {
  int mb = Mp / 32;   // 1, 2, 4 or a multiple of 8
  if (mb >= 8) gemm_lds_launch<8, 4, 2, EPI>(out, Xp, Wp, Mp, Np, Kp, g.nsplit, st);
  else if (mb == 1) gemm_lds_dispatch_rows<1, EPI>(out, Xp, Wp, Mp, Np, Kp, g, st);
  else if (mb == 2) gemm_lds_dispatch_rows<2, EPI>(out, Xp, Wp, Mp, Np, Kp, g, st);
  else gemm_lds_dispatch_rows<4, EPI>(out, Xp, Wp, Mp, Np, Kp, g, st);
}

template <int EPI>
static void gemm_dispatch(void *out, const void *Xp, const void *Wp, int Mp, int Np, int Kp, GemmShape g, hipStream_t st) {
  if (g.lds == 2) {   // row blocks fastest once the weights are far larger than the last-level cache
    if ((size_t)Np * Kp * 2 >= ((size_t)256 << 20)) gemm_ring_launch<EPI, true>(out, Xp, Wp, Mp, Np, Kp, st, g.nsplit);
    else gemm_ring_launch<EPI, false>(out, Xp, Wp, Mp, Np, Kp, st, g.nsplit);
    return;
  }
  if (g.lds == 3) { gemm_ring_launch<EPI, false, 2>(out, Xp, Wp, Mp, Np, Kp, st, g.nsplit); return; }
  if (g.lds) { gemm_lds_dispatch<EPI>(out, Xp, Wp, Mp, Np, Kp, g, st); return; }
  int mbt = Mp / 32;
  int MB = mbt >= 8 ? 8 : mbt;
  int ksteps = Kp / 16, kps = (ksteps + g.nsplit - 1) / g.nsplit;
  int per_wg = g.nbw * g.waves_n, nblocks = Np / 32;
  dim3 grid((nblocks + per_wg - 1) / per_wg, g.nsplit, mbt / MB), block(64 * g.waves_n * g.waves_k);
  size_t lds = (size_t)(g.waves_k - 1) * g.waves_n * g.nbw * MB * 16 * 64 * sizeof(float);
  const h16x8 *X = (const h16x8 *)Xp, *W = (const h16x8 *)Wp;
#define GEMM_LAUNCH(MBV, NBWV) \
  hipLaunchKernelGGL((gemm_kernel<MBV, NBWV, EPI>), grid, block, lds, st, out, X, W, Mp, Np, Kp, kps, g.waves_n)
  if (g.nbw == 2) {
    switch (MB) {
      case 1: GEMM_LAUNCH(1, 2); break;
      case 2: GEMM_LAUNCH(2, 2); break;
      default: GEMM_LAUNCH(4, 2); break;
    }
  } else {
    switch (MB) {
      case 1: GEMM_LAUNCH(1, 1); break;
      case 2: GEMM_LAUNCH(2, 1); break;
      case 4: GEMM_LAUNCH(4, 1); break;
      default: GEMM_LAUNCH(8, 1); break;
    }
  }
#undef GEMM_LAUNCH
}

void fast_gemm(void *out, const void *Xp, const void *Wp, int Mp, int Np, int Kp, GemmShape g, GemmEpilogue epi,
               hipStream_t st) {
  if (epi == EPI_PARTIAL) gemm_dispatch<EPI_PARTIAL>(out, Xp, Wp, Mp, Np, Kp, g, st);
  else { g.nsplit = 1; gemm_dispatch<EPI_SWIGLU>(out, Xp, Wp, Mp, Np, Kp, g, st); }
}

// ---- lm_head ---------------------------------------------------------------------------------------------
// grid (ceil(Np/32 / 4), 1, Mp/(32*MB)); block 256.  The GEMM main loop over the full K (four weight blocks per
// workgroup), then every logit is folded into a running (max, sum-exp, best perturbed score, its index, its z) per
// batch row: per wavefront, then over the four wavefronts in wavefront order, one partial per workgroup.
constexpr int LM_WN = 4;
template <int MB> struct LmLds {   // epilogue of the 256-row kernel: accumulators of four wavefronts + their partial results
  static constexpr int DUMP_PER_WAVE = MB * 16 * 64 * 4;
  static constexpr int BYTES = LM_WN * DUMP_PER_WAVE + LM_WN * MB * 32 * (int)sizeof(SampleAcc);
};

// The vocabulary takes several rounds of workgroups (1187 for 151936 rows on 256 compute units), and a workgroup's
// sampler epilogue moves no weights.  With two workgroups resident per compute unit one's epilogue and first loads run
// under the other's weight stream: 64 rows 199 -> 146 us, 32 rows 158 -> 133 us, 128 rows (sampler) 306 -> 280 us.  That
// needs the kernel inside 256 registers per lane, which a two-chunk weight pipeline allows (three chunks in flight
// fit only at 32 rows; the 128-row forms spill a little, and the 128-row logits form, which has no long epilogue to
// hide, is faster alone on the unit with its three-chunk pipeline).
template <int MB, bool LOGITS> constexpr int lm_wgs_per_cu() { return MB <= 2 || (MB == 4 && !LOGITS) ? 2 : 1; }

template <int MB, int NSTAGE, bool LOGITS>
__global__ __launch_bounds__(256, (lm_wgs_per_cu<MB, LOGITS>())) void lmhead_kernel(const u32x4v *__restrict__ Xp, const h16x8 *__restrict__ Wp, int Mp,
                                                     int Np, int Kp, int V, float temperature, uint64_t seed,
                                                     DrawIds ids, const int32_t *target, float *target_z,
                                                     float *part, int n_wg, float *logits, int64_t ld) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  using L = GemmLds<MB, LM_WN>;
  int w = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int nblocks = Np >> 5, mrow0 = blockIdx.z * 32 * MB;
  const int nb_own = blockIdx.x * LM_WN + w, nb = min(nb_own, nblocks - 1);
  f32x16 acc[MB];
  gemm_lds_mainloop<MB, LM_WN, NSTAGE>(acc, lds_raw, Xp, Wp, Mp, Np, Kp, nb, 0, (Kp >> 4) / L::KC, mrow0);
  // One logit: temperature, running (max, sum-exp), perturbed-score argmax, the target's z.
  auto fold = [&](SampleAcc &sa, float a, uint32_t bits, int v, int m, int tgt) {
    if (v < V) {
      float z = a * W_UNSCALE / temperature;
      sample_acc_add(sa, z, z + gumbel_from_bits(bits), v);
      if (v == tgt) target_z[m] = z;
    }
  };
  auto fold_plain = [&](SampleAcc &sa, float a, int v, int m, int tgt) {
    if (v < V) {
      float z = a * W_UNSCALE / temperature;
      sample_acc_add(sa, z, z, v);
      if (v == tgt) target_z[m] = z;
    }
  };
  auto fold4 = [&](SampleAcc &sa, f32x4 a, int v0, int m, int tgt, uint32_t stream, uint32_t step) {
    if (target) {   // scoring: only the target's log-prob is wanted, so no noise is drawn (the token output is the plain argmax)
      fold_plain(sa, a[0], v0, m, tgt); fold_plain(sa, a[1], v0 + 1, m, tgt);
      fold_plain(sa, a[2], v0 + 2, m, tgt); fold_plain(sa, a[3], v0 + 3, m, tgt);
    } else {
      u32x4 r = draw4(seed, stream, step, (uint32_t)(v0 >> 2));
      fold(sa, a[0], r.x, v0, m, tgt); fold(sa, a[1], r.y, v0 + 1, m, tgt);
      fold(sa, a[2], r.z, v0 + 2, m, tgt); fold(sa, a[3], r.w, v0 + 3, m, tgt);
    }
  };
  auto write_partial = [&](const SampleAcc &sa, int m) {
    int64_t o = (int64_t)blockIdx.x * Mp + m, plane = (int64_t)n_wg * Mp;
    part[o] = sa.zmax;
    part[plane + o] = sa.zsum;
    part[2 * plane + o] = sa.best;
    part[3 * plane + o] = sa.zbest;
    part[4 * plane + o] = __int_as_float(sa.idx);
  };
  if constexpr (LOGITS) {
    if (nb_own < nblocks) {
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        int m = mrow0 + j * 32 + col;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          int v0 = nb * 32 + 8 * g + 4 * half;
          f32x4 o = {acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]};
          if (v0 < V) *(f32x4 *)(logits + (int64_t)m * ld + v0) = o * W_UNSCALE;
        }
      }
    }
  } else if constexpr (MB >= 8) {
    // Unrolling the sampler over eight row tiles is more code than the compiler will unroll, and a rolled loop over
    // the accumulator array would move it out of the registers for the whole kernel.  So the accumulators are parked
    // in LDS with static indices (each lane reads back only what it wrote) and the row tiles are folded in a loop.
    using LM = LmLds<MB>;
    __syncthreads();   // the main loop's buffers are free once every wavefront has left it
    f32x4 *dump = (f32x4 *)(lds_raw + w * LM::DUMP_PER_WAVE) + lane;
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) dump[(j * 4 + g) * 64] = f32x4{acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]};
    SampleAcc (*sh)[MB][32] = (SampleAcc (*)[MB][32])(lds_raw + LM_WN * LM::DUMP_PER_WAVE);   // [4][MB][32]
#pragma unroll 1
    for (int j = 0; j < MB; ++j) {
      SampleAcc sa = sample_acc_init();
      if (nb_own < nblocks) {
        int m = mrow0 + j * 32 + col, tgt = target ? target[m] : -1;
        const uint32_t stream = draw_stream(ids, m), step = target ? 0u : draw_step(ids, m);
#pragma unroll
        for (int g = 0; g < 4; ++g) fold4(sa, dump[(j * 4 + g) * 64], nb * 32 + 8 * g + 4 * half, m, tgt, stream, step);
      }
      SampleAcc o = sample_acc_shfl_xor(sa, 32);
      sample_acc_merge(sa, o);
      if (half == 0) sh[w][j][col] = sa;
    }
    __syncthreads();
    if (w == 0 && half == 0) {
#pragma unroll 1
      for (int j = 0; j < MB; ++j) {
        SampleAcc sa = sh[0][j][col];
        for (int ww = 1; ww < LM_WN; ++ww) sample_acc_merge(sa, sh[ww][j][col]);
        write_partial(sa, mrow0 + j * 32 + col);
      }
    }
  } else {
    SampleAcc sa[MB];
#pragma unroll
    for (int j = 0; j < MB; ++j) sa[j] = sample_acc_init();
    if (nb_own < nblocks) {
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        int m = mrow0 + j * 32 + col, tgt = target ? target[m] : -1;
        const uint32_t stream = draw_stream(ids, m), step = target ? 0u : draw_step(ids, m);
#pragma unroll
        for (int g = 0; g < 4; ++g)
          fold4(sa[j], f32x4{acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]}, nb * 32 + 8 * g + 4 * half, m, tgt,
                stream, step);
      }
    }
    // lanes l and l^32 hold the same batch row; then fold the four wavefronts in wavefront order
    SampleAcc (*sh)[MB][32] = (SampleAcc (*)[MB][32])lds_raw;   // [3][MB][32]; the main loop's buffers are free by now
#pragma unroll
    for (int j = 0; j < MB; ++j) { SampleAcc b = sample_acc_shfl_xor(sa[j], 32); sample_acc_merge(sa[j], b); }
    __syncthreads();   // every wavefront has left the main loop before its buffers are overwritten
    if (w > 0 && half == 0)
#pragma unroll
      for (int j = 0; j < MB; ++j) sh[w - 1][j][col] = sa[j];
    __syncthreads();
    if (w == 0 && half == 0) {
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        for (int ww = 0; ww < 3; ++ww) sample_acc_merge(sa[j], sh[ww][j][col]);
        write_partial(sa[j], mrow0 + j * 32 + col);
      }
    }
  }
}

// ---- lm_head on 256 x 256 tiles (batches of 256 rows and more: scoring passes, wide decode batches) -----------------
// A register-streaming main loop (four wavefronts, two weight blocks each, 256 rows, operands eight k-steps ahead),
// then the sampler of the kernel above over the 2 x 8 accumulator tiles of a wavefront: parked in LDS one weight block
// at a time (static indices, so the accumulators stay registers during the main loop) and folded in a rolled loop.
// grid: ceil(Np/256) column strips x Mp/256 row blocks, the row blocks of a strip neighbours in launch order (the
// vocabulary matrix is far larger than the caches); one partial per (row, strip).
struct LmWideLds {
  static constexpr int DUMP_PER_WAVE = 8 * 16 * 64 * 4;   // one weight block's eight accumulator tiles
  static constexpr int BYTES = LM_WN * DUMP_PER_WAVE + LM_WN * 8 * 32 * (int)sizeof(SampleAcc);
};

// SCORE (teacher-forced scoring, target set): only the log-sum-exp of the row and the target's z are wanted, so a
// lane takes the 16 logits of an accumulator tile at once -- their maximum, then 16 hardware exp2 of the differences
// -- instead of the sampler's per-logit running update (which costs more than the main loop at this tile size).
template <bool SCORE>
__global__ __launch_bounds__(256) void lmhead_wide_kernel(const u32x4v *__restrict__ Xp, const h16x8 *__restrict__ Wp, int Mp, int Np,
                                                          int Kp, int V, float temperature, uint64_t seed, DrawIds ids,
                                                          const int32_t *target, float *target_z, float *part, int n_wg) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  using L = GemmWide;
  constexpr int MB = L::MB, NBW = L::NBW, T = L::T, XU = L::CHUNK_UNITS, XL = L::XL, ROWS = L::ROWS, NSTAGE = L::NSTAGE;
  u32x4v *xs = (u32x4v *)lds_raw;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, tid = threadIdx.x, half = lane >> 5, col = lane & 31;
  const int nblocks = Np >> 5, nchunks = Kp >> 4, nz = Mp / ROWS;
  const int bx = blockIdx.x / nz, bz = blockIdx.x % nz;
  const int nb0 = (bx * L::WN + w) * NBW, mrow0 = bz * ROWS;
  const int64_t a_step = w_kstep_stride(Np);
  const h16x8 *a_ptr[NBW];
#pragma unroll
  for (int n = 0; n < NBW; ++n) a_ptr[n] = Wp + w_block_base(min(nb0 + n, nblocks - 1), Kp) + (lane >> 5) * 32 + (lane & 31);
  f32x16 acc[NBW][MB];
#pragma unroll
  for (int n = 0; n < NBW; ++n)
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[n][j][r] = 0.f;
  h16x8 a[NSTAGE][NBW];
  u32x4v xr[NSTAGE][XL];
  auto load_a = [&](int st, int c) {
#pragma unroll
    for (int n = 0; n < NBW; ++n) a[st][n] = __builtin_nontemporal_load(a_ptr[n] + (int64_t)c * a_step);
  };
  auto load_x = [&](int st, int c) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      int idx = i * T + tid;
      xr[st][i] = Xp[(int64_t)(c * 2 + idx / ROWS) * Mp + mrow0 + idx % ROWS];
    }
  };
  auto store_x = [&](int st, int buf) {
#pragma unroll
    for (int i = 0; i < XL; ++i) xs[buf * XU + i * T + tid] = xr[st][i];
  };
  auto compute = [&](int st, int buf) {
    const u32x4v *bp = xs + buf * XU + (lane >> 5) * ROWS + (lane & 31);
    u32x4v b[MB];
#pragma unroll
    for (int j = 0; j < MB; ++j) b[j] = bp[j * 32];
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int n = 0; n < NBW; ++n) acc[n][j] = mfma_h16(a[st][n], __builtin_bit_cast(h16x8, b[j]), acc[n][j]);
  };
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s) { load_x(s, s); load_a(s, s); }
  store_x(0, 0);
  __syncthreads();
  for (int c0 = 0; c0 < nchunks; c0 += NSTAGE) {
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s) {
      const int c = c0 + s, cn = min(c + NSTAGE - 1, nchunks - 1);
      load_x((s + NSTAGE - 1) % NSTAGE, cn);
      load_a((s + NSTAGE - 1) % NSTAGE, cn);
      compute(s, s & 1);
      store_x((s + 1) % NSTAGE, (s + 1) & 1);
      __syncthreads();
    }
  }
  // ---- sampler epilogue
  auto fold4 = [&](SampleAcc &sa, f32x4 av, int v0, int m, int tgt, uint32_t stream, uint32_t step) {
    u32x4 r = {0u, 0u, 0u, 0u};
    if (!target) r = draw4(seed, stream, step, (uint32_t)(v0 >> 2));
    const uint32_t bits[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int v = v0 + i;
      if (v < V) {
        float z = av[i] * W_UNSCALE / temperature;
        sample_acc_add(sa, z, target ? z : z + gumbel_from_bits(bits[i]), v);   // scoring draws no noise
        if (v == tgt) target_z[m] = z;
      }
    }
  };
  f32x4 *dump = (f32x4 *)(lds_raw + w * LmWideLds::DUMP_PER_WAVE) + lane;
  SampleAcc (*sh)[MB][32] = (SampleAcc (*)[MB][32])(lds_raw + LM_WN * LmWideLds::DUMP_PER_WAVE);   // [4][MB][32]
#pragma unroll
  for (int n = 0; n < NBW; ++n) {
    // (the loop above ended with a barrier: its buffers are free; between the two blocks each lane re-reads only its own dump)
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) dump[(j * 4 + g) * 64] = f32x4{acc[n][j][4 * g], acc[n][j][4 * g + 1], acc[n][j][4 * g + 2], acc[n][j][4 * g + 3]};
    const int nb = nb0 + n;
#pragma unroll 1
    for (int j = 0; j < MB; ++j) {
      SampleAcc sa = sample_acc_init();
      if (nb < nblocks) {
        int m = mrow0 + j * 32 + col, tgt = target ? target[m] : -1;
        if (SCORE) {
          const float c2 = W_UNSCALE / temperature * 1.44269504088896341f;   // logits in log2 units
          float z2[16], bm = -INFINITY;
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            f32x4 av = dump[(j * 4 + g) * 64];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              int v = nb * 32 + 8 * g + 4 * half + i;
              z2[4 * g + i] = v < V ? av[i] * c2 : -INFINITY;
              bm = fmaxf(bm, z2[4 * g + i]);
              if (v == tgt) target_z[m] = av[i] * W_UNSCALE / temperature;
            }
          }
          if (bm > -INFINITY) {
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(z2[i] - bm);
            sa.zmax = bm * 0.693147180559945309f;   // back to natural units: exp(z - zmax) = exp2(z2 - bm)
            sa.zsum = sum;
          }
        } else {
          const uint32_t stream = draw_stream(ids, m), step = target ? 0u : draw_step(ids, m);
#pragma unroll
          for (int g = 0; g < 4; ++g) fold4(sa, dump[(j * 4 + g) * 64], nb * 32 + 8 * g + 4 * half, m, tgt, stream, step);
        }
      }
      SampleAcc o = sample_acc_shfl_xor(sa, 32);
      sample_acc_merge(sa, o);
      if (half == 0) {
        if (n > 0) { SampleAcc prev = sh[w][j][col]; sample_acc_merge(prev, sa); sa = prev; }   // block order: lower indices first
        sh[w][j][col] = sa;
      }
    }
  }
  __syncthreads();
  if (w == 0 && half == 0) {
#pragma unroll 1
    for (int j = 0; j < MB; ++j) {
      SampleAcc sa = sh[0][j][col];
      for (int ww = 1; ww < LM_WN; ++ww) sample_acc_merge(sa, sh[ww][j][col]);
      int m = mrow0 + j * 32 + col;
      int64_t o = (int64_t)bx * Mp + m, plane = (int64_t)n_wg * Mp;
      part[o] = sa.zmax;
      part[plane + o] = sa.zsum;
      part[2 * plane + o] = sa.best;
      part[3 * plane + o] = sa.zbest;
      part[4 * plane + o] = __int_as_float(sa.idx);
    }
  }
}

static int lm_wide_wgs(int Np) { return (Np / 32 + 7) / 8; }
static bool lm_use_wide(int Mp, int Kp) { return Mp % 256 == 0 && Kp % GEMM_K_PAD == 0; }

// grid M rows, block 256: fold the per-workgroup partials of one row in workgroup order.
__global__ void sample_combine_kernel(int32_t *tok, float *lp, float *target_lp, const float *part, int n_wg, int Mp,
                                      const int32_t *row_active, const int32_t *target, const float *target_z) {
  __shared__ SampleAcc sh[4];
  int m = blockIdx.x;
  if (row_active && !row_active[m]) return;
  int64_t plane = (int64_t)n_wg * Mp;
  SampleAcc a = sample_acc_init();
  for (int g = threadIdx.x; g < n_wg; g += blockDim.x) {
    int64_t o = (int64_t)g * Mp + m;
    SampleAcc b = {part[o], part[plane + o], part[2 * plane + o], part[3 * plane + o], __float_as_int(part[4 * plane + o])};
    sample_acc_merge(a, b);
  }
  for (int o = 32; o > 0; o >>= 1) { SampleAcc b = sample_acc_shfl_xor(a, o); sample_acc_merge(a, b); }
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) sample_acc_merge(a, sh[w]);
    float lse = a.zmax + logf(a.zsum);
    tok[m] = a.idx;
    lp[m] = a.zbest - lse;
    if (target_lp) target_lp[m] = (target && target[m] >= 0) ? target_z[m] - lse : 0.f;
  }
}

static int lm_wgs(int Np) { return (Np / 32 + LM_WN - 1) / LM_WN; }
size_t fast_lmhead_partial_floats(int Np, int Mp) { return (size_t)5 * lm_wgs(Np) * Mp + Mp; }

template <int MB, int NSTAGE, bool LOGITS>
static void lmhead_launch(const void *Xp, const void *Wp, int Mp, int Np, int Kp, int V, float temperature, uint64_t seed,
                          DrawIds ids, const int32_t *target, float *target_z, float *part, float *logits, int64_t ld,
                          hipStream_t st) {
  using L = GemmLds<MB, LM_WN>;
  constexpr int SH = (MB >= 8 && !LOGITS) ? LmLds<MB>::BYTES : 3 * MB * 32 * (int)sizeof(SampleAcc);
  constexpr int BYTES = L::X_BYTES > SH ? L::X_BYTES : SH;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)lmhead_kernel<MB, NSTAGE, LOGITS>, hipFuncAttributeMaxDynamicSharedMemorySize, BYTES);
    attr_set = true;
  }
  int n_wg = lm_wgs(Np);
  dim3 grid(n_wg, 1, Mp / (32 * MB)), block(256);
  hipLaunchKernelGGL((lmhead_kernel<MB, NSTAGE, LOGITS>), grid, block, BYTES, st, (const u32x4v *)Xp, (const h16x8 *)Wp, Mp, Np, Kp, V,
                     temperature, seed, ids, target, target_z, part, n_wg, logits, ld);
}

template <bool LOGITS>
static void lmhead_dispatch(const void *Xp, const void *Wp, int Mp, int Np, int Kp, int V, float temperature, uint64_t seed,
                            DrawIds ids, const int32_t *target, float *target_z, float *part, float *logits,
                            int64_t ld, hipStream_t st) {
  int mbt = Mp / 32;
#define LM_ARGS Xp, Wp, Mp, Np, Kp, V, temperature, seed, ids, target, target_z, part, logits, ld, st
  if (mbt >= 8) lmhead_launch<8, 2, LOGITS>(LM_ARGS);
  else if (mbt == 4) lmhead_launch<4, LOGITS ? 3 : 2, LOGITS>(LM_ARGS);
  else if (mbt == 2) lmhead_launch<2, 2, LOGITS>(LM_ARGS);
  else lmhead_launch<1, 3, LOGITS>(LM_ARGS);
#undef LM_ARGS
}

void fast_lmhead_sample(int32_t *tok, float *lp, float *target_lp, const void *Xp, const void *Wp, int Mp, int M, int V,
                        int Np, int Kp, float temperature, uint64_t seed, DrawIds ids, const int32_t *row_active,
                        const int32_t *target, float *partials, hipStream_t st) {
  const bool wide = lm_use_wide(Mp, Kp);
  int n_wg = wide ? lm_wide_wgs(Np) : lm_wgs(Np);
  float *target_z = partials + (size_t)5 * lm_wgs(Np) * Mp;   // behind the partials of either form
  if (wide) {
    static bool attr_set = false;
    constexpr int BYTES = LmWideLds::BYTES > GemmWide::BYTES ? LmWideLds::BYTES : GemmWide::BYTES;
    if (!attr_set) {
      (void)hipFuncSetAttribute((const void *)lmhead_wide_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, BYTES);
      (void)hipFuncSetAttribute((const void *)lmhead_wide_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, BYTES);
      attr_set = true;
    }
    if (target)
      hipLaunchKernelGGL(lmhead_wide_kernel<true>, dim3(n_wg * (Mp / 256)), dim3(256), BYTES, st, (const u32x4v *)Xp, (const h16x8 *)Wp, Mp,
                         Np, Kp, V, temperature, seed, ids, target, target_z, partials, n_wg);
    else
      hipLaunchKernelGGL(lmhead_wide_kernel<false>, dim3(n_wg * (Mp / 256)), dim3(256), BYTES, st, (const u32x4v *)Xp, (const h16x8 *)Wp, Mp,
                         Np, Kp, V, temperature, seed, ids, target, target_z, partials, n_wg);
  } else {
    lmhead_dispatch<false>(Xp, Wp, Mp, Np, Kp, V, temperature, seed, ids, target, target_z, partials, nullptr, 0, st);
  }
  hipLaunchKernelGGL(sample_combine_kernel, dim3(M), dim3(256), 0, st, tok, lp, target_lp, partials, n_wg, Mp, row_active,
                     target, target_z);
}

void fast_sample_combine(int32_t *tok, float *lp, const float *part, int n_parts, int M, int Mp, const int32_t *row_active, hipStream_t st) {
  hipLaunchKernelGGL(sample_combine_kernel, dim3(M), dim3(256), 0, st, tok, lp, (float *)nullptr, part, n_parts, Mp, row_active,
                     (const int32_t *)nullptr, (const float *)nullptr);
}

void fast_lmhead_logits(float *logits, int64_t ld, const void *Xp, const void *Wp, int Mp, int Np, int Kp, int V,
                        hipStream_t st) {
  lmhead_dispatch<true>(Xp, Wp, Mp, Np, Kp, V, 1.0f, 0, DrawIds{nullptr, nullptr, nullptr}, nullptr, nullptr, nullptr, logits, ld, st);
}

}  // namespace echo
