// A C-ABI client without Python: allocates the arena with hipMalloc, installs a random bf16 snapshot of a dense decoder
// and runs one rollout through include/echo.h.  It exists to show the boundary in use from plain C/C++ and to give
// profilers a small host process to attach to (rocprofv3 counter collection on this program:
//   rocprofv3 --pmc FETCH_SIZE -- paper_2602_02192_amd/echo_client 4b 64 512 64).
// usage: echo_client <tiny|4b|8b|32b>[:LAYERS] <sequences (multiple of 8)> <prompt_len> <max_new> [score]
//   (":LAYERS" keeps a model's width and cuts its depth; "score" adds a teacher-forced echo_logprobs pass over every
//   prompt + generated string, i.e. the 4096-row GEMM and causal-attention kernels)
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/echo.h"

static uint16_t bf16_of(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// counter-hash normal variates: weights only need the right scale here (matrices N(0, 0.02^2), gains 1)
static inline uint32_t mix(uint64_t x) {
  x ^= x >> 33; x *= 0xff51afd7ed558ccdull; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ull; x ^= x >> 33;
  return (uint32_t)x;
}
static inline float approx_normal(uint64_t i) {   // sum of four uniforms, variance 1
  float s = 0.f;
  for (int k = 0; k < 4; ++k) s += (float)(mix(i * 4 + k) >> 8) * (1.0f / 16777216.0f);
  return (s - 2.0f) * 1.7320508f;
}

int main(int argc, char **argv) {
  const char *model = argc > 1 ? argv[1] : "tiny";
  int N = argc > 2 ? atoi(argv[2]) : 8, plen = argc > 3 ? atoi(argv[3]) : 16, max_new = argc > 4 ? atoi(argv[4]) : 16;
  echo_model_desc d;
  memset(&d, 0, sizeof d);
  const char *colon = strchr(model, ':');
  const size_t name_len = colon ? (size_t)(colon - model) : strlen(model);
  auto is = [&](const char *n) { return strlen(n) == name_len && !strncmp(model, n, name_len); };
  if (is("4b")) { d.n_layers = 36; d.hidden = 2560; d.n_q_heads = 32; d.n_kv_heads = 8; d.head_dim = 128; d.ffn = 9728; d.vocab = 151936; }
  else if (is("8b")) { d.n_layers = 36; d.hidden = 4096; d.n_q_heads = 32; d.n_kv_heads = 8; d.head_dim = 128; d.ffn = 12288; d.vocab = 151936; }
  else if (is("32b")) { d.n_layers = 64; d.hidden = 5120; d.n_q_heads = 64; d.n_kv_heads = 8; d.head_dim = 128; d.ffn = 25600; d.vocab = 151936; }
  else if (is("tiny")) { d.n_layers = 2; d.hidden = 256; d.n_q_heads = 4; d.n_kv_heads = 2; d.head_dim = 64; d.ffn = 704; d.vocab = 1024; }
  else { fprintf(stderr, "unknown model %s\n", model); return 2; }
  if (colon) d.n_layers = atoi(colon + 1);
  if (d.n_layers < 1) { fprintf(stderr, "bad layer count\n"); return 2; }
  const bool score = argc > 5 && !strcmp(argv[5], "score");
  d.rms_eps = 1e-6f; d.rope_base = 1e4f; d.dtype = ECHO_BF16; d.max_seqs = N; d.max_ctx = plen + max_new; d.n_weight_slots = 1;
  const int G = 8, P = N / G;
  if (P < 1 || N % G || plen < 1 || max_new < 1) { fprintf(stderr, "sequences must be a positive multiple of %d\n", G); return 2; }
  size_t arena_bytes = echo_arena_bytes(&d), blob_bytes = echo_blob_bytes(&d);
  if (!arena_bytes) { fprintf(stderr, "bad shape\n"); return 2; }
  void *arena = nullptr;
  if (hipMalloc(&arena, arena_bytes) != hipSuccess) { fprintf(stderr, "hipMalloc of %zu bytes failed\n", arena_bytes); return 1; }
  // blob order: embed; per layer attn_norm, wq|wk|wv, wo, ffn_norm, w_gate, w_up, w_down; final_norm; lm_head
  std::vector<uint16_t> blob(blob_bytes / 2);
  {
    const int64_t H = d.hidden, hd = d.head_dim, Q = (int64_t)d.n_q_heads * hd, KV = (int64_t)d.n_kv_heads * hd, F = d.ffn, V = d.vocab;
    const uint16_t one = bf16_of(1.0f);
    int64_t off = 0;
    auto matrix = [&](int64_t n) {
#pragma omp parallel for
      for (int64_t i = 0; i < n; ++i) blob[off + i] = bf16_of(0.02f * approx_normal((uint64_t)(off + i)));
      off += n;
    };
    auto gain = [&](int64_t n) { for (int64_t i = 0; i < n; ++i) blob[off + i] = one; off += n; };
    matrix(V * H);
    for (int l = 0; l < d.n_layers; ++l) { gain(H); matrix((Q + 2 * KV) * H); matrix(H * Q); gain(H); matrix(2 * F * H); matrix(H * F); }
    gain(H);
    matrix(V * H);
    if ((size_t)off * 2 != blob_bytes) { fprintf(stderr, "blob layout mismatch\n"); return 1; }
  }
  // a plain device-to-device copy of known size (256 MiB when the arena allows): the yardstick for traffic counters
  {
    size_t cal = (size_t)256 << 20;
    if (arena_bytes >= 2 * cal && hipMemcpy((char *)arena + cal, arena, cal, hipMemcpyDeviceToDevice) != hipSuccess) return 1;
  }
  echo_ctx *ctx = nullptr;
  int rc = echo_init(&d, 0, arena, arena_bytes, nullptr, nullptr, &ctx);
  if (rc) { fprintf(stderr, "echo_init: %s\n", echo_last_error(nullptr)); return 1; }
  if ((rc = echo_load_policy(ctx, 0, blob.data(), blob_bytes))) { fprintf(stderr, "echo_load_policy: %s\n", echo_last_error(ctx)); return 1; }
  std::vector<int32_t> prompts((size_t)P * plen), lens(P, plen), toks((size_t)N * max_new), out_lens(N);
  std::vector<float> lps((size_t)N * max_new);
  for (size_t i = 0; i < prompts.size(); ++i) prompts[i] = (int32_t)(mix(0x9e3779b97f4a7c15ull + i) % (uint32_t)d.vocab);
  echo_rollout_opts o;
  memset(&o, 0, sizeof o);
  o.eos_id = -1; o.top_p = 1.0f;
  o.no_graph = getenv("ECHO_CLIENT_NO_GRAPH") ? 1 : 0;
  auto t0 = std::chrono::steady_clock::now();
  rc = echo_rollout(ctx, prompts.data(), plen, lens.data(), P, G, max_new, 1.0f, 2, &o, toks.data(), lps.data(), out_lens.data(), nullptr);
  double s = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  if (rc) { fprintf(stderr, "echo_rollout: %s\n", echo_last_error(ctx)); return 1; }
  long total = 0;
  double lp = 0;
  for (int n = 0; n < N; ++n) { total += out_lens[n]; for (int t = 0; t < out_lens[n]; ++t) lp += lps[(size_t)n * max_new + t]; }
  printf("%s: %d sequences, prompt %d, %ld tokens generated in %.3f s (%.0f tokens/s), mean log-prob %.3f\n", model, N, plen, total, s,
         total / s, lp / total);
  if (score) {   // every string (prompt + generated tokens) through echo_logprobs
    const int stride = plen + max_new;
    std::vector<int32_t> full((size_t)N * stride), flen(N);
    std::vector<float> slp((size_t)N * stride);
    long rows = 0;
    for (int n = 0; n < N; ++n) {
      memcpy(&full[(size_t)n * stride], &prompts[(size_t)(n / G) * plen], (size_t)plen * 4);
      for (int t = 0; t < out_lens[n]; ++t) full[(size_t)n * stride + plen + t] = toks[(size_t)n * max_new + t];
      flen[n] = plen + out_lens[n];
      rows += flen[n] - 1;
    }
    t0 = std::chrono::steady_clock::now();
    rc = echo_logprobs(ctx, full.data(), stride, flen.data(), N, 1.0f, slp.data());
    s = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    if (rc) { fprintf(stderr, "echo_logprobs: %s\n", echo_last_error(ctx)); return 1; }
    const double H = d.hidden, Q = (double)d.n_q_heads * d.head_dim, KV = (double)d.n_kv_heads * d.head_dim;
    const double per_layer = H * (Q + 2 * KV) + Q * H + 3.0 * H * d.ffn, flop = 2.0 * rows * (d.n_layers * per_layer + (double)d.vocab * H);
    double dev = 0;
    for (int n = 0; n < N; ++n)
      for (int t = 0; t < out_lens[n]; ++t) {
        double e = slp[(size_t)n * stride + plen + t] - lps[(size_t)n * max_new + t];
        dev = e < 0 ? (-e > dev ? -e : dev) : (e > dev ? e : dev);
      }
    printf("scoring: %ld rows in %.3f s, %.1f TFLOP/s in the GEMMs (%.1f %% of 2.5 PFLOP/s); max |scored - sampled log-prob| %.4f\n", rows, s,
           flop / s / 1e12, 100.0 * flop / s / 2.5e15, dev);
  }
  echo_destroy(ctx);
  (void)hipFree(arena);
  return 0;
}
