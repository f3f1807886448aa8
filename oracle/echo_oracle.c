/*
 * CPU oracle for GRPO rollout generation -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, definition-level implementation of what a rollout worker
 * computes: for a prompt x it draws y ~ pi_v(. | x) token by token from the
 * policy's autoregressive distribution (ECHO-2, Sec. 4.1 "Versioned Execution and
 * Bounded Staleness";
 * Algorithm 1, rollout-plane loop) and records, for every sampled token, the
 * probability the sampler assigned to it (the denominator pi_sampler of the
 * truncated importance ratio, App. "GRPO-Style Policy Gradient Objective"),
 * tagged with the snapshot version in use (Sec. 4.1: immutable snapshots;
 * Sec. 4.2: a worker switches version once a snapshot is fully installed).
 *
 * The paper does not define the policy network; the decoder evaluated here is
 * the dense pre-norm transformer the workloads name (RMSNorm, grouped-query
 * causal attention with rotary embeddings, SwiGLU feed-forward, no biases).
 *
 * Nothing here is shared with the GPU library; only tests, the smoke check and
 * the benchmark's CPU-baseline leg may call it.  There is no blocking, no
 * fusion and no reordering: every output element is one sequential sum in
 * index order.  OpenMP only distributes independent output elements.
 *
 * Built twice from this file: ORC_REAL=double (the parity reference) and
 * ORC_REAL=float (the all-fp32 variant).  Decisions that floating point takes
 * about an integer (the sampled token) are taken in fp32 in both builds.
 *
 * Pins (tests/test_oracle_*.py): incremental decode == full recompute, softmax
 * rows sum to 1, RoPE(pos 0) = identity and relative-position property,
 * single-key attention returns V, closed-form 1-layer examples (one of them
 * for the per-head q/k norm: before the rotation, each with its own gains), Philox
 * known-answer vectors, Gumbel-max frequencies vs softmax (chi-square), silu
 * closed forms, batch/seed independence.  No function is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef ORC_REAL
#define ORC_REAL double
#endif
typedef ORC_REAL real;

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rms_eps, rope_base;
  int32_t qk_norm, tie_embeddings;
} orc_desc;

typedef struct {
  const float *attn_norm, *wq, *wk, *wv, *q_norm, *k_norm, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
} orc_layer;

typedef struct {
  orc_desc d;
  const float *embed, *final_norm, *lm_head;
  orc_layer *layers;
} orc_model;

int orc_real_bytes(void) { return (int)sizeof(real); }

/* Progress notes of the long calls (a line every 32 tokens of a string), appended to a file when one is set:
 * a caller that is watched for signs of life can show that a minutes-long call is moving.  No arithmetic here. */
static char progress_path[1024];
void orc_set_progress_file(const char *path) {
  progress_path[0] = 0;
  if (path && strlen(path) < sizeof progress_path) strcpy(progress_path, path);
}
static void progress_note(const char *what, int seq, int done, int total) {
  if (!progress_path[0] || (done & 31) != 0) return;
  FILE *f = fopen(progress_path, "a");
  if (!f) return;
  fprintf(f, "[oracle] %s: sequence %d, token %d of %d\n", what, seq, done, total);
  fclose(f);
}

void orc_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int orc_get_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- weight blob: embed; per layer attn_norm,wq,wk,wv,(q_norm,k_norm),wo,ffn_norm,
 *      w_gate,w_up,w_down; final_norm; lm_head (absent when tied).  Row-major [out,in]. */
int64_t orc_blob_numel(const orc_desc *d) {
  int64_t h = d->hidden, hd = d->head_dim, q = (int64_t)d->n_q_heads * hd, kv = (int64_t)d->n_kv_heads * hd;
  int64_t per = h + q * h + 2 * kv * h + (d->qk_norm ? 2 * hd : 0) + h * q + h + 3 * (int64_t)d->ffn * h;
  return (int64_t)d->vocab * h + d->n_layers * per + h + (d->tie_embeddings ? 0 : (int64_t)d->vocab * h);
}

static orc_model *model_bind(const orc_desc *d, const float *blob) {
  orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
  m->d = *d;
  m->layers = (orc_layer *)calloc((size_t)d->n_layers, sizeof(orc_layer));
  int64_t h = d->hidden, hd = d->head_dim, q = (int64_t)d->n_q_heads * hd, kv = (int64_t)d->n_kv_heads * hd;
  const float *p = blob;
  m->embed = p; p += (int64_t)d->vocab * h;
  for (int l = 0; l < d->n_layers; ++l) {
    orc_layer *L = &m->layers[l];
    L->attn_norm = p; p += h;
    L->wq = p; p += q * h;
    L->wk = p; p += kv * h;
    L->wv = p; p += kv * h;
    if (d->qk_norm) { L->q_norm = p; p += hd; L->k_norm = p; p += hd; }
    L->wo = p; p += h * q;
    L->ffn_norm = p; p += h;
    L->w_gate = p; p += (int64_t)d->ffn * h;
    L->w_up = p; p += (int64_t)d->ffn * h;
    L->w_down = p; p += h * (int64_t)d->ffn;
  }
  m->final_norm = p; p += h;
  m->lm_head = d->tie_embeddings ? m->embed : p;
  return m;
}

static void model_free(orc_model *m) { if (m) { free(m->layers); free(m); } }

/* ---- Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter-based generator. */
void orc_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Raw 32-bit draw for vocabulary entry i of sequence n at generation step s:
 * word (i mod 4) of Philox(counter = (i div 4, s, n, 0), key = seed). */
uint32_t orc_draw_bits(uint64_t seed, uint32_t n, uint32_t s, uint32_t i) {
  uint32_t ctr[4] = {i >> 2, s, n, 0u}, key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)}, out[4];
  orc_philox4x32(ctr, key, out);
  return out[i & 3u];
}

/* 23 random bits -> u = (2k+1) 2^-24 in (0,1), exactly representable in fp32. */
float orc_uniform(uint32_t bits) { return (float)(2u * (bits >> 9) + 1u) * 0x1p-24f; }

/* Standard Gumbel variate g = -log(-log u), evaluated in fp32. */
float orc_gumbel(float u) { return -logf(-logf(u)); }

/* ---- primitives ---- */

/* RMSNorm: y_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i */
void orc_rmsnorm(real *y, const real *x, const float *g, int n, float eps) {
  real ss = 0;
  for (int i = 0; i < n; ++i) ss += x[i] * x[i];
  real inv = (real)1 / (real)sqrt((double)(ss / (real)n + (real)eps));
  for (int i = 0; i < n; ++i) y[i] = x[i] * inv * (real)g[i];
}

/* Rotary embedding at position pos on one head vector of length hd: the pair
 * (x_i, x_{i+hd/2}) is rotated by the angle pos * base^(-2i/hd). */
void orc_rope(real *x, int hd, int pos, float base) {
  int half = hd / 2;
  for (int i = 0; i < half; ++i) {
    double theta = pow((double)base, -2.0 * (double)i / (double)hd);
    double ang = (double)pos * theta;
    real c = (real)cos(ang), s = (real)sin(ang);
    real a = x[i], b = x[i + half];
    x[i] = a * c - b * s;
    x[i + half] = a * s + b * c;
  }
}

real orc_silu(real x) { return x / ((real)1 + (real)exp((double)-x)); }

/* y = W x, W row-major [n_out, n_in] (fp32 storage), one sequential sum per output. */
static void matvec(real *y, const float *W, const real *x, int n_out, int n_in) {
#pragma omp parallel for schedule(static)
  for (int o = 0; o < n_out; ++o) {
    const float *w = W + (int64_t)o * n_in;
    real acc = 0;
    for (int k = 0; k < n_in; ++k) acc += (real)w[k] * x[k];
    y[o] = acc;
  }
}

/* Softmax-weighted sum for ONE query head vector q[hd] over keys/values
 * 0..n_keys-1: s_t = q.k_t / sqrt(hd); w = softmax(s); o = sum_t w_t v_t.
 * Key/value t for this head starts at k + t*stride (resp. v + t*stride). */
void orc_attend(real *o, const real *q, const real *k, const real *v, int n_keys, int hd, int64_t stride, real *scratch) {
  real scale = (real)1 / (real)sqrt((double)hd);
  real mx = 0;
  for (int t = 0; t < n_keys; ++t) {
    real s = 0;
    for (int i = 0; i < hd; ++i) s += q[i] * k[t * stride + i];
    s *= scale;
    scratch[t] = s;
    if (t == 0 || s > mx) mx = s;
  }
  real den = 0;
  for (int t = 0; t < n_keys; ++t) { scratch[t] = (real)exp((double)(scratch[t] - mx)); den += scratch[t]; }
  for (int i = 0; i < hd; ++i) o[i] = 0;
  for (int t = 0; t < n_keys; ++t) {
    real w = scratch[t] / den;
    for (int i = 0; i < hd; ++i) o[i] += w * v[t * stride + i];
  }
}

/* log softmax(z)[j] for all j, z = logits / temperature. */
void orc_log_softmax(real *out, const real *logits, int n, float temperature) {
  real mx = logits[0] / (real)temperature;
  for (int i = 1; i < n; ++i) { real z = logits[i] / (real)temperature; if (z > mx) mx = z; }
  real den = 0;
  for (int i = 0; i < n; ++i) den += (real)exp((double)(logits[i] / (real)temperature - mx));
  real lse = mx + (real)log((double)den);
  for (int i = 0; i < n; ++i) out[i] = logits[i] / (real)temperature - lse;
}

/* ---- incremental (KV-cached) decoder state for one sequence ---- */
typedef struct {
  int max_ctx, len;
  real *k, *v; /* [L][max_ctx][Hkv*hd] */
  real *h, *a, *q, *kv_k, *kv_v, *att, *o, *b, *gate, *up, *dn, *sc;
} orc_seq;

static orc_seq *seq_new(const orc_desc *d, int max_ctx) {
  orc_seq *s = (orc_seq *)calloc(1, sizeof(orc_seq));
  int64_t kvw = (int64_t)d->n_kv_heads * d->head_dim, qw = (int64_t)d->n_q_heads * d->head_dim;
  s->max_ctx = max_ctx;
  s->k = (real *)calloc((size_t)(d->n_layers * (int64_t)max_ctx * kvw), sizeof(real));
  s->v = (real *)calloc((size_t)(d->n_layers * (int64_t)max_ctx * kvw), sizeof(real));
  s->h = (real *)calloc((size_t)d->hidden, sizeof(real));
  s->a = (real *)calloc((size_t)d->hidden, sizeof(real));
  s->b = (real *)calloc((size_t)d->hidden, sizeof(real));
  s->o = (real *)calloc((size_t)d->hidden, sizeof(real));
  s->dn = (real *)calloc((size_t)d->hidden, sizeof(real));
  s->q = (real *)calloc((size_t)qw, sizeof(real));
  s->att = (real *)calloc((size_t)qw, sizeof(real));
  s->kv_k = (real *)calloc((size_t)kvw, sizeof(real));
  s->kv_v = (real *)calloc((size_t)kvw, sizeof(real));
  s->gate = (real *)calloc((size_t)d->ffn, sizeof(real));
  s->up = (real *)calloc((size_t)d->ffn, sizeof(real));
  s->sc = (real *)calloc((size_t)max_ctx, sizeof(real));
  return s;
}

static void seq_free(orc_seq *s) {
  if (!s) return;
  free(s->k); free(s->v); free(s->h); free(s->a); free(s->b); free(s->o); free(s->dn); free(s->q);
  free(s->att); free(s->kv_k); free(s->kv_v); free(s->gate); free(s->up); free(s->sc); free(s);
}

/* Feed one token at position s->len through the decoder, appending its K/V to the
 * cache; writes the vocabulary logits when `logits` is non-NULL. */
static void decode_token(const orc_model *m, orc_seq *s, int32_t token, real *logits) {
  const orc_desc *d = &m->d;
  int H = d->hidden, hd = d->head_dim, Hq = d->n_q_heads, Hkv = d->n_kv_heads, grp = Hq / Hkv;
  int64_t kvw = (int64_t)Hkv * hd;
  int pos = s->len;
  for (int i = 0; i < H; ++i) s->h[i] = (real)m->embed[(int64_t)token * H + i];
  for (int l = 0; l < d->n_layers; ++l) {
    const orc_layer *L = &m->layers[l];
    real *kc = s->k + ((int64_t)l * s->max_ctx) * kvw, *vc = s->v + ((int64_t)l * s->max_ctx) * kvw;
    orc_rmsnorm(s->a, s->h, L->attn_norm, H, d->rms_eps);
    matvec(s->q, L->wq, s->a, Hq * hd, H);
    matvec(s->kv_k, L->wk, s->a, Hkv * hd, H);
    matvec(s->kv_v, L->wv, s->a, Hkv * hd, H);
    for (int j = 0; j < Hq; ++j) {
      if (d->qk_norm) orc_rmsnorm(s->q + j * hd, s->q + j * hd, L->q_norm, hd, d->rms_eps);
      orc_rope(s->q + j * hd, hd, pos, d->rope_base);
    }
    for (int j = 0; j < Hkv; ++j) {
      if (d->qk_norm) orc_rmsnorm(s->kv_k + j * hd, s->kv_k + j * hd, L->k_norm, hd, d->rms_eps);
      orc_rope(s->kv_k + j * hd, hd, pos, d->rope_base);
    }
    memcpy(kc + (int64_t)pos * kvw, s->kv_k, sizeof(real) * (size_t)kvw);
    memcpy(vc + (int64_t)pos * kvw, s->kv_v, sizeof(real) * (size_t)kvw);
    for (int j = 0; j < Hq; ++j) {
      int g = j / grp; /* query head j reads key/value head floor(j / (Hq/Hkv)) */
      orc_attend(s->att + j * hd, s->q + j * hd, kc + g * hd, vc + g * hd, pos + 1, hd, kvw, s->sc);
    }
    matvec(s->o, L->wo, s->att, H, Hq * hd);
    for (int i = 0; i < H; ++i) s->h[i] += s->o[i];
    orc_rmsnorm(s->b, s->h, L->ffn_norm, H, d->rms_eps);
    matvec(s->gate, L->w_gate, s->b, d->ffn, H);
    matvec(s->up, L->w_up, s->b, d->ffn, H);
    for (int i = 0; i < d->ffn; ++i) s->gate[i] = orc_silu(s->gate[i]) * s->up[i];
    matvec(s->dn, L->w_down, s->gate, H, d->ffn);
    for (int i = 0; i < H; ++i) s->h[i] += s->dn[i];
  }
  s->len = pos + 1;
  if (logits) {
    orc_rmsnorm(s->a, s->h, m->final_norm, H, d->rms_eps);
    matvec(logits, m->lm_head, s->a, d->vocab, H);
  }
}

/* Incremental decode of a whole token string; logits_out [T][V] as double. */
int orc_forward_cached(const orc_desc *d, const float *blob, const int32_t *tokens, int T, double *logits_out) {
  orc_model *m = model_bind(d, blob);
  orc_seq *s = seq_new(d, T);
  real *lg = (real *)malloc(sizeof(real) * (size_t)d->vocab);
  for (int t = 0; t < T; ++t) {
    decode_token(m, s, tokens[t], lg);
    for (int i = 0; i < d->vocab; ++i) logits_out[(int64_t)t * d->vocab + i] = (double)lg[i];
  }
  free(lg); seq_free(s); model_free(m);
  return 0;
}

/* Full-sequence recompute without a cache: every layer is evaluated for all T
 * positions at once, attention by explicit causal sums.  logits_out [T][V]. */
int orc_forward_full(const orc_desc *d, const float *blob, const int32_t *tokens, int T, double *logits_out) {
  orc_model *m = model_bind(d, blob);
  int H = d->hidden, hd = d->head_dim, Hq = d->n_q_heads, Hkv = d->n_kv_heads, grp = Hq / Hkv, F = d->ffn;
  int64_t qw = (int64_t)Hq * hd, kvw = (int64_t)Hkv * hd;
  real *h = (real *)malloc(sizeof(real) * (size_t)T * H), *a = (real *)malloc(sizeof(real) * (size_t)T * H);
  real *q = (real *)malloc(sizeof(real) * (size_t)T * qw), *k = (real *)malloc(sizeof(real) * (size_t)T * kvw);
  real *v = (real *)malloc(sizeof(real) * (size_t)T * kvw), *att = (real *)malloc(sizeof(real) * (size_t)T * qw);
  real *tmp = (real *)malloc(sizeof(real) * (size_t)(H > F ? H : F)), *up = (real *)malloc(sizeof(real) * (size_t)F);
  real *sc = (real *)malloc(sizeof(real) * (size_t)T), *lg = (real *)malloc(sizeof(real) * (size_t)d->vocab);
  for (int t = 0; t < T; ++t)
    for (int i = 0; i < H; ++i) h[(int64_t)t * H + i] = (real)m->embed[(int64_t)tokens[t] * H + i];
  for (int l = 0; l < d->n_layers; ++l) {
    const orc_layer *L = &m->layers[l];
    for (int t = 0; t < T; ++t) {
      orc_rmsnorm(a + (int64_t)t * H, h + (int64_t)t * H, L->attn_norm, H, d->rms_eps);
      matvec(q + t * qw, L->wq, a + (int64_t)t * H, (int)qw, H);
      matvec(k + t * kvw, L->wk, a + (int64_t)t * H, (int)kvw, H);
      matvec(v + t * kvw, L->wv, a + (int64_t)t * H, (int)kvw, H);
      for (int j = 0; j < Hq; ++j) {
        if (d->qk_norm) orc_rmsnorm(q + t * qw + j * hd, q + t * qw + j * hd, L->q_norm, hd, d->rms_eps);
        orc_rope(q + t * qw + j * hd, hd, t, d->rope_base);
      }
      for (int j = 0; j < Hkv; ++j) {
        if (d->qk_norm) orc_rmsnorm(k + t * kvw + j * hd, k + t * kvw + j * hd, L->k_norm, hd, d->rms_eps);
        orc_rope(k + t * kvw + j * hd, hd, t, d->rope_base);
      }
    }
    for (int t = 0; t < T; ++t) /* causal: position t sees keys 0..t */
      for (int j = 0; j < Hq; ++j)
        orc_attend(att + t * qw + j * hd, q + t * qw + j * hd, k + (j / grp) * hd, v + (j / grp) * hd, t + 1, hd, kvw, sc);
    for (int t = 0; t < T; ++t) {
      real *ht = h + (int64_t)t * H;
      matvec(tmp, L->wo, att + t * qw, H, (int)qw);
      for (int i = 0; i < H; ++i) ht[i] += tmp[i];
      orc_rmsnorm(a + (int64_t)t * H, ht, L->ffn_norm, H, d->rms_eps);
      matvec(tmp, L->w_gate, a + (int64_t)t * H, F, H);
      matvec(up, L->w_up, a + (int64_t)t * H, F, H);
      for (int i = 0; i < F; ++i) up[i] = orc_silu(tmp[i]) * up[i];
      matvec(tmp, L->w_down, up, H, F);
      for (int i = 0; i < H; ++i) ht[i] += tmp[i];
    }
  }
  for (int t = 0; t < T; ++t) {
    orc_rmsnorm(a, h + (int64_t)t * H, m->final_norm, H, d->rms_eps);
    matvec(lg, m->lm_head, a, d->vocab, H);
    for (int i = 0; i < d->vocab; ++i) logits_out[(int64_t)t * d->vocab + i] = (double)lg[i];
  }
  free(h); free(a); free(q); free(k); free(v); free(att); free(tmp); free(up); free(sc); free(lg);
  model_free(m);
  return 0;
}

/* Sampling at step s of sequence n from softmax(logits / temperature) by the
 * Gumbel-max rule: tok = argmax_i (z_i + g_i), lowest index on exact ties.  The
 * decision is taken in fp32.  Returns log softmax(z)[tok] and the gap between the
 * best and second-best perturbed score (a gap near zero marks a near-tie). */
void orc_sample(const real *logits, int V, float temperature, uint64_t seed, uint32_t n, uint32_t s,
                int32_t *tok_out, double *logprob_out, float *gap_out) {
  float best = 0.f, second = 0.f;
  int32_t bi = -1;
  real mx = 0;
  for (int i = 0; i < V; ++i) {
    float z = (float)logits[i] / temperature;
    float g = orc_gumbel(orc_uniform(orc_draw_bits(seed, n, s, (uint32_t)i)));
    float sc = z + g;
    if (bi < 0) { best = sc; bi = i; second = -INFINITY; }
    else if (sc > best) { second = best; best = sc; bi = i; }
    else if (sc > second) second = sc;
    real zr = logits[i] / (real)temperature;
    if (i == 0 || zr > mx) mx = zr;
  }
  real den = 0;
  for (int i = 0; i < V; ++i) den += (real)exp((double)(logits[i] / (real)temperature - mx));
  *tok_out = bi;
  *logprob_out = (double)(logits[bi] / (real)temperature - (mx + (real)log((double)den)));
  if (gap_out) *gap_out = best - second;
}

/* Nucleus (top-p) sampling, the paper's rollout setting (Sec. 5.1: temperature 1.0, top-p 0.95): with
 * p = softmax(logits / temperature), order the tokens by probability, highest first and the lower index
 * first among equals, keep the shortest prefix of that order whose probabilities sum to at least top_p,
 * and sample from the kept set in proportion to p -- here again by the Gumbel-max rule with the same
 * noise g_i per vocabulary index, restricted to the kept set.  The returned log-prob is that of the
 * distribution actually sampled, i.e. renormalised over the kept set (the sampler's probability is what
 * the importance ratio of App. "GRPO-Style Policy Gradient Objective" divides by).  top_p >= 1 keeps
 * everything and is orc_sample.  kept_out: size of the kept set; margin_out: how far the cumulative
 * probability is from top_p on either side of the cut (a margin near zero marks a cut that rounding
 * could move by one token). */
typedef struct { real z; int32_t i; } orc_zi;
static int zi_desc(const void *a, const void *b) {
  const orc_zi *x = (const orc_zi *)a, *y = (const orc_zi *)b;
  if (x->z > y->z) return -1;
  if (x->z < y->z) return 1;
  return x->i < y->i ? -1 : (x->i > y->i ? 1 : 0);
}
void orc_sample_top_p(const real *logits, int V, float temperature, float top_p, uint64_t seed, uint32_t n,
                      uint32_t s, int32_t *tok_out, double *logprob_out, float *gap_out, int32_t *kept_out,
                      double *margin_out) {
  if (!(top_p < 1.0f)) {
    orc_sample(logits, V, temperature, seed, n, s, tok_out, logprob_out, gap_out);
    if (kept_out) *kept_out = V;
    if (margin_out) *margin_out = 1.0;
    return;
  }
  orc_zi *zs = (orc_zi *)malloc(sizeof(orc_zi) * (size_t)V);
  real mx = logits[0] / (real)temperature;
  for (int i = 0; i < V; ++i) { zs[i].z = logits[i] / (real)temperature; zs[i].i = i; if (zs[i].z > mx) mx = zs[i].z; }
  real den = 0;
  for (int i = 0; i < V; ++i) den += (real)exp((double)(zs[i].z - mx));
  qsort(zs, (size_t)V, sizeof(orc_zi), zi_desc);
  real cum = 0, before = 0;
  int k = 0;
  while (k < V) {   /* shortest prefix with cumulative probability >= top_p */
    before = cum;
    cum += (real)exp((double)(zs[k].z - mx)) / den;
    ++k;
    if (cum >= (real)top_p) break;
  }
  float best = 0.f, second = -INFINITY;
  int32_t bi = -1;
  real bz = 0, den_kept = 0;
  for (int j = 0; j < k; ++j) {
    int i = zs[j].i;
    float z = (float)logits[i] / temperature;
    float sc = z + orc_gumbel(orc_uniform(orc_draw_bits(seed, n, s, (uint32_t)i)));
    if (bi < 0 || sc > best || (sc == best && i < bi)) { if (bi >= 0) second = best > second ? best : second; best = sc; bi = i; bz = zs[j].z; }
    else if (sc > second) second = sc;
    den_kept += (real)exp((double)(zs[j].z - mx));
  }
  *tok_out = bi;
  *logprob_out = (double)(bz - (mx + (real)log((double)den_kept)));
  if (gap_out) *gap_out = best - second;
  if (kept_out) *kept_out = k;
  if (margin_out) {
    double lo = (double)top_p - (double)before, hi = (double)cum - (double)top_p;
    *margin_out = k < V ? (lo < hi ? lo : hi) : lo;
  }
  free(zs);
}

/* Rollout of P prompts x G samples (sequence n = p*G + g), each sequence on its own.
 *   blobs[j], versions[j], j < n_models: policy snapshots; snapshot j+1 replaces j
 *     for every forward pass that produces the logits of generation step >=
 *     swap_at_step[j] (the KV cache built so far is kept).  Prompts are always
 *     processed under snapshot 0.
 *   stop_lens (nullable): sequence n ends after min(max_new, stop_lens[n]) tokens;
 *   eos_id >= 0: it also ends after emitting eos_id (the token is kept).
 *   forced (nullable, [N][max_new]): teacher forcing -- the sampled token and its
 *     log-prob are still recorded, but the token fed back is forced[n][s].
 * Outputs: tokens [N][max_new] (pad -1), logprobs [N][max_new] (pad 0), lens [N],
 *   versions [N][max_new] (pad -1); optional logits [N][max_new][V] and gaps. */
int orc_rollout_top_p(const orc_desc *d, int n_models, const float *const *blobs, const int64_t *versions,
                      const int32_t *swap_at_step, const int32_t *prompts, int prompt_stride,
                      const int32_t *prompt_lens, int P, int G, int max_new, float temperature, float top_p,
                      uint64_t seed, const int32_t *stop_lens, int eos_id, const int32_t *forced,
                      int32_t *out_tokens, double *out_logprobs, int32_t *out_lens, int64_t *out_versions,
                      double *out_logits, float *out_gaps, double *out_margins) {
  if (!(top_p > 0.f)) return -1;
  if (n_models < 1 || P < 0 || G < 1 || max_new < 0 || !(temperature > 0.f)) return -1;
  orc_model **ms = (orc_model **)calloc((size_t)n_models, sizeof(orc_model *));
  for (int j = 0; j < n_models; ++j) ms[j] = model_bind(d, blobs[j]);
  real *lg = (real *)malloc(sizeof(real) * (size_t)d->vocab);
  int V = d->vocab;
  for (int n = 0; n < P * G; ++n) {
    int p = n / G, pl = prompt_lens[p];
    int limit = max_new;
    if (stop_lens && stop_lens[n] < limit) limit = stop_lens[n];
    for (int s = 0; s < max_new; ++s) {
      out_tokens[(int64_t)n * max_new + s] = -1;
      out_logprobs[(int64_t)n * max_new + s] = 0.0;
      out_versions[(int64_t)n * max_new + s] = -1;
    }
    orc_seq *sq = seq_new(d, pl + max_new + 1);
    for (int t = 0; t < pl; ++t) {
      decode_token(ms[0], sq, prompts[(int64_t)p * prompt_stride + t], t == pl - 1 ? lg : NULL);
      progress_note("rollout, prompt", n, t + 1, pl);
    }
    int len = 0, cur = 0;
    for (int s = 0; s < limit; ++s) {
      while (cur + 1 < n_models && swap_at_step[cur] <= s) ++cur;
      if (s > 0) {
        int32_t fed = forced ? forced[(int64_t)n * max_new + s - 1] : out_tokens[(int64_t)n * max_new + s - 1];
        decode_token(ms[cur], sq, fed, lg);
      }
      int32_t tok; double lp, margin; float gap;
      orc_sample_top_p(lg, V, temperature, top_p, seed, (uint32_t)n, (uint32_t)s, &tok, &lp, &gap, NULL, &margin);
      if (out_margins) out_margins[(int64_t)n * max_new + s] = margin;
      out_tokens[(int64_t)n * max_new + s] = tok;
      out_logprobs[(int64_t)n * max_new + s] = lp;
      out_versions[(int64_t)n * max_new + s] = versions[s == 0 ? 0 : cur];
      if (out_logits) for (int i = 0; i < V; ++i) out_logits[((int64_t)n * max_new + s) * V + i] = (double)lg[i];
      if (out_gaps) out_gaps[(int64_t)n * max_new + s] = gap;
      len = s + 1;
      int32_t kept = forced ? forced[(int64_t)n * max_new + s] : tok;
      if (eos_id >= 0 && kept == eos_id) break;
    }
    out_lens[n] = len;
    seq_free(sq);
  }
  free(lg);
  for (int j = 0; j < n_models; ++j) model_free(ms[j]);
  free(ms);
  return 0;
}

int orc_rollout(const orc_desc *d, int n_models, const float *const *blobs, const int64_t *versions,
                const int32_t *swap_at_step, const int32_t *prompts, int prompt_stride,
                const int32_t *prompt_lens, int P, int G, int max_new, float temperature, uint64_t seed,
                const int32_t *stop_lens, int eos_id, const int32_t *forced, int32_t *out_tokens,
                double *out_logprobs, int32_t *out_lens, int64_t *out_versions, double *out_logits,
                float *out_gaps) {
  return orc_rollout_top_p(d, n_models, blobs, versions, swap_at_step, prompts, prompt_stride, prompt_lens, P, G, max_new,
                           temperature, 1.0f, seed, stop_lens, eos_id, forced, out_tokens, out_logprobs, out_lens,
                           out_versions, out_logits, out_gaps, NULL);
}

/* Learner-side tensors of a batch of records (App. "Turn-Aware Masking" and "Outcome-Based Returns and
 * Group-wise Normalization").
 *   Turn index c[n][t] = number of positions k <= t with tokens[n][k] == turn_start; the response mask
 *   selects the tokens of the odd turns after the first: m[n][t] = [c > 1][c odd]; positions >= lens[n]
 *   are 0.
 *   Advantage of sequence n within its group of G consecutive sequences:
 *   A_n = (R_n - mean) / (std + eps), std the sample standard deviation (divisor G - 1), which is what the
 *   paper's listing computes; adv_tok[n][t] = A_n * m[n][t].  G >= 2. */
int orc_grpo_tensors(const int32_t *tokens, int stride, const int32_t *lens, int n_seqs, int G, int32_t turn_start,
                     const double *rewards, double eps, uint8_t *out_mask, double *out_adv, double *out_adv_tok) {
  if (n_seqs < 0 || G < 2 || n_seqs % G) return -1;
  for (int g0 = 0; g0 < n_seqs; g0 += G) {
    double mean = 0, ss = 0;
    for (int j = 0; j < G; ++j) mean += rewards[g0 + j];
    mean /= G;
    for (int j = 0; j < G; ++j) ss += (rewards[g0 + j] - mean) * (rewards[g0 + j] - mean);
    double sd = sqrt(ss / (G - 1));
    for (int j = 0; j < G; ++j) out_adv[g0 + j] = (rewards[g0 + j] - mean) / (sd + eps);
  }
  for (int n = 0; n < n_seqs; ++n) {
    int c = 0;
    for (int t = 0; t < stride; ++t) {
      uint8_t m = 0;
      if (t < lens[n]) {
        if (tokens[(int64_t)n * stride + t] == turn_start) ++c;
        m = (uint8_t)(c > 1 && (c & 1));
      }
      out_mask[(int64_t)n * stride + t] = m;
      if (out_adv_tok) out_adv_tok[(int64_t)n * stride + t] = m ? out_adv[n] : 0.0;
    }
  }
  return 0;
}

/* Teacher-forced scoring of one token string under one snapshot:
 * out[t] = log softmax(logits_{t-1} / temperature)[tokens[t]] for t >= 1, out[0] = 0. */
int orc_logprobs(const orc_desc *d, const float *blob, const int32_t *tokens, int T, float temperature, double *out) {
  orc_model *m = model_bind(d, blob);
  orc_seq *s = seq_new(d, T);
  real *lg = (real *)malloc(sizeof(real) * (size_t)d->vocab), *ls = (real *)malloc(sizeof(real) * (size_t)d->vocab);
  if (T > 0) out[0] = 0.0;
  for (int t = 0; t + 1 < T; ++t) {
    decode_token(m, s, tokens[t], lg);
    orc_log_softmax(ls, lg, d->vocab, temperature);
    out[t + 1] = (double)ls[tokens[t + 1]];
    progress_note("scoring", 0, t + 1, T - 1);
  }
  free(lg); free(ls); seq_free(s); model_free(m);
  return 0;
}

/* Thin array entry points over the primitives (double in/out) for the pin tests. */
void orc_rmsnorm_d(double *y, const double *x, const float *g, int n, float eps) {
  real *xi = (real *)malloc(sizeof(real) * (size_t)n), *yo = (real *)malloc(sizeof(real) * (size_t)n);
  for (int i = 0; i < n; ++i) xi[i] = (real)x[i];
  orc_rmsnorm(yo, xi, g, n, eps);
  for (int i = 0; i < n; ++i) y[i] = (double)yo[i];
  free(xi); free(yo);
}

void orc_rope_d(double *x, int hd, int pos, float base) {
  real *xi = (real *)malloc(sizeof(real) * (size_t)hd);
  for (int i = 0; i < hd; ++i) xi[i] = (real)x[i];
  orc_rope(xi, hd, pos, base);
  for (int i = 0; i < hd; ++i) x[i] = (double)xi[i];
  free(xi);
}

double orc_silu_d(double x) { return (double)orc_silu((real)x); }

void orc_attend_d(double *o, const double *q, const double *k, const double *v, int n_keys, int hd) {
  real *qi = (real *)malloc(sizeof(real) * (size_t)hd), *oi = (real *)malloc(sizeof(real) * (size_t)hd);
  real *ki = (real *)malloc(sizeof(real) * (size_t)n_keys * hd), *vi = (real *)malloc(sizeof(real) * (size_t)n_keys * hd);
  real *sc = (real *)malloc(sizeof(real) * (size_t)n_keys);
  for (int i = 0; i < hd; ++i) qi[i] = (real)q[i];
  for (int i = 0; i < n_keys * hd; ++i) { ki[i] = (real)k[i]; vi[i] = (real)v[i]; }
  orc_attend(oi, qi, ki, vi, n_keys, hd, hd, sc);
  for (int i = 0; i < hd; ++i) o[i] = (double)oi[i];
  free(qi); free(oi); free(ki); free(vi); free(sc);
}

void orc_log_softmax_d(double *out, const double *logits, int n, float temperature) {
  real *li = (real *)malloc(sizeof(real) * (size_t)n), *lo = (real *)malloc(sizeof(real) * (size_t)n);
  for (int i = 0; i < n; ++i) li[i] = (real)logits[i];
  orc_log_softmax(lo, li, n, temperature);
  for (int i = 0; i < n; ++i) out[i] = (double)lo[i];
  free(li); free(lo);
}

void orc_sample_top_p_d(const double *logits, int V, float temperature, float top_p, uint64_t seed, uint32_t n, uint32_t s,
                        int32_t *tok_out, double *logprob_out, float *gap_out, int32_t *kept_out, double *margin_out) {
  real *li = (real *)malloc(sizeof(real) * (size_t)V);
  for (int i = 0; i < V; ++i) li[i] = (real)logits[i];
  orc_sample_top_p(li, V, temperature, top_p, seed, n, s, tok_out, logprob_out, gap_out, kept_out, margin_out);
  free(li);
}

void orc_sample_d(const double *logits, int V, float temperature, uint64_t seed, uint32_t n, uint32_t s,
                  int32_t *tok_out, double *logprob_out, float *gap_out) {
  real *li = (real *)malloc(sizeof(real) * (size_t)V);
  for (int i = 0; i < V; ++i) li[i] = (real)logits[i];
  orc_sample(li, V, temperature, seed, n, s, tok_out, logprob_out, gap_out);
  free(li);
}
