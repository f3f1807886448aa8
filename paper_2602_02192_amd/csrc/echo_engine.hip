// Host engine behind the C ABI: arena planning, snapshot install and swap, prefill, the decode loop
// (one HIP graph per snapshot, replayed per generation step), teacher-forced scoring, statistics.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/echo.h"
#include "echo_kernels.h"

using namespace echo;

namespace {

thread_local std::string g_init_error;

struct LayerW {
  const void *attn_norm, *wqkv, *q_norm, *k_norm, *wo, *ffn_norm, *wgu, *wdown;
};
struct Slot {
  int64_t version = -1;
  char *base = nullptr;
  const void *embed = nullptr, *final_norm = nullptr, *lm_head = nullptr;
  std::vector<LayerW> layers;
};

struct Bump {  // plans offsets inside the caller's arena
  size_t off = 0;
  size_t take(size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; }
};

struct Plan {
  bool ok = false, fast = false;
  int elt = 4;                  // bytes per weight element
  int Mcap = 0;                 // row capacity of one pass
  int Np_qkv, Np_d, Np_gu, Np_v, Kp_d, Kp_q, Kp_f;
  size_t slot_bytes, o_slot[2], o_kv, kv_bytes;
  size_t o_h, o_x, o_qkv, o_att, o_gu, o_ff, o_logits, o_q16, o_xa, o_xatt, o_xff, o_part, o_rope, o_lmpart;
  size_t o_attn_o, o_attn_ml, o_topp, o_pjobs;
  size_t o_blocks, o_rows, o_seq, o_samp, o_out_tok, o_out_lp, o_out_ver, o_forced, o_scal, o_first_h, o_stage, o_maps;
  size_t stage_bytes, part_floats, logit_rows = 0, total;
  int attn_chunk, attn_max_splits;
};

constexpr int PREFILL_ROWS = 4096;   // rows per pass of prefill and of teacher-forced scoring
constexpr size_t STAGE_BYTES = (size_t)64 << 20;
constexpr int MAX_GRID_SPLIT = REDUCE_MAX_SPLIT;

int pad_rows(int m) {  // 32 * pow2 up to 256, then multiples of 256
  int p = 32;
  while (p < m && p < 256) p *= 2;
  if (m > 256) p = (int)round_up(m, 256);
  return p;
}

size_t packed_bytes(int64_t N, int64_t K) { return (size_t)(round_up(N, 32) * round_up(K, GEMM_K_PAD) * 2); }

bool valid_desc(const echo_model_desc *d, std::string *why) {
  auto bad = [&](const char *m) { if (why) *why = m; return false; };
  if (!d) return bad("desc is NULL");
  if (d->n_layers < 1 || d->hidden < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->head_dim < 2 || d->ffn < 1 || d->vocab < 1)
    return bad("non-positive model dimension");
  if (d->n_q_heads % d->n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
  if (d->head_dim % 2 || d->head_dim > 256) return bad("head_dim must be even and <= 256");
  if (d->dtype != ECHO_F32 && d->dtype != ECHO_BF16) return bad("dtype must be ECHO_F32 or ECHO_BF16");
  if (d->max_seqs < 1 || d->max_ctx < 2) return bad("max_seqs / max_ctx too small");
  if (d->n_weight_slots != 1 && d->n_weight_slots != 2) return bad("n_weight_slots must be 1 or 2");
  if (!(d->rms_eps >= 0.f) || !(d->rope_base > 0.f)) return bad("rms_eps / rope_base out of range");
  bool fast = d->dtype == ECHO_BF16 && !d->debug_naive;
  if (fast) {
    if (d->hidden % 16 || d->ffn % 16 || (d->n_q_heads * d->head_dim) % 16) return bad("bf16 path needs hidden, ffn and Hq*head_dim multiples of 16");
    if (d->hidden > 8192) return bad("bf16 path needs hidden <= 8192");
    if (d->head_dim != 64 && d->head_dim != 128) return bad("bf16 path needs head_dim 64 or 128");
    int grp = d->n_q_heads / d->n_kv_heads;
    if (grp > 8 || (grp & (grp - 1))) return bad("bf16 path needs Hq/Hkv in {1,2,4,8}");
  }
  return true;
}

int64_t blob_numel(const echo_model_desc *d) {
  int64_t h = d->hidden, hd = d->head_dim, q = (int64_t)d->n_q_heads * hd, kv = (int64_t)d->n_kv_heads * hd;
  int64_t per = h + q * h + 2 * kv * h + (d->qk_norm ? 2 * hd : 0) + h * q + h + 3 * (int64_t)d->ffn * h;
  return (int64_t)d->vocab * h + d->n_layers * per + h + (d->tie_embeddings ? 0 : (int64_t)d->vocab * h);
}

Plan make_plan(const echo_model_desc *d) {
  Plan p;
  if (!valid_desc(d, nullptr)) return p;
  p.fast = d->dtype == ECHO_BF16 && !d->debug_naive;
  p.elt = d->dtype == ECHO_BF16 ? 2 : 4;
  int64_t H = d->hidden, hd = d->head_dim, Q = (int64_t)d->n_q_heads * hd, KV = (int64_t)d->n_kv_heads * hd, F = d->ffn, V = d->vocab;
  p.Mcap = std::max(pad_rows(d->max_seqs), PREFILL_ROWS);
  p.Np_qkv = (int)round_up(Q + 2 * KV, 32); p.Np_d = (int)round_up(H, 32); p.Np_gu = (int)round_up(2 * F, 32);
  p.Np_v = (int)round_up(V, 64);
  p.Kp_d = (int)round_up(H, GEMM_K_PAD); p.Kp_q = (int)round_up(Q, GEMM_K_PAD); p.Kp_f = (int)round_up(F, GEMM_K_PAD);
  Bump b;
  if (p.fast) {
    size_t per = 2 * H * 2 + (d->qk_norm ? 2 * hd * 2 : 0) + 4 * 256 /*alignment slack*/ + packed_bytes(Q + 2 * KV, H) +
                 packed_bytes(H, Q) + packed_bytes(2 * F, H) + packed_bytes(H, F);
    p.slot_bytes = (size_t)V * H * 2 + 256 + H * 2 + 256 + packed_bytes(round_up(V, 64), H) + d->n_layers * (per + 8 * 256);
  } else {
    p.slot_bytes = (size_t)blob_numel(d) * p.elt;
  }
  for (int s = 0; s < d->n_weight_slots; ++s) p.o_slot[s] = b.take(p.slot_bytes);
  int kv_elt = p.fast ? 2 : 4;
  int64_t ctx_cap = p.fast ? round_up(d->max_ctx, 32) : d->max_ctx;   // the tiled cache holds whole tiles of 32 keys
  p.kv_bytes = (size_t)d->max_seqs * d->n_layers * 2 * d->n_kv_heads * ctx_cap * hd * kv_elt;
  p.o_kv = b.take(p.kv_bytes);
  size_t M = p.Mcap, Md = pad_rows(d->max_seqs);   // rows of a prefill / scoring pass, rows of a decode step
  p.o_h = b.take(M * H * 4);
  p.o_first_h = b.take((size_t)d->max_seqs * H * 4);
  p.logit_rows = p.fast ? Md : M;   // the MFMA path never writes logits of a scoring pass
  p.o_logits = b.take(p.logit_rows * (size_t)p.Np_v * 4);
  p.o_rope = b.take(M * hd * 4);
  if (p.fast) {
    p.o_xa = b.take(M * p.Kp_d * 2);
    p.o_xatt = b.take(M * p.Kp_q * 2);
    p.o_xff = b.take(M * p.Kp_f * 2);
    p.o_q16 = b.take(M * Q * 2);
    // split-K partials: every split count the reducers take for a decode step, fewer for the long passes
    p.part_floats = std::max((size_t)MAX_GRID_SPLIT * Md, (size_t)2 * M) * std::max(p.Np_qkv, p.Np_d);
    p.o_part = b.take(p.part_floats * 4);
    p.o_lmpart = b.take(fast_lmhead_partial_floats(p.Np_v, (int)M) * 4);
    p.attn_chunk = 32;
    p.attn_max_splits = 32;   // partial-buffer capacity in splits per (row, head)
    p.o_attn_o = b.take(Md * d->n_q_heads * (size_t)p.attn_max_splits * hd * 4);   // decode rows only
    p.o_attn_ml = b.take(Md * d->n_q_heads * (size_t)p.attn_max_splits * 2 * 4);
    p.stage_bytes = STAGE_BYTES;
    p.o_stage = b.take(p.stage_bytes);
  } else {
    p.o_x = b.take(M * H * 4);
    p.o_qkv = b.take(M * (Q + 2 * KV) * 4);
    p.o_att = b.take(M * Q * 4);
    p.o_gu = b.take(M * 2 * F * 4);
    p.o_ff = b.take(M * F * 4);
  }
  p.o_blocks = b.take(M * sizeof(PrefillBlock));   // at worst every row of a pass is a block of its own
  p.o_topp = b.take(fast_topp_scratch_floats((int)pad_rows(d->max_seqs)) * 4);
  p.o_pjobs = b.take((pad_rows(d->max_seqs) / 2 + 1) * sizeof(PrefixJob));   // a job has at least two rows
  p.o_rows = b.take(6 * M * 4);
  p.o_maps = b.take(2 * M * 4 + (size_t)d->max_seqs * 4);
  p.o_seq = b.take(4 * (size_t)pad_rows(d->max_seqs) * 4);   // samplers read the step and stream of padding rows too
  p.o_samp = b.take(4 * M * 4);
  size_t outn = (size_t)d->max_seqs * d->max_ctx;
  p.o_out_tok = b.take(outn * 4);
  p.o_out_lp = b.take(outn * 4);
  p.o_out_ver = b.take(outn * 8);
  p.o_forced = b.take(outn * 4);
  p.o_scal = b.take(256);
  p.total = b.off;
  p.ok = true;
  return p;
}

}  // namespace

// A byte range of a snapshot blob and where it goes: a plain copy to dst (rows == 0), or rows x K bf16 values that are
// packed into the weight at dst, blob row r becoming packed row dst_row0 + r * stride.
struct BlobSeg {
  size_t off, bytes;
  char *dst;
  int64_t rows = 0;
  int K = 0;
  int64_t dst_row0 = 0;
  int stride = 1;
  std::vector<char> carry;
};

// A snapshot that is arriving piece by piece (echo_load_policy_begin .. _commit).
struct Loading {
  bool open = false;
  int64_t version = -1;
  int target = -1;
  size_t received = 0, total = 0;
  std::vector<BlobSeg> segs;
};

struct echo_ctx {
  echo_model_desc d;
  Plan p;
  int device = 0;
  char *arena = nullptr;
  hipStream_t cs = nullptr, ks = nullptr;  // compute, copy
  bool own_cs = false, own_ks = false;
  Slot slots[2];
  int active = -1, staged = -1;
  hipEvent_t staged_ev = nullptr;
  Loading load;
  int64_t newest_version = -1;
  int stage_flip = 0;
  bool rollout_running = false;
  std::mutex mu;
  std::condition_variable cv;
  std::string err;
  echo_stats_t st;
  // device views
  RowState rows;
  KvGeom kv;
  int32_t *d_prompt_len_seq, *d_gen_len, *d_limit, *d_samp_tok, *d_target, *d_step, *d_n_active, *d_map_a, *d_map_b, *d_plen_p;
  float *d_samp_lp, *d_target_lp;
  int32_t *d_stream;  // per-row stream ids of a continuous rollout
  DrawIds ids{nullptr, nullptr, nullptr};
  PrefixPlan px{nullptr, 0, 0, 1};       // shared-prompt attention jobs of the running rollout (n_jobs = 0: none)
  hipGraphExec_t graph = nullptr;
  // kernel timing (time_kernels)
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_attn, ev_gemm;
  bool timing = false;
  double t_attn_bytes = 0, t_gemm_bytes = 0, cur_attn_bytes = 0;
};

namespace {

int fail(echo_ctx *c, int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_init_error = buf;
  return code;
}

#define HIPCHK(c, expr)                                                                      \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return fail(c, ECHO_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

template <typename T> T *at(echo_ctx *c, size_t off) { return (T *)(c->arena + off); }

void bind_slot(echo_ctx *c, int s) {
  const echo_model_desc &d = c->d;
  Slot &S = c->slots[s];
  S.base = c->arena + c->p.o_slot[s];
  S.layers.assign(d.n_layers, LayerW{});
  int64_t H = d.hidden, hd = d.head_dim, Q = (int64_t)d.n_q_heads * hd, KV = (int64_t)d.n_kv_heads * hd, F = d.ffn, V = d.vocab;
  if (!c->p.fast) {  // the raw blob itself
    size_t e = c->p.elt;
    char *p = S.base;
    S.embed = p; p += V * H * e;
    for (int l = 0; l < d.n_layers; ++l) {
      LayerW &L = S.layers[l];
      L.attn_norm = p; p += H * e;
      L.wqkv = p; p += (Q + 2 * KV) * H * e;
      if (d.qk_norm) { L.q_norm = p; p += hd * e; L.k_norm = p; p += hd * e; }
      L.wo = p; p += H * Q * e;
      L.ffn_norm = p; p += H * e;
      L.wgu = p; p += 2 * F * H * e;
      L.wdown = p; p += H * F * e;
    }
    S.final_norm = p; p += H * e;
    S.lm_head = d.tie_embeddings ? S.embed : p;
    return;
  }
  Bump b;
  auto take = [&](size_t n) { return (const void *)(S.base + b.take(n)); };
  S.embed = take((size_t)V * H * 2);
  S.final_norm = take(H * 2);
  S.lm_head = take(packed_bytes(round_up(V, 64), H));
  for (int l = 0; l < d.n_layers; ++l) {
    LayerW &L = S.layers[l];
    L.attn_norm = take(H * 2);
    L.ffn_norm = take(H * 2);
    if (d.qk_norm) { L.q_norm = take(hd * 2); L.k_norm = take(hd * 2); }
    L.wqkv = take(packed_bytes(Q + 2 * KV, H));
    L.wo = take(packed_bytes(H, Q));
    L.wgu = take(packed_bytes(2 * F, H));
    L.wdown = take(packed_bytes(H, F));
  }
}

// Upload rows r0 .. r0+n-1 of a row-major bf16 matrix through the staging buffer and pack them into its weight.
int stage_rows(echo_ctx *c, const BlobSeg &g, const char *src, int64_t r0, int64_t n_rows) {
  int Np = (int)round_up(g.rows * g.stride, 32);
  int Kp = (int)round_up(g.K, GEMM_K_PAD);
  int64_t row_bytes = (int64_t)g.K * 2, rows_per = std::max<int64_t>(1, (int64_t)(c->p.stage_bytes / 2) / row_bytes);
  for (int64_t r = 0; r < n_rows; r += rows_per) {
    int64_t n = std::min(rows_per, n_rows - r);
    char *stg = c->arena + c->p.o_stage + (c->stage_flip ? c->p.stage_bytes / 2 : 0);
    c->stage_flip ^= 1;
    HIPCHK(c, hipMemcpyAsync(stg, src + r * row_bytes, (size_t)(n * row_bytes), hipMemcpyHostToDevice, c->ks));
    fast_pack_weight(g.dst, stg, g.dst_row0 + (r0 + r) * g.stride, g.stride, n, g.K, Kp, Np, c->ks);
  }
  return 0;
}

// The byte ranges of a snapshot blob for weight slot s, each with the place its bytes go to.
std::vector<BlobSeg> blob_segments(echo_ctx *c, int s) {
  const echo_model_desc &d = c->d;
  Slot &S = c->slots[s];
  std::vector<BlobSeg> v;
  if (!c->p.fast) {  // the slot holds the blob as it is
    v.push_back(BlobSeg{0, c->p.slot_bytes, S.base});
    return v;
  }
  int64_t H = d.hidden, hd = d.head_dim, Q = (int64_t)d.n_q_heads * hd, KV = (int64_t)d.n_kv_heads * hd, F = d.ffn, V = d.vocab;
  size_t off = 0;
  auto raw = [&](const void *dst, size_t bytes) { v.push_back(BlobSeg{off, bytes, (char *)dst}); off += bytes; };
  auto mat = [&](const void *dst, int64_t rows, int64_t K, int64_t row0, int stride, size_t at_off, bool advance) {
    BlobSeg g{at_off, (size_t)(rows * K * 2), (char *)dst};
    g.rows = rows; g.K = (int)K; g.dst_row0 = row0; g.stride = stride;
    v.push_back(g);
    if (advance) off += g.bytes;
  };
  size_t embed_off = off;
  raw(S.embed, (size_t)V * H * 2);
  for (int l = 0; l < d.n_layers; ++l) {
    LayerW &L = S.layers[l];
    raw(L.attn_norm, H * 2);
    mat(L.wqkv, Q + 2 * KV, H, 0, 1, off, true);
    if (d.qk_norm) { raw(L.q_norm, hd * 2); raw(L.k_norm, hd * 2); }
    mat(L.wo, H, Q, 0, 1, off, true);
    raw(L.ffn_norm, H * 2);
    mat(L.wgu, F, H, 0, 2, off, true);  // gate -> even rows
    mat(L.wgu, F, H, 1, 2, off, true);  // up   -> odd rows
    mat(L.wdown, H, F, 0, 1, off, true);
  }
  raw(S.final_norm, H * 2);
  if (d.tie_embeddings) mat(S.lm_head, V, H, 0, 1, embed_off, false);  // a second consumer of the embedding's bytes
  else mat(S.lm_head, V, H, 0, 1, off, true);
  return v;
}

// Bytes [lo, lo + n) of the blob have arrived at `data`: send the part of every segment they cover on its way.
// A matrix moves in whole rows; the bytes of a row cut by the end of a piece wait in the segment's carry buffer.
int feed_segments(echo_ctx *c, std::vector<BlobSeg> &segs, const char *data, size_t lo, size_t n) {
  size_t hi = lo + n;
  for (BlobSeg &g : segs) {
    size_t a = std::max(lo, g.off), b = std::min(hi, g.off + g.bytes);
    if (a >= b) continue;
    const char *src = data + (a - lo);
    size_t rel = a - g.off, len = b - a;
    if (g.rows == 0) {
      for (size_t o = 0; o < len; o += (size_t)256 << 20)
        HIPCHK(c, hipMemcpyAsync(g.dst + rel + o, src + o, std::min((size_t)256 << 20, len - o), hipMemcpyHostToDevice, c->ks));
      continue;
    }
    size_t row_bytes = (size_t)g.K * 2;
    if (!g.carry.empty()) {  // finish the row the last piece left open
      size_t take = std::min(row_bytes - g.carry.size(), len);
      int64_t row = (int64_t)((rel - g.carry.size()) / row_bytes);
      g.carry.insert(g.carry.end(), src, src + take);
      src += take; rel += take; len -= take;
      if (g.carry.size() < row_bytes) continue;
      int rc = stage_rows(c, g, g.carry.data(), row, 1);
      if (rc) return rc;
      HIPCHK(c, hipStreamSynchronize(c->ks));  // the carry buffer is reused below
      g.carry.clear();
    }
    size_t whole = len / row_bytes;
    if (whole) {
      int rc = stage_rows(c, g, src, (int64_t)(rel / row_bytes), (int64_t)whole);
      if (rc) return rc;
    }
    g.carry.assign(src + whole * row_bytes, src + len);
  }
  return 0;
}

// ---- one forward pass over M rows (row state already on the device) ----------------------------------------
struct TimerScope {
  echo_ctx *c; std::vector<std::pair<hipEvent_t, hipEvent_t>> *v; hipEvent_t a = nullptr, b = nullptr;
  TimerScope(echo_ctx *c_, std::vector<std::pair<hipEvent_t, hipEvent_t>> *v_) : c(c_), v(v_) {
    if (!c->timing) return;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { a = b = nullptr; return; }
    hipEventRecord(a, c->cs);
  }
  ~TimerScope() { if (a && b) { hipEventRecord(b, c->cs); v->push_back({a, b}); } }
};

void gemm_fast(echo_ctx *c, void *out, const void *Xp, const void *Wp, int Mp, int Np, int Kp, GemmEpilogue epi, int *nsplit_out) {
  GemmShape g;
  fast_gemm_pick(Np, Kp, Mp, epi == EPI_SWIGLU, &g);
  if (g.nsplit > MAX_GRID_SPLIT) g.nsplit = MAX_GRID_SPLIT;
  if (epi == EPI_PARTIAL) {   // the partial buffer holds part_floats
    int room = (int)(c->p.part_floats / ((size_t)Np * Mp));
    if (g.nsplit > room) g.nsplit = room;
  }
  if (g.lds == 3) g.nsplit = fast_gemm_even_split(Kp, g.nsplit);
  {
    TimerScope t(c, &c->ev_gemm);
    fast_gemm(out, Xp, Wp, Mp, Np, Kp, g, epi, c->cs);
  }
  if (c->timing) c->t_gemm_bytes += (double)Np * Kp * 2;
  if (nsplit_out) *nsplit_out = g.nsplit;
}

void forward_layers(echo_ctx *c, const Slot &S, int M, bool use_splitk_attn, int n_prefill_blocks = 0) {
  const echo_model_desc &d = c->d;
  const Plan &p = c->p;
  hipStream_t st = c->cs;
  int Hq = d.n_q_heads, Hkv = d.n_kv_heads, hd = d.head_dim, H = d.hidden, F = d.ffn;
  float *h = at<float>(c, p.o_h), *rope = at<float>(c, p.o_rope);
  launch_rope_table(rope, c->rows.pos, M, hd, d.rope_base, st);
  if (!p.fast) {
    int bf = d.dtype == ECHO_BF16;
    float *x = at<float>(c, p.o_x), *qkv = at<float>(c, p.o_qkv), *att = at<float>(c, p.o_att), *gu = at<float>(c, p.o_gu),
          *ff = at<float>(c, p.o_ff);
    dbg_embed(h, S.embed, bf, c->rows.token, M, H, st);
    for (int l = 0; l < d.n_layers; ++l) {
      const LayerW &L = S.layers[l];
      dbg_rmsnorm(x, h, L.attn_norm, bf, M, H, d.rms_eps, st);
      dbg_gemm(qkv, x, L.wqkv, bf, M, (Hq + 2 * Hkv) * hd, H, 0, st);
      dbg_qkv_post(qkv, L.q_norm, L.k_norm, bf, d.qk_norm, d.rms_eps, rope, c->rows, c->kv, l, M, Hq, Hkv, st);
      dbg_attention(att, qkv, c->rows, c->kv, l, M, Hq, Hkv, st);
      dbg_gemm(h, att, L.wo, bf, M, H, Hq * hd, 1, st);
      dbg_rmsnorm(x, h, L.ffn_norm, bf, M, H, d.rms_eps, st);
      dbg_gemm(gu, x, L.wgu, bf, M, 2 * F, H, 0, st);
      dbg_swiglu(ff, gu, M, F, st);
      dbg_gemm(h, ff, L.wdown, bf, M, H, F, 1, st);
    }
    dbg_rmsnorm(x, h, S.final_norm, bf, M, H, d.rms_eps, st);
    return;
  }
  int Mp = pad_rows(M), ns;
  void *xa = at<void>(c, p.o_xa), *xatt = at<void>(c, p.o_xatt), *xff = at<void>(c, p.o_xff), *q16 = at<void>(c, p.o_q16);
  float *part = at<float>(c, p.o_part);
  fast_resid_norm(h, S.embed, c->rows.token, nullptr, 0, p.Np_d, xa, S.layers[0].attn_norm, M, Mp, H, d.rms_eps, st);
  for (int l = 0; l < d.n_layers; ++l) {
    const LayerW &L = S.layers[l];
    gemm_fast(c, part, xa, L.wqkv, Mp, p.Np_qkv, p.Kp_d, EPI_PARTIAL, &ns);
    fast_qkv_post(part, ns, p.Np_qkv, Mp, q16, L.q_norm, L.k_norm, d.qk_norm, d.rms_eps, rope, c->rows, c->kv, l, M, Hq, Hkv, st);
    if (n_prefill_blocks == 0 && use_splitk_attn)   // the groups' shared prompt tiles, once per group (outside the timed launch)
      fast_attention_prefix(q16, c->kv, l, Hq, Hkv, at<float>(c, p.o_attn_o), at<float>(c, p.o_attn_ml), c->px, st);
    {
      TimerScope t(c, &c->ev_attn);
      if (n_prefill_blocks > 0)
        fast_attention_prefill(xatt, q16, at<PrefillBlock>(c, p.o_blocks), n_prefill_blocks, c->kv, l, Mp, Hq, Hkv, st);
      else if (use_splitk_attn)
        fast_attention(xatt, q16, c->rows, c->kv, l, M, Mp, Hq, Hkv, fast_attention_splits(M, Hkv, p.attn_max_splits),
                       at<float>(c, p.o_attn_o), at<float>(c, p.o_attn_ml), c->px, st);
      else
        fast_attention_simple(xatt, q16, c->rows, c->kv, l, M, Mp, Hq, Hkv, st);
    }
    if (c->timing) c->t_attn_bytes += c->cur_attn_bytes;
    gemm_fast(c, part, xatt, L.wo, Mp, p.Np_d, p.Kp_q, EPI_PARTIAL, &ns);
    fast_resid_norm(h, nullptr, nullptr, part, ns, p.Np_d, xa, L.ffn_norm, M, Mp, H, d.rms_eps, st);
    gemm_fast(c, xff, xa, L.wgu, Mp, p.Np_gu, p.Kp_d, EPI_SWIGLU, nullptr);
    gemm_fast(c, part, xff, L.wdown, Mp, p.Np_d, p.Kp_f, EPI_PARTIAL, &ns);
    const void *next_gain = l + 1 < d.n_layers ? S.layers[l + 1].attn_norm : S.final_norm;
    fast_resid_norm(h, nullptr, nullptr, part, ns, p.Np_d, xa, next_gain, M, Mp, H, d.rms_eps, st);
  }
}

// lm_head + sampler over the normed rows left by forward_layers (or by norm_only).
// top_p < 1: cut, slice partials, combine -> d_samp_tok / d_samp_lp
void nucleus(echo_ctx *c, const float *logits, int64_t ld, int M, float temperature, float top_p, uint64_t seed) {
  int Mp = pad_rows(M);
  float *scratch = at<float>(c, c->p.o_topp);
  fast_topp_cut_and_draw(scratch, logits, ld, M, Mp, c->d.vocab, temperature, top_p, seed, c->ids, nullptr, c->cs);
  fast_sample_combine(c->d_samp_tok, c->d_samp_lp, scratch, TOPP_CHUNKS_PER_ROW, M, Mp, nullptr, c->cs);
}

void sample_rows(echo_ctx *c, const Slot &S, int M, float temperature, uint64_t seed, bool unfused, const int32_t *target,
                 float top_p = 1.0f) {
  const echo_model_desc &d = c->d;
  const Plan &p = c->p;
  hipStream_t st = c->cs;
  float *logits = at<float>(c, p.o_logits);
  if (!p.fast) {
    int bf = d.dtype == ECHO_BF16;
    dbg_gemm(logits, at<float>(c, p.o_x), S.lm_head, bf, M, d.vocab, d.hidden, 0, st);
    if (top_p < 1.0f) nucleus(c, logits, d.vocab, M, temperature, top_p, seed);
    else dbg_sample(c->d_samp_tok, c->d_samp_lp, logits, d.vocab, M, d.vocab, temperature, seed, c->ids, nullptr, st);
    if (target) dbg_target_logprob(c->d_target_lp, logits, d.vocab, M, d.vocab, temperature, target, st);
    return;
  }
  int Mp = pad_rows(M);
  if (unfused) {
    {
      TimerScope t(c, &c->ev_gemm);
      fast_lmhead_logits(logits, p.Np_v, at<void>(c, p.o_xa), S.lm_head, Mp, p.Np_v, p.Kp_d, d.vocab, st);
    }
    if (top_p < 1.0f) nucleus(c, logits, p.Np_v, M, temperature, top_p, seed);
    else dbg_sample(c->d_samp_tok, c->d_samp_lp, logits, p.Np_v, M, d.vocab, temperature, seed, c->ids, nullptr, st);
    if (target) dbg_target_logprob(c->d_target_lp, logits, p.Np_v, M, d.vocab, temperature, target, st);
  } else {
    TimerScope t(c, &c->ev_gemm);
    fast_lmhead_sample(c->d_samp_tok, c->d_samp_lp, c->d_target_lp, at<void>(c, p.o_xa), S.lm_head, Mp, M, d.vocab, p.Np_v, p.Kp_d,
                       temperature, seed, c->ids, nullptr, target, at<float>(c, p.o_lmpart), st);
  }
  if (c->timing) c->t_gemm_bytes += (double)p.Np_v * p.Kp_d * 2;
}

int64_t logits_ld(echo_ctx *c) { return c->p.fast ? c->p.Np_v : c->d.vocab; }

// h rows -> normed rows (no layers): used for the first sampled token of every sequence.
void norm_only(echo_ctx *c, const Slot &S, int M) {
  const echo_model_desc &d = c->d;
  const Plan &p = c->p;
  if (!p.fast) dbg_rmsnorm(at<float>(c, p.o_x), at<float>(c, p.o_h), S.final_norm, d.dtype == ECHO_BF16, M, d.hidden, d.rms_eps, c->cs);
  else fast_resid_norm(at<float>(c, p.o_h), nullptr, nullptr, nullptr, 0, p.Np_d, at<void>(c, p.o_xa), S.final_norm, M, pad_rows(M),
                       d.hidden, d.rms_eps, c->cs);
}

bool env_flag(const char *name) { const char *v = getenv(name); return v && v[0] && v[0] != '0'; }

struct ChunkRow { int32_t token, slot, pos; };

// Feed the token strings (one per cache slot slot0 + q*slot_step) through the decoder in chunks of rows.
// After each chunk `after(chunk_rows, M)` runs (still on the compute stream).
struct ChunkSeq { const int32_t *tokens; int len, slot; };

template <typename F>
int run_chunk_seqs(echo_ctx *c, const Slot &S, const std::vector<ChunkSeq> &seqs, F after) {
  std::vector<ChunkRow> all;
  for (const ChunkSeq &q : seqs)
    for (int t = 0; t < q.len; ++t) all.push_back({q.tokens[t], (int32_t)q.slot, t});
  int R = std::min(PREFILL_ROWS, c->p.Mcap);
  std::vector<int32_t> tok(R), slot(R), pos(R), act(R);
  std::vector<PrefillBlock> blocks;
  const int block_rows = ATT_PREFILL_WAVES * ATT_PREFILL_COLS / (c->d.n_q_heads / c->d.n_kv_heads);
  bool splitk = !env_flag("ECHO_ATTN_SIMPLE"), causal_blocks = c->p.fast && splitk;
  for (size_t a = 0; a < all.size(); a += R) {
    int M = (int)std::min<size_t>(R, all.size() - a);
    for (int i = 0; i < M; ++i) { tok[i] = all[a + i].token; slot[i] = all[a + i].slot; pos[i] = all[a + i].pos; act[i] = 1; }
    HIPCHK(c, hipMemcpyAsync(c->rows.token, tok.data(), M * 4, hipMemcpyHostToDevice, c->cs));
    HIPCHK(c, hipMemcpyAsync(c->rows.slot, slot.data(), M * 4, hipMemcpyHostToDevice, c->cs));
    HIPCHK(c, hipMemcpyAsync(c->rows.pos, pos.data(), M * 4, hipMemcpyHostToDevice, c->cs));
    HIPCHK(c, hipMemcpyAsync(c->rows.active, act.data(), M * 4, hipMemcpyHostToDevice, c->cs));
    launch_fill_i32(c->rows.ptiles, 0, M, c->cs);   // rows of a pass share no prefix tiles
    blocks.clear();
    if (causal_blocks) {   // runs of consecutive positions of one slot, cut every block_rows rows
      for (int i = 0; i < M; ++i) {
        bool extend = !blocks.empty() && blocks.back().nrows < block_rows && blocks.back().slot == slot[i] &&
                      blocks.back().pos0 + blocks.back().nrows == pos[i];
        if (extend) ++blocks.back().nrows; else blocks.push_back({i, 1, slot[i], pos[i]});
      }
      HIPCHK(c, hipMemcpyAsync(at<PrefillBlock>(c, c->p.o_blocks), blocks.data(), blocks.size() * sizeof(PrefillBlock),
                               hipMemcpyHostToDevice, c->cs));
    }
    HIPCHK(c, hipStreamSynchronize(c->cs));  // the host vectors are reused by the next chunk
    forward_layers(c, S, M, splitk, (int)blocks.size());
    int rc = after(&all[a], M);
    if (rc) return rc;
  }
  return 0;
}

template <typename F>
int run_chunks(echo_ctx *c, const Slot &S, const int32_t *tokens, int stride, const std::vector<int> &lens, int slot_step, F after) {
  std::vector<ChunkSeq> seqs;
  for (size_t q = 0; q < lens.size(); ++q) seqs.push_back({tokens + (int64_t)q * stride, lens[q], (int)(q * slot_step)});
  return run_chunk_seqs(c, S, seqs, after);
}

int capture_step(echo_ctx *c, const Slot &S, int N, int max_new, float temperature, uint64_t seed, bool unfused, const int32_t *forced,
                 int eos, float top_p, int per_row = 0) {
  if (c->graph) { hipGraphExecDestroy(c->graph); c->graph = nullptr; }
  hipGraph_t g = nullptr;
  HIPCHK(c, hipStreamBeginCapture(c->cs, hipStreamCaptureModeThreadLocal));
  forward_layers(c, S, N, !env_flag("ECHO_ATTN_SIMPLE"));
  sample_rows(c, S, N, temperature, seed, unfused, nullptr, top_p);
  launch_bookkeeping(N, max_new, per_row, c->d_step, c->d_samp_tok, c->d_samp_lp, forced, c->d_limit, eos, S.version, c->d_prompt_len_seq,
                     c->d_gen_len, c->rows, at<int32_t>(c, c->p.o_out_tok), at<float>(c, c->p.o_out_lp), at<int64_t>(c, c->p.o_out_ver),
                     c->d_n_active, c->cs);
  HIPCHK(c, hipStreamEndCapture(c->cs, &g));
  hipError_t e = hipGraphInstantiate(&c->graph, g, nullptr, nullptr, 0);
  hipGraphDestroy(g);
  if (e != hipSuccess) return fail(c, ECHO_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e));
  return 0;
}

double drain_events(std::vector<std::pair<hipEvent_t, hipEvent_t>> &v, int64_t *count) {
  double ms = 0;
  for (auto &pr : v) {
    float t = 0;
    if (hipEventElapsedTime(&t, pr.first, pr.second) == hipSuccess) { ms += t; ++*count; }
    hipEventDestroy(pr.first);
    hipEventDestroy(pr.second);
  }
  v.clear();
  return ms;
}

// Plans the shared-prompt attention of a decode batch of R rows.  Rows that read whole prompt tiles from a common cache slot
// (ptiles >= 1) and are still generating are grouped by that slot; every group of two or more is cut into jobs of up to
// 32 / grp rows, whose rows get ATT_PREFIX_DONE in ptiles (host copy: the caller uploads it).  max_ptiles fixes the chunking
// for the whole rollout and grid_jobs the launch's job count (unused job slots are empty), so a captured step stays valid
// when the list is rebuilt.  Leaves c->px.n_jobs = 0 when there is nothing to share or the decode kernel splits keys.
int plan_prefix_jobs(echo_ctx *c, std::vector<int32_t> &ptiles, const std::vector<int32_t> &pslot, const std::vector<int32_t> &live, int R,
                     int max_ptiles, int grid_jobs) {
  const int grp = c->d.n_q_heads / c->d.n_kv_heads, per_job = std::max(1, 32 / grp);
  const int cap = pad_rows(c->d.max_seqs) / 2 + 1;
  c->px = PrefixPlan{at<PrefixJob>(c, c->p.o_pjobs), 0, 0, 1};
  for (int r = 0; r < R; ++r) ptiles[r] &= ~ATT_PREFIX_DONE;
  if (!c->p.fast || max_ptiles < 1 || fast_attention_splits(R, c->d.n_kv_heads, c->p.attn_max_splits) != 1 || env_flag("ECHO_NO_PREFIX_KERNEL")) return 0;
  std::vector<PrefixJob> jobs;
  std::vector<int> order(R);
  for (int r = 0; r < R; ++r) order[r] = r;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return pslot[a] < pslot[b]; });
  for (int i = 0; i < R;) {
    int j = i;
    std::vector<int> members;
    while (j < R && pslot[order[j]] == pslot[order[i]]) {
      if (live[order[j]] && ptiles[order[j]] >= 1) members.push_back(order[j]);
      ++j;
    }
    if (members.size() >= 2) {
      for (size_t k = 0; k < members.size(); k += per_job) {
        size_t n = std::min<size_t>(per_job, members.size() - k);
        if (n < 2 && k > 0) break;   // a lone last row reads its prompt tiles itself
        PrefixJob jb;
        memset(&jb, 0, sizeof jb);
        jb.pslot = pslot[members[k]]; jb.ptiles = ptiles[members[k]]; jb.nrows = (int)n;
        for (size_t q = 0; q < n; ++q) { jb.rows[q] = members[k + q]; ptiles[members[k + q]] |= ATT_PREFIX_DONE; }
        jobs.push_back(jb);
      }
    }
    i = j;
  }
  // The extra launch costs more than it saves at 64 rows x 16 tiles (measured: -7 % there; +1 % at 256 x 16, -2 % at a
  // draining 128 x 32, +5 % at 256 x 32), so small batches with short prompts keep reading their shared tiles in the
  // decode kernel.
  int64_t covered = 0, min_covered = 6144;
  for (const PrefixJob &jb : jobs) covered += (int64_t)jb.nrows * jb.ptiles;
  if (const char *v = getenv("ECHO_PREFIX_KERNEL_MIN")) min_covered = atoll(v);
  if (jobs.empty() || (int)jobs.size() > cap || covered < min_covered) {
    for (int r = 0; r < R; ++r) ptiles[r] &= ~ATT_PREFIX_DONE;
    return 0;
  }
  int n_grid = std::max(grid_jobs, (int)jobs.size());
  if (n_grid > cap) n_grid = cap;
  PrefixJob empty;
  memset(&empty, 0, sizeof empty);
  jobs.resize(n_grid, empty);
  int est = grid_jobs > 0 ? std::max(1, R / per_job) : (int)jobs.size();
  int np = (256 + est * c->d.n_kv_heads - 1) / (est * c->d.n_kv_heads);
  np = std::max(1, std::min({np, c->p.attn_max_splits, max_ptiles}));
  int tpc = (max_ptiles + np - 1) / np;
  np = (max_ptiles + tpc - 1) / tpc;
  HIPCHK(c, hipMemcpyAsync(at<PrefixJob>(c, c->p.o_pjobs), jobs.data(), jobs.size() * sizeof(PrefixJob), hipMemcpyHostToDevice, c->cs));
  HIPCHK(c, hipStreamSynchronize(c->cs));   // the host list goes out of scope
  c->px = PrefixPlan{at<PrefixJob>(c, c->p.o_pjobs), n_grid, np, tpc};
  return 0;
}

// Argument checks shared by the two rollout entry points; o receives the options (defaults when opts is NULL).
int check_rollout_args(echo_ctx *c, const int32_t *prompt_tokens, int32_t prompt_stride, const int32_t *prompt_lens, int32_t P, int32_t G,
                       int32_t max_new, float temperature, const echo_rollout_opts *opts, const int32_t *out_tokens,
                       const float *out_logprobs, const int32_t *out_lens, echo_rollout_opts *o) {
  memset(o, 0, sizeof *o);
  o->eos_id = -1; o->top_p = 1.0f;
  if (opts) *o = *opts;
  if (!prompt_tokens || !prompt_lens || !out_tokens || !out_logprobs || !out_lens) return fail(c, ECHO_EINVAL, "NULL argument");
  if (P < 1 || G < 1 || max_new < 1 || prompt_stride < 1) return fail(c, ECHO_EINVAL, "n_prompts, G, max_new and prompt_stride must be positive");
  if (!(temperature > 0.f)) return fail(c, ECHO_EINVAL, "temperature must be positive");
  if (!(o->top_p > 0.f) || o->top_p > 1.0f) return fail(c, ECHO_EINVAL, "top_p must be in (0, 1]");
  if ((int64_t)P * G * max_new > INT32_MAX) return fail(c, ECHO_EINVAL, "n_prompts * G * max_new exceeds 2^31 - 1");
  int max_pl = 0;
  for (int p = 0; p < P; ++p) {
    if (prompt_lens[p] < 1 || prompt_lens[p] > prompt_stride) return fail(c, ECHO_EINVAL, "prompt_lens[%d] = %d out of range", p, prompt_lens[p]);
    max_pl = std::max(max_pl, prompt_lens[p]);
    for (int t = 0; t < prompt_lens[p]; ++t) {
      int tk = prompt_tokens[(int64_t)p * prompt_stride + t];
      if (tk < 0 || tk >= c->d.vocab) return fail(c, ECHO_EINVAL, "prompt token %d of prompt %d is outside the vocabulary", t, p);
    }
  }
  if ((int64_t)max_pl + max_new > c->d.max_ctx) return fail(c, ECHO_ENOMEM, "prompt %d + max_new %d exceeds max_ctx = %d", max_pl, max_new, c->d.max_ctx);
  if (o->forced_tokens)
    for (int64_t i = 0; i < (int64_t)P * G * max_new; ++i)
      if (o->forced_tokens[i] < 0 || o->forced_tokens[i] >= c->d.vocab) return fail(c, ECHO_EINVAL, "forced token outside the vocabulary");
  return ECHO_OK;
}

// Marks the context as running a rollout for the lifetime of the object; begin() fails when it cannot start.  When the
// rollout ends a staged snapshot becomes the active one and the samplers' draw ids return to their default.
struct RolloutGuard {
  echo_ctx *c;
  bool held = false;
  explicit RolloutGuard(echo_ctx *c_) : c(c_) {}
  int begin() {
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->active < 0) return fail(c, ECHO_ESTATE, "no policy snapshot installed");
    if (c->load.open && c->load.target == c->active) return fail(c, ECHO_ESTATE, "a snapshot is arriving in the only weight slot");
    if (c->rollout_running) return fail(c, ECHO_ESTATE, "a rollout is already running on this context");
    c->rollout_running = held = true;
    return ECHO_OK;
  }
  ~RolloutGuard() {
    if (!held) return;
    std::lock_guard<std::mutex> lk(c->mu);
    c->rollout_running = false;
    c->ids = DrawIds{c->d_step, nullptr, nullptr};
    c->px.n_jobs = 0;
    if (c->staged >= 0) { c->active = c->staged; c->staged = -1; c->st.active_version = c->slots[c->active].version; c->st.staged_version = -1; }
  }
};

}  // namespace

// =================================================================================================== C ABI
extern "C" {

size_t echo_arena_bytes(const echo_model_desc *desc) {
  Plan p = make_plan(desc);
  return p.ok ? p.total : 0;
}

size_t echo_blob_bytes(const echo_model_desc *desc) {
  if (!valid_desc(desc, nullptr)) return 0;
  return (size_t)blob_numel(desc) * (desc->dtype == ECHO_BF16 ? 2 : 4);
}

int echo_init(const echo_model_desc *desc, int device, void *dev_arena, size_t arena_bytes, void *compute_stream, void *copy_stream,
              echo_ctx **out) {
  if (!out) return fail(nullptr, ECHO_EINVAL, "out is NULL");
  *out = nullptr;
  std::string why;
  if (!valid_desc(desc, &why)) return fail(nullptr, ECHO_EINVAL, "invalid model description: %s", why.c_str());
  Plan p = make_plan(desc);
  if (!dev_arena || ((uintptr_t)dev_arena & 255)) return fail(nullptr, ECHO_EINVAL, "dev_arena must be a 256-byte aligned device pointer");
  if (arena_bytes < p.total) return fail(nullptr, ECHO_ENOMEM, "arena has %zu bytes, this shape needs %zu", arena_bytes, p.total);
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return fail(nullptr, ECHO_EHIP, "no HIP device %d", device);
  echo_ctx *c = new echo_ctx();
  c->d = *desc; c->p = p; c->device = device; c->arena = (char *)dev_arena;
  memset(&c->st, 0, sizeof c->st);
  c->st.active_version = c->st.staged_version = -1;
  auto bail = [&](const char *what, hipError_t e) { int rc = fail(nullptr, ECHO_EHIP, "%s: %s", what, hipGetErrorString(e)); delete c; return rc; };
  hipError_t e;
  if ((e = hipSetDevice(device)) != hipSuccess) return bail("hipSetDevice", e);
  // graph capture is not possible on the null stream, so it is replaced by a stream of the library's own
  c->cs = (hipStream_t)compute_stream; c->ks = (hipStream_t)copy_stream;
  if (!c->cs) { if ((e = hipStreamCreateWithFlags(&c->cs, hipStreamNonBlocking)) != hipSuccess) return bail("hipStreamCreate", e); c->own_cs = true; }
  if (!c->ks) { if ((e = hipStreamCreateWithFlags(&c->ks, hipStreamNonBlocking)) != hipSuccess) return bail("hipStreamCreate", e); c->own_ks = true; }
  if ((e = hipEventCreateWithFlags(&c->staged_ev, hipEventDisableTiming)) != hipSuccess) return bail("hipEventCreate", e);
  for (int s = 0; s < desc->n_weight_slots; ++s) bind_slot(c, s);
  int32_t *r = at<int32_t>(c, p.o_rows);
  size_t M = p.Mcap;
  c->rows = {r, r + M, r + 2 * M, r + 3 * M, r + 4 * M, r + 5 * M};
  c->kv = {c->arena + p.o_kv, desc->n_layers, desc->n_kv_heads, p.fast ? (int32_t)round_up(desc->max_ctx, 32) : desc->max_ctx, desc->head_dim,
           p.fast ? 2 : 4, p.fast ? 1 : 0};
  int32_t *q = at<int32_t>(c, p.o_seq);
  size_t Ms = pad_rows(desc->max_seqs);
  c->d_prompt_len_seq = q; c->d_gen_len = q + Ms; c->d_limit = q + 2 * Ms; c->d_stream = q + 3 * Ms;
  int32_t *sm = at<int32_t>(c, p.o_samp);
  c->d_samp_tok = sm; c->d_samp_lp = (float *)(sm + M); c->d_target = sm + 2 * M; c->d_target_lp = (float *)(sm + 3 * M);
  int32_t *mp = at<int32_t>(c, p.o_maps);
  c->d_map_a = mp; c->d_map_b = mp + M; c->d_plen_p = mp + 2 * M;
  c->d_step = at<int32_t>(c, p.o_scal); c->d_n_active = c->d_step + 1;
  c->ids = DrawIds{c->d_step, nullptr, nullptr};
  // activations, row state and scratch start from zero (padding rows and columns are never written); so does the
  // KV cache: the keys of a sequence's last tile that lie beyond its length get weight zero, which only cancels
  // a finite value
  size_t zero_from = p.o_kv;
  if ((e = hipMemsetAsync(c->arena + zero_from, 0, p.total - zero_from, c->cs)) != hipSuccess) return bail("hipMemsetAsync", e);
  if ((e = hipStreamSynchronize(c->cs)) != hipSuccess) return bail("hipStreamSynchronize", e);
  *out = c;
  return ECHO_OK;
}

int echo_load_policy_begin(echo_ctx *c, int64_t version, size_t nbytes) {
  if (!c) return ECHO_EINVAL;
  std::unique_lock<std::mutex> lk(c->mu);
  if (nbytes != echo_blob_bytes(&c->d)) return fail(c, ECHO_EINVAL, "blob has %zu bytes, this shape needs %zu", nbytes, echo_blob_bytes(&c->d));
  if (c->load.open) return fail(c, ECHO_ESTATE, "snapshot %lld is still arriving (commit or abort it first)", (long long)c->load.version);
  int64_t newest = c->newest_version;  // of the snapshots committed so far
  if (version <= newest || version < 0) return fail(c, ECHO_ESTATE, "version %lld does not advance past %lld", (long long)version, (long long)newest);
  if (c->staged >= 0) return fail(c, ECHO_ESTATE, "a staged snapshot is still waiting to be switched in");
  bool running = c->rollout_running;
  int target;
  if (c->active < 0) target = 0;
  else if (c->d.n_weight_slots == 2) target = 1 - c->active;
  else if (!running) target = c->active;
  else return fail(c, ECHO_ESTATE, "installing during a rollout needs n_weight_slots = 2");
  c->load.open = true;  // from here on a rollout cannot start on the target slot
  c->load.version = version; c->load.target = target; c->load.received = 0; c->load.total = nbytes;
  lk.unlock();
  auto undo = [&](int rc) { lk.lock(); c->load.open = false; if (target == c->active) { c->active = -1; c->st.active_version = -1; } return rc; };
  if (hipSetDevice(c->device) != hipSuccess) return undo(fail(c, ECHO_EHIP, "hipSetDevice failed"));
  if (!running && hipStreamSynchronize(c->cs) != hipSuccess) return undo(fail(c, ECHO_EHIP, "hipStreamSynchronize failed"));
  c->load.segs = blob_segments(c, target);
  // zero rows and columns of padding in the packed weights
  if (c->p.fast && hipMemsetAsync(c->slots[target].base, 0, c->p.slot_bytes, c->ks) != hipSuccess) return undo(fail(c, ECHO_EHIP, "hipMemsetAsync failed"));
  return ECHO_OK;
}

int echo_load_policy_chunk(echo_ctx *c, const void *data, size_t nbytes) {
  if (!c) return ECHO_EINVAL;
  {
    std::lock_guard<std::mutex> lk(c->mu);
    if (!c->load.open) return fail(c, ECHO_ESTATE, "no snapshot is being loaded");
    if (!data && nbytes) return fail(c, ECHO_EINVAL, "data is NULL");
    if (nbytes > c->load.total - c->load.received)
      return fail(c, ECHO_EINVAL, "%zu bytes after %zu overrun the blob of %zu", nbytes, c->load.received, c->load.total);
  }
  HIPCHK(c, hipSetDevice(c->device));
  int rc = feed_segments(c, c->load.segs, (const char *)data, c->load.received, nbytes);
  if (rc) return rc;
  HIPCHK(c, hipStreamSynchronize(c->ks));  // the piece may be freed when this call returns
  c->load.received += nbytes;
  return ECHO_OK;
}

int echo_load_policy_commit(echo_ctx *c) {
  if (!c) return ECHO_EINVAL;
  {
    std::lock_guard<std::mutex> lk(c->mu);
    if (!c->load.open) return fail(c, ECHO_ESTATE, "no snapshot is being loaded");
    if (c->load.received != c->load.total) return fail(c, ECHO_ESTATE, "%zu of %zu bytes have arrived", c->load.received, c->load.total);
  }
  HIPCHK(c, hipSetDevice(c->device));
  HIPCHK(c, hipEventRecord(c->staged_ev, c->ks));
  HIPCHK(c, hipStreamSynchronize(c->ks));
  std::lock_guard<std::mutex> lk(c->mu);
  int target = c->load.target;
  c->slots[target].version = c->load.version;
  c->newest_version = c->load.version;
  if (c->rollout_running) {
    c->staged = target;
    c->st.staged_version = c->load.version;
  } else {
    c->active = target;
    c->st.active_version = c->load.version;
  }
  c->load.open = false;
  c->load.segs.clear();
  c->cv.notify_all();
  return ECHO_OK;
}

int echo_load_policy_abort(echo_ctx *c) {
  if (!c) return ECHO_EINVAL;
  hipSetDevice(c->device);
  hipStreamSynchronize(c->ks);
  std::lock_guard<std::mutex> lk(c->mu);
  if (!c->load.open) return fail(c, ECHO_ESTATE, "no snapshot is being loaded");
  if (c->load.target == c->active) {  // the only slot now holds part of two snapshots
    c->active = -1;
    c->st.active_version = -1;
  }
  c->load.open = false;
  c->load.segs.clear();
  return ECHO_OK;
}

int echo_load_policy(echo_ctx *c, int64_t version, const void *host_weights, size_t nbytes) {
  if (!c) return ECHO_EINVAL;
  if (!host_weights) return fail(c, ECHO_EINVAL, "host_weights is NULL");
  int rc = echo_load_policy_begin(c, version, nbytes);
  if (rc) return rc;
  if ((rc = echo_load_policy_chunk(c, host_weights, nbytes)) || (rc = echo_load_policy_commit(c))) {
    std::string msg = c->err;
    echo_load_policy_abort(c);
    c->err = msg;
  }
  return rc;
}

int echo_rollout(echo_ctx *c, const int32_t *prompt_tokens, int32_t prompt_stride, const int32_t *prompt_lens, int32_t P, int32_t G,
                 int32_t max_new, float temperature, uint64_t seed, const echo_rollout_opts *opts, int32_t *out_tokens,
                 float *out_logprobs, int32_t *out_lens, int64_t *out_versions) {
  if (!c) return ECHO_EINVAL;
  echo_rollout_opts o;
  int rc = check_rollout_args(c, prompt_tokens, prompt_stride, prompt_lens, P, G, max_new, temperature, opts, out_tokens, out_logprobs,
                              out_lens, &o);
  if (rc) return rc;
  if ((int64_t)P * G > c->d.max_seqs) return fail(c, ECHO_ENOMEM, "%lld sequences exceed max_seqs = %d", (long long)P * G, c->d.max_seqs);
  const int N = P * G;
  if (o.n_swaps < 0 || (o.n_swaps > 0 && !o.swap_at_step)) return fail(c, ECHO_EINVAL, "bad swap schedule");
  for (int j = 0; j < o.n_swaps; ++j)
    if (o.swap_at_step[j] < 1 || (j && o.swap_at_step[j] <= o.swap_at_step[j - 1])) return fail(c, ECHO_EINVAL, "swap_at_step must be ascending and >= 1");
  if (o.n_swaps > 0 && c->d.n_weight_slots < 2) return fail(c, ECHO_ESTATE, "snapshot swaps inside a rollout need n_weight_slots = 2");
  RolloutGuard guard(c);
  if ((rc = guard.begin())) return rc;

  HIPCHK(c, hipSetDevice(c->device));
  const Plan &p = c->p;
  hipStream_t st = c->cs;
  auto t0 = std::chrono::steady_clock::now();
  bool unfused = o.unfused_sampler || o.debug_logits || o.top_p < 1.0f;   // the nucleus cut needs the whole row of logits
  bool want_timing = o.time_kernels != 0;
  c->timing = false;
  bool use_graph = !o.no_graph && !want_timing && !o.debug_logits;
  c->t_attn_bytes = c->t_gemm_bytes = 0;

  // per-sequence state
  std::vector<int32_t> plen_seq(N), limit(N);
  int steps = 0;
  for (int n = 0; n < N; ++n) {
    plen_seq[n] = prompt_lens[n / G];
    limit[n] = o.stop_lens ? std::max(1, std::min(max_new, o.stop_lens[n])) : max_new;
    steps = std::max(steps, limit[n]);
  }
  HIPCHK(c, hipMemcpyAsync(c->d_prompt_len_seq, plen_seq.data(), N * 4, hipMemcpyHostToDevice, st));
  HIPCHK(c, hipMemcpyAsync(c->d_limit, limit.data(), N * 4, hipMemcpyHostToDevice, st));
  HIPCHK(c, hipMemcpyAsync(c->d_plen_p, prompt_lens, P * 4, hipMemcpyHostToDevice, st));
  int32_t *d_forced = nullptr;
  if (o.forced_tokens) {
    d_forced = at<int32_t>(c, p.o_forced);
    HIPCHK(c, hipMemcpyAsync(d_forced, o.forced_tokens, (size_t)N * max_new * 4, hipMemcpyHostToDevice, st));
  }
  int64_t outn = (int64_t)N * max_new;
  launch_fill_i32(at<int32_t>(c, p.o_out_tok), -1, outn, st);
  launch_fill_i32(at<int32_t>(c, p.o_out_lp), 0, outn, st);
  launch_fill_i32(at<int32_t>(c, p.o_out_ver), -1, outn * 2, st);
  launch_fill_i32(c->d_gen_len, 0, N, st);
  launch_fill_i32(c->d_step, 0, 1, st);
  HIPCHK(c, hipStreamSynchronize(st));

  int cur = c->active;
  const bool share_prefix = p.fast && !env_flag("ECHO_NO_PREFIX_SHARING") && !env_flag("ECHO_ATTN_SIMPLE");
  // ---- prefill the P unique prompts into cache slots p*G, keep each prompt's last hidden state
  std::vector<int> lens(prompt_lens, prompt_lens + P);
  std::vector<int32_t> map(std::max(P, N));
  float *first_h = at<float>(c, p.o_first_h);
  rc = run_chunks(c, c->slots[cur], prompt_tokens, prompt_stride, lens, G, [&](const ChunkRow *rows, int M) -> int {
    std::fill(map.begin(), map.begin() + P, -1);
    bool any = false;
    for (int i = 0; i < M; ++i) {
      int pp = rows[i].slot / G;
      if (rows[i].pos == prompt_lens[pp] - 1) { map[pp] = i; any = true; }
    }
    if (!any) return 0;
    HIPCHK(c, hipMemcpyAsync(c->d_map_a, map.data(), P * 4, hipMemcpyHostToDevice, st));
    launch_gather_rows_f32(first_h, at<float>(c, p.o_h), c->d_map_a, P, c->d.hidden, st);
    HIPCHK(c, hipStreamSynchronize(st));
    return 0;
  });
  if (rc) return rc;
  // ---- first token of all N sequences from the shared prompt state; replicate the prompt K/V
  for (int n = 0; n < N; ++n) map[n] = n / G;
  HIPCHK(c, hipMemcpyAsync(c->d_map_a, map.data(), N * 4, hipMemcpyHostToDevice, st));
  launch_gather_rows_f32(at<float>(c, p.o_h), first_h, c->d_map_a, N, c->d.hidden, st);
  launch_fill_i32(c->rows.active, 1, N, st);
  for (int n = 0; n < N; ++n) map[n] = n;
  HIPCHK(c, hipMemcpyAsync(c->rows.slot, map.data(), N * 4, hipMemcpyHostToDevice, st));
  {   // decode attention reads the whole tiles of a group's prompt from the group's first slot
    std::vector<int32_t> pslot(N), ptiles(N), live(N, 1);
    int max_ptiles = 0;
    for (int n = 0; n < N; ++n) {
      pslot[n] = n / G * G;
      ptiles[n] = share_prefix ? prompt_lens[n / G] / 32 : 0;
      max_ptiles = std::max(max_ptiles, ptiles[n]);
    }
    if ((rc = plan_prefix_jobs(c, ptiles, pslot, live, N, max_ptiles, 0))) return rc;
    HIPCHK(c, hipMemcpyAsync(c->rows.pslot, pslot.data(), N * 4, hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(c->rows.ptiles, ptiles.data(), N * 4, hipMemcpyHostToDevice, st));
    HIPCHK(c, hipStreamSynchronize(st));   // the host vectors go out of scope
  }
  norm_only(c, c->slots[cur], N);
  sample_rows(c, c->slots[cur], N, temperature, seed, unfused, nullptr, o.top_p);
  auto grab_logits = [&](int s) -> int {
    if (!o.debug_logits) return 0;
    HIPCHK(c, hipMemcpy2DAsync(o.debug_logits + (int64_t)s * c->d.vocab, (size_t)max_new * c->d.vocab * 4, at<float>(c, p.o_logits),
                               (size_t)logits_ld(c) * 4, (size_t)c->d.vocab * 4, N, hipMemcpyDeviceToHost, st));
    HIPCHK(c, hipStreamSynchronize(st));
    return 0;
  };
  if ((rc = grab_logits(0))) return rc;
  auto book = [&](int slot) {
    launch_bookkeeping(N, max_new, 0, c->d_step, c->d_samp_tok, c->d_samp_lp, d_forced, c->d_limit, o.eos_id, c->slots[slot].version,
                       c->d_prompt_len_seq, c->d_gen_len, c->rows, at<int32_t>(c, p.o_out_tok), at<float>(c, p.o_out_lp),
                       at<int64_t>(c, p.o_out_ver), c->d_n_active, st);
  };
  book(cur);
  launch_kv_replicate(c->kv, c->d_plen_p, P, G, st);
  HIPCHK(c, hipStreamSynchronize(st));
  auto t1 = std::chrono::steady_clock::now();

  // ---- decode
  c->timing = want_timing;
  double swap_wait = 0;
  int next_swap = 0, decode_steps = 0;
  bool have_graph = false;
  bool splitk = !env_flag("ECHO_ATTN_SIMPLE");
  for (int s = 1; s < steps; ++s) {
    if (next_swap < o.n_swaps && o.swap_at_step[next_swap] == s) {
      auto w0 = std::chrono::steady_clock::now();
      std::unique_lock<std::mutex> lk(c->mu);
      int tmo = o.swap_timeout_ms > 0 ? o.swap_timeout_ms : 10000;
      if (!c->cv.wait_for(lk, std::chrono::milliseconds(tmo), [&] { return c->staged >= 0; }))
        return fail(c, ECHO_ESTATE, "no snapshot was staged for the swap at step %d within %d ms", s, tmo);
      cur = c->staged; c->active = cur; c->staged = -1;
      c->st.active_version = c->slots[cur].version; c->st.staged_version = -1;
      lk.unlock();
      HIPCHK(c, hipStreamWaitEvent(st, c->staged_ev, 0));
      swap_wait += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - w0).count();
      have_graph = false;
      ++next_swap;
    }
    if (o.eos_id >= 0 && (s % 16) == 0) {  // sequences may have ended early: look at the active count
      int32_t na = 0;
      HIPCHK(c, hipMemcpyAsync(&na, c->d_n_active, 4, hipMemcpyDeviceToHost, st));
      HIPCHK(c, hipStreamSynchronize(st));
      if (na == 0) break;
    }
    bool time_this = c->timing;
    if (c->timing) {
      c->timing = (s % 16) == 1;
      // K/V bytes one launch of the decode attention kernel has to read: the rest of every active sequence, and (when it
      // reads them itself) a group's whole prompt tiles once
      double keys = 0;
      for (int g0 = 0; g0 < N; g0 += G) {
        int shared = share_prefix ? plen_seq[g0] / 32 * 32 : 0;
        bool any = false;
        for (int n = g0; n < g0 + G; ++n) if (s < limit[n]) { keys += plen_seq[n] - shared + s; any = true; }
        if (any && c->px.n_jobs == 0) keys += shared;   // with the prefix kernel the shared tiles are not this kernel's to read
      }
      c->cur_attn_bytes = keys * 2 * c->d.n_kv_heads * c->d.head_dim * 2;
    }
    if (use_graph) {
      if (!have_graph) {
        if ((rc = capture_step(c, c->slots[cur], N, max_new, temperature, seed, unfused, d_forced, o.eos_id, o.top_p))) return rc;
        have_graph = true;
      }
      HIPCHK(c, hipGraphLaunch(c->graph, st));
    } else {
      forward_layers(c, c->slots[cur], N, splitk);
      sample_rows(c, c->slots[cur], N, temperature, seed, unfused, nullptr, o.top_p);
      if ((rc = grab_logits(s))) return rc;
      book(cur);
    }
    c->timing = time_this;
    ++decode_steps;
  }
  HIPCHK(c, hipStreamSynchronize(st));
  auto t2 = std::chrono::steady_clock::now();

  // ---- results
  HIPCHK(c, hipMemcpyAsync(out_tokens, at<int32_t>(c, p.o_out_tok), outn * 4, hipMemcpyDeviceToHost, st));
  HIPCHK(c, hipMemcpyAsync(out_logprobs, at<float>(c, p.o_out_lp), outn * 4, hipMemcpyDeviceToHost, st));
  if (out_versions) HIPCHK(c, hipMemcpyAsync(out_versions, at<int64_t>(c, p.o_out_ver), outn * 8, hipMemcpyDeviceToHost, st));
  HIPCHK(c, hipMemcpyAsync(out_lens, c->d_gen_len, N * 4, hipMemcpyDeviceToHost, st));
  HIPCHK(c, hipStreamSynchronize(st));
  auto t3 = std::chrono::steady_clock::now();
  c->st.decode_steps = decode_steps;
  c->st.prefill_ms = std::chrono::duration<float, std::milli>(t1 - t0).count();
  c->st.decode_ms = std::chrono::duration<float, std::milli>(t2 - t1).count();
  c->st.total_ms = std::chrono::duration<float, std::milli>(t3 - t0).count();
  c->st.swap_wait_ms = (float)swap_wait;
  if (c->timing) {
    c->st.attn_launches = c->st.gemm_launches = 0;
    c->st.attn_ms = drain_events(c->ev_attn, &c->st.attn_launches);
    c->st.gemm_ms = drain_events(c->ev_gemm, &c->st.gemm_launches);
    c->st.attn_bytes = c->t_attn_bytes;
    c->st.gemm_bytes = c->t_gemm_bytes;
    c->timing = false;
  }
  return ECHO_OK;
}

int echo_rollout_continuous(echo_ctx *c, const int32_t *prompt_tokens, int32_t prompt_stride, const int32_t *prompt_lens, int32_t P,
                            int32_t G, int32_t max_new, float temperature, uint64_t seed, const echo_rollout_opts *opts,
                            int32_t *out_tokens, float *out_logprobs, int32_t *out_lens, int64_t *out_versions) {
  if (!c) return ECHO_EINVAL;
  echo_rollout_opts o;
  int rc = check_rollout_args(c, prompt_tokens, prompt_stride, prompt_lens, P, G, max_new, temperature, opts, out_tokens, out_logprobs,
                              out_lens, &o);
  if (rc) return rc;
  if (o.n_swaps || o.debug_logits || o.time_kernels)
    return fail(c, ECHO_EINVAL, "a continuous rollout takes no pinned swaps (it switches when a snapshot is staged), no debug_logits and no time_kernels");
  if (G > c->d.max_seqs) return fail(c, ECHO_ENOMEM, "one group of %d sequences exceeds max_seqs = %d", G, c->d.max_seqs);
  const int N = P * G;
  int max_pl = 0;
  for (int p = 0; p < P; ++p) max_pl = std::max(max_pl, prompt_lens[p]);
  RolloutGuard guard(c);
  if ((rc = guard.begin())) return rc;

  HIPCHK(c, hipSetDevice(c->device));
  const Plan &p = c->p;
  hipStream_t st = c->cs;
  auto t0 = std::chrono::steady_clock::now();
  const bool unfused = o.unfused_sampler || o.top_p < 1.0f;
  const bool use_graph = !o.no_graph;
  const bool share_prefix = p.fast && !env_flag("ECHO_NO_PREFIX_SHARING") && !env_flag("ECHO_ATTN_SIMPLE");
  const bool splitk = !env_flag("ECHO_ATTN_SIMPLE");
  const int R = std::min(N, c->d.max_seqs);   // cache slots in use; rows of the batch until the rows are compacted
  int Rc = R;                                 // rows of the batch now
  // host mirrors of the per-row state; token, pos, active and gen are read back at every check
  std::vector<int32_t> tok(R, 0), pos(R, 0), act(R, 0), slot(R), pslot(R, 0), ptiles(R, 0), plen(R, 1), gen(R, 0), lim(R, 1), stream(R, 0);
  std::vector<int> row_seq(R, -1);      // the sequence a row is generating, -1: none
  std::vector<int> row_holds(R, -1);    // the prompt whose shared key tiles live in this row's cache slot, -1: none
  std::vector<int> group_left(P, 0);    // sequences of a prompt that have not ended yet
  for (int r = 0; r < R; ++r) slot[r] = r;
  int32_t *d_forced = o.forced_tokens ? at<int32_t>(c, p.o_forced) : nullptr;
  int32_t *d_out_tok = at<int32_t>(c, p.o_out_tok);
  float *d_out_lp = at<float>(c, p.o_out_lp);
  int64_t *d_out_ver = at<int64_t>(c, p.o_out_ver);
  auto upload_rows = [&]() -> int {
    struct { int32_t *dst; std::vector<int32_t> *src; } cp[] = {
        {c->rows.token, &tok}, {c->rows.pos, &pos}, {c->rows.active, &act}, {c->rows.slot, &slot}, {c->rows.pslot, &pslot},
        {c->rows.ptiles, &ptiles}, {c->d_prompt_len_seq, &plen}, {c->d_gen_len, &gen}, {c->d_limit, &lim}, {c->d_stream, &stream}};
    for (auto &x : cp) HIPCHK(c, hipMemcpyAsync(x.dst, x.src->data(), (size_t)R * 4, hipMemcpyHostToDevice, st));   // R: also the rows given up
    return 0;
  };
  auto limit_of = [&](int n) { return o.stop_lens ? std::max(1, std::min(max_new, o.stop_lens[n])) : max_new; };
  launch_fill_i32(c->d_step, 0, 1, st);
  c->ids = DrawIds{c->d_step, c->d_gen_len, c->d_stream};

  int cur = c->active, next_prompt = 0, done_seqs = 0, decode_steps = 0, until_check = 0;
  bool have_graph = false, first = true, dirty = false;
  double admit_ms = 0, swap_wait = 0;
  std::vector<int> free_rows;
  std::vector<int32_t> quads;
  const int max_quads = 2 * c->p.Mcap / 4;   // the two row maps serve as the copy list
  for (;;) {
    if (until_check <= 0) {
      if (!first) {
        HIPCHK(c, hipMemcpyAsync(tok.data(), c->rows.token, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(c, hipMemcpyAsync(pos.data(), c->rows.pos, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(c, hipMemcpyAsync(act.data(), c->rows.active, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(c, hipMemcpyAsync(gen.data(), c->d_gen_len, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(c, hipStreamSynchronize(st));
      }
      first = false;
      // a sequence that has ended hands its record over
      for (int r = 0; r < Rc; ++r) {
        int n = row_seq[r];
        if (n < 0 || act[r]) continue;
        int64_t r0 = (int64_t)slot[r] * max_new, n0 = (int64_t)n * max_new;
        HIPCHK(c, hipMemcpyAsync(out_tokens + n0, d_out_tok + r0, (size_t)max_new * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(c, hipMemcpyAsync(out_logprobs + n0, d_out_lp + r0, (size_t)max_new * 4, hipMemcpyDeviceToHost, st));
        if (out_versions) HIPCHK(c, hipMemcpyAsync(out_versions + n0, d_out_ver + r0, (size_t)max_new * 8, hipMemcpyDeviceToHost, st));
        out_lens[n] = gen[r];
        row_seq[r] = -1;
        --group_left[n / G];
        ++done_seqs;
      }
      if (done_seqs == N) break;
      // its row is free again, unless the cache slot still holds the prompt tiles that running siblings read
      free_rows.clear();
      for (int r = 0; r < Rc && next_prompt < P; ++r) {
        if (row_seq[r] >= 0) continue;
        if (row_holds[r] >= 0 && group_left[row_holds[r]] > 0) continue;
        row_holds[r] = -1;
        free_rows.push_back(r);
      }
      // waiting prompts take G free rows each
      struct Admit { int prompt; std::vector<int> rows; };
      std::vector<Admit> admitted;
      while (next_prompt < P && (int)free_rows.size() >= G) {
        Admit ad{next_prompt++, {}};
        ad.rows.assign(free_rows.end() - G, free_rows.end());
        free_rows.resize(free_rows.size() - G);
        admitted.push_back(ad);
      }
      if (!admitted.empty()) {
        auto a0 = std::chrono::steady_clock::now();
        // All of a prompt but its last token goes through the causal-block pass into one of the group's cache slots
        // (the holder); the last token is every member's first decode input, so the first sampled token comes out of
        // an ordinary step.  The holder is the member that will run longest when that is known (stop lengths only).
        std::vector<ChunkSeq> seqs;
        quads.clear();
        for (Admit &ad : admitted) {
          int pp = ad.prompt, L = prompt_lens[pp], hold = 0;
          for (int g = 1; g < G; ++g) if (limit_of(pp * G + g) > limit_of(pp * G + hold)) hold = g;
          std::swap(ad.rows[0], ad.rows[hold]);   // member `hold` gets rows[hold], which now is the holder row
          int hr = ad.rows[hold];
          if (L > 1) seqs.push_back({prompt_tokens + (int64_t)pp * prompt_stride, L - 1, hr});
          int shared = share_prefix ? (L - 1) / 32 : 0;
          int begin = c->kv.tiled ? shared : 0, end = c->kv.tiled ? (L - 1 + 31) / 32 : L - 1;
          for (int g = 0; g < G; ++g) {
            int r = ad.rows[g], n = pp * G + g;
            if (r != hr && end > begin) { quads.push_back(hr); quads.push_back(r); quads.push_back(begin); quads.push_back(end); }
            tok[r] = prompt_tokens[(int64_t)pp * prompt_stride + L - 1];
            pos[r] = L - 1; act[r] = 1; pslot[r] = hr; ptiles[r] = shared;
            plen[r] = L; gen[r] = 0; stream[r] = n; lim[r] = limit_of(n);
            row_seq[r] = n;
          }
          row_holds[hr] = pp;
          group_left[pp] = G;
        }
        if (!seqs.empty() && (rc = run_chunk_seqs(c, c->slots[cur], seqs, [&](const ChunkRow *, int) { return 0; }))) return rc;
        for (size_t q0 = 0; q0 < quads.size() / 4; q0 += max_quads) {
          int nq = (int)std::min<size_t>(max_quads, quads.size() / 4 - q0);
          HIPCHK(c, hipMemcpyAsync(c->d_map_a, quads.data() + 4 * q0, (size_t)nq * 16, hipMemcpyHostToDevice, st));
          launch_kv_copy_ranges(c->kv, c->d_map_a, nq, st);
          HIPCHK(c, hipStreamSynchronize(st));   // the list is rewritten by the next round
        }
        for (Admit &ad : admitted)
          for (int g = 0; g < G; ++g) {
            int64_t r0 = (int64_t)slot[ad.rows[g]] * max_new;
            launch_fill_i32(d_out_tok + r0, -1, max_new, st);
            launch_fill_i32((int32_t *)(d_out_lp + r0), 0, max_new, st);
            launch_fill_i32((int32_t *)(d_out_ver + r0), -1, (int64_t)max_new * 2, st);
            if (d_forced)
              HIPCHK(c, hipMemcpyAsync(d_forced + r0, o.forced_tokens + (int64_t)(ad.prompt * G + g) * max_new, (size_t)max_new * 4,
                                       hipMemcpyHostToDevice, st));
          }
        dirty = true;   // the upload below also restores the rows the prefill pass used as its own
        admit_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - a0).count();
      }
      // No prompt is waiting any more: once the live rows fit a smaller padded batch they are moved to the front (their
      // cache slots and records stay where they are) and the step is captured again for fewer rows.
      if (next_prompt == P) {
        int live = 0;
        for (int r = 0; r < Rc; ++r) live += row_seq[r] >= 0;
        if (live > 0 && pad_rows(live) < pad_rows(Rc)) {
          int w = 0;
          for (int r = 0; r < Rc; ++r) {
            if (row_seq[r] < 0) continue;
            tok[w] = tok[r]; pos[w] = pos[r]; act[w] = act[r]; slot[w] = slot[r]; pslot[w] = pslot[r]; ptiles[w] = ptiles[r];
            plen[w] = plen[r]; gen[w] = gen[r]; lim[w] = lim[r]; stream[w] = stream[r]; row_seq[w] = row_seq[r];
            ++w;
          }
          for (int r = w; r < Rc; ++r) { act[r] = 0; row_seq[r] = -1; }
          Rc = w;
          dirty = true;
          have_graph = false;
        }
      }
      if (dirty) {   // the rows changed: plan the shared-prompt attention for them, then put the row state on the device
        std::vector<int32_t> live(R, 0);
        for (int r = 0; r < Rc; ++r) live[r] = row_seq[r] >= 0 && act[r];
        const PrefixPlan was = c->px;
        if ((rc = plan_prefix_jobs(c, ptiles, pslot, live, Rc, share_prefix ? (max_pl - 1) / 32 : 0, Rc / 2 + 1))) return rc;
        if (was.n_jobs != c->px.n_jobs || was.np != c->px.np || was.tiles_per_chunk != c->px.tiles_per_chunk) have_graph = false;
        if ((rc = upload_rows())) return rc;
        HIPCHK(c, hipStreamSynchronize(st));
        dirty = false;
      }
      // the next event: with stop lengths only, the step at which the next sequence ends is known
      until_check = 8;
      if (o.eos_id < 0) {
        int soonest = INT32_MAX;
        for (int r = 0; r < Rc; ++r)
          if (row_seq[r] >= 0 && act[r]) soonest = std::min(soonest, std::max(lim[r] - gen[r], 1));
        until_check = soonest;
      }
    }
    {   // a snapshot that has been staged meanwhile is switched in between two steps
      std::unique_lock<std::mutex> lk(c->mu);
      if (c->staged >= 0) {
        auto w0 = std::chrono::steady_clock::now();
        cur = c->staged; c->active = cur; c->staged = -1;
        c->st.active_version = c->slots[cur].version; c->st.staged_version = -1;
        lk.unlock();
        HIPCHK(c, hipStreamWaitEvent(st, c->staged_ev, 0));
        swap_wait += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - w0).count();
        have_graph = false;
      }
    }
    if (use_graph) {
      if (!have_graph) {
        if ((rc = capture_step(c, c->slots[cur], Rc, max_new, temperature, seed, unfused, d_forced, o.eos_id, o.top_p, 1))) return rc;
        have_graph = true;
      }
      HIPCHK(c, hipGraphLaunch(c->graph, st));
    } else {
      forward_layers(c, c->slots[cur], Rc, splitk);
      sample_rows(c, c->slots[cur], Rc, temperature, seed, unfused, nullptr, o.top_p);
      launch_bookkeeping(Rc, max_new, 1, c->d_step, c->d_samp_tok, c->d_samp_lp, d_forced, c->d_limit, o.eos_id, c->slots[cur].version,
                         c->d_prompt_len_seq, c->d_gen_len, c->rows, d_out_tok, d_out_lp, d_out_ver, c->d_n_active, st);
    }
    ++decode_steps;
    --until_check;
  }
  HIPCHK(c, hipStreamSynchronize(st));
  auto t1 = std::chrono::steady_clock::now();
  c->st.decode_steps = decode_steps;
  c->st.prefill_ms = (float)admit_ms;
  c->st.total_ms = std::chrono::duration<float, std::milli>(t1 - t0).count();
  c->st.decode_ms = c->st.total_ms - (float)admit_ms;
  c->st.swap_wait_ms = (float)swap_wait;
  return ECHO_OK;
}

int echo_logprobs(echo_ctx *c, const int32_t *tokens, int32_t stride, const int32_t *lens_in, int32_t n_seqs, float temperature,
                  float *out) {
  if (!c) return ECHO_EINVAL;
  if (!tokens || !lens_in || !out || n_seqs < 1 || stride < 1) return fail(c, ECHO_EINVAL, "bad argument");
  if (!(temperature > 0.f)) return fail(c, ECHO_EINVAL, "temperature must be positive");
  if (n_seqs > c->d.max_seqs) return fail(c, ECHO_ENOMEM, "%d sequences exceed max_seqs = %d", n_seqs, c->d.max_seqs);
  std::vector<int> lens(n_seqs);
  for (int n = 0; n < n_seqs; ++n) {
    if (lens_in[n] < 1 || lens_in[n] > stride || lens_in[n] > c->d.max_ctx) return fail(c, ECHO_ENOMEM, "lens[%d] = %d out of range", n, lens_in[n]);
    lens[n] = lens_in[n] - 1;  // the last token is only a target
    for (int t = 0; t < lens_in[n]; ++t) {
      int tk = tokens[(int64_t)n * stride + t];
      if (tk < 0 || tk >= c->d.vocab) return fail(c, ECHO_EINVAL, "token %d of sequence %d is outside the vocabulary", t, n);
    }
  }
  {
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->active < 0) return fail(c, ECHO_ESTATE, "no policy snapshot installed");
    if (c->load.open && c->load.target == c->active) return fail(c, ECHO_ESTATE, "a snapshot is arriving in the only weight slot");
    if (c->rollout_running) return fail(c, ECHO_ESTATE, "a rollout is running on this context");
  }
  HIPCHK(c, hipSetDevice(c->device));
  memset(out, 0, (size_t)n_seqs * stride * sizeof(float));
  hipStream_t st = c->cs;
  launch_fill_i32(c->d_step, 0, 1, st);
  std::vector<int32_t> tgt(c->p.Mcap);
  std::vector<float> lp(c->p.Mcap);
  const Slot &S = c->slots[c->active];
  return run_chunks(c, S, tokens, stride, lens, 1, [&](const ChunkRow *rows, int M) -> int {
    for (int i = 0; i < M; ++i) tgt[i] = tokens[(int64_t)rows[i].slot * stride + rows[i].pos + 1];
    HIPCHK(c, hipMemcpyAsync(c->d_target, tgt.data(), M * 4, hipMemcpyHostToDevice, st));
    sample_rows(c, S, M, temperature, 0, false, c->d_target);
    HIPCHK(c, hipMemcpyAsync(lp.data(), c->d_target_lp, M * 4, hipMemcpyDeviceToHost, st));
    HIPCHK(c, hipStreamSynchronize(st));
    for (int i = 0; i < M; ++i) out[(int64_t)rows[i].slot * stride + rows[i].pos + 1] = lp[i];
    return 0;
  });
}

int echo_grpo_tensors(echo_ctx *c, const int32_t *tokens, int32_t stride, const int32_t *lens, int32_t n_seqs, int32_t G,
                      int32_t turn_start_id, const float *rewards, float eps, uint8_t *out_mask, float *out_adv, float *out_adv_tok) {
  if (!c) return ECHO_EINVAL;
  if (!tokens || !lens || !rewards || !out_mask || !out_adv || stride < 1) return fail(c, ECHO_EINVAL, "bad argument");
  if (G < 2) return fail(c, ECHO_EINVAL, "a group needs at least 2 samples for a standard deviation (G = %d)", G);
  if (n_seqs < G || n_seqs % G) return fail(c, ECHO_EINVAL, "n_seqs = %d is not a positive multiple of G = %d", n_seqs, G);
  if (!(eps >= 0.f)) return fail(c, ECHO_EINVAL, "eps must be >= 0");
  for (int n = 0; n < n_seqs; ++n)
    if (lens[n] < 0 || lens[n] > stride) return fail(c, ECHO_EINVAL, "lens[%d] = %d outside 0..%d", n, lens[n], stride);
  {
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->rollout_running) return fail(c, ECHO_ESTATE, "a rollout is running on this context");
  }
  // The logits buffer is borrowed as staging, whole groups at a time:
  // tokens i32 [ns, stride] | adv_tok f32 [ns, stride] | mask u8 [ns, stride] | lens i32 [ns] | rewards f32 [ns] | adv f32 [ns]
  auto up16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
  size_t cap = c->p.logit_rows * (size_t)c->p.Np_v * 4;
  auto need = [&](size_t ns) { return 2 * up16(ns * stride * 4) + up16(ns * stride) + 3 * up16(ns * 4); };
  if (need(G) > cap) return fail(c, ECHO_ENOMEM, "one group (%d x %d tokens) needs %zu bytes of staging, the context has %zu", G, stride, need(G), cap);
  size_t groups_per_pass = 1;
  while (need((groups_per_pass * 2) * G) <= cap && groups_per_pass * G < (size_t)n_seqs) groups_per_pass *= 2;
  HIPCHK(c, hipSetDevice(c->device));
  hipStream_t st = c->cs;
  char *base = at<char>(c, c->p.o_logits);
  for (int n0 = 0; n0 < n_seqs; n0 += (int)(groups_per_pass * G)) {
    size_t ns = std::min<size_t>(groups_per_pass * G, n_seqs - n0);
    size_t cells = ns * stride;
    int32_t *d_tok = (int32_t *)base;
    float *d_at = (float *)(base + up16(cells * 4));
    uint8_t *d_mask = (uint8_t *)(base + 2 * up16(cells * 4));
    int32_t *d_len = (int32_t *)((char *)d_mask + up16(cells));
    float *d_rew = (float *)((char *)d_len + up16(ns * 4));
    float *d_adv = (float *)((char *)d_rew + up16(ns * 4));
    HIPCHK(c, hipMemcpyAsync(d_tok, tokens + (int64_t)n0 * stride, cells * 4, hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(d_len, lens + n0, ns * 4, hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(d_rew, rewards + n0, ns * 4, hipMemcpyHostToDevice, st));
    launch_grpo_tensors(d_mask, d_adv, out_adv_tok ? d_at : nullptr, d_tok, d_len, d_rew, (int)ns, G, stride, turn_start_id, eps, st);
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipMemcpyAsync(out_mask + (int64_t)n0 * stride, d_mask, cells, hipMemcpyDeviceToHost, st));
    HIPCHK(c, hipMemcpyAsync(out_adv + n0, d_adv, ns * 4, hipMemcpyDeviceToHost, st));
    if (out_adv_tok) HIPCHK(c, hipMemcpyAsync(out_adv_tok + (int64_t)n0 * stride, d_at, cells * 4, hipMemcpyDeviceToHost, st));
    HIPCHK(c, hipStreamSynchronize(st));
  }
  return ECHO_OK;
}

int echo_debug_draw_bits(echo_ctx *c, uint64_t seed, uint32_t n, uint32_t s, uint32_t i0, int32_t count, uint32_t *out_bits) {
  if (!c || !out_bits || count < 1) return c ? fail(c, ECHO_EINVAL, "bad argument") : ECHO_EINVAL;
  size_t cap = c->p.logit_rows * (size_t)c->p.Np_v;  // the logits buffer is borrowed as scratch
  if ((size_t)count > cap) return fail(c, ECHO_EINVAL, "count exceeds %zu", cap);
  {
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->rollout_running) return fail(c, ECHO_ESTATE, "a rollout is running on this context");
  }
  HIPCHK(c, hipSetDevice(c->device));
  uint32_t *buf = at<uint32_t>(c, c->p.o_logits);
  launch_draw_bits(buf, seed, n, s, i0, count, c->cs);
  HIPCHK(c, hipMemcpyAsync(out_bits, buf, (size_t)count * 4, hipMemcpyDeviceToHost, c->cs));
  HIPCHK(c, hipStreamSynchronize(c->cs));
  return ECHO_OK;
}

int echo_stats(echo_ctx *c, echo_stats_t *out) {
  if (!c || !out) return ECHO_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  *out = c->st;
  out->rollout_running = c->rollout_running ? 1 : 0;
  return ECHO_OK;
}

const char *echo_last_error(const echo_ctx *c) { return c ? c->err.c_str() : g_init_error.c_str(); }

void echo_destroy(echo_ctx *c) {
  if (!c) return;
  hipSetDevice(c->device);
  hipStreamSynchronize(c->cs);
  hipStreamSynchronize(c->ks);
  if (c->graph) hipGraphExecDestroy(c->graph);
  if (c->staged_ev) hipEventDestroy(c->staged_ev);
  if (c->own_cs) hipStreamDestroy(c->cs);
  if (c->own_ks) hipStreamDestroy(c->ks);
  delete c;
}

}  // extern "C"
