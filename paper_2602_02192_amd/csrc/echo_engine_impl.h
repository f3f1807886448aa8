// Internals of the host engine, shared by its translation units (echo_engine.hip: planning, context, scoring;
// echo_install.hip: snapshot install; echo_rollout.hip: the two rollout entry points): the arena plan, the context,
// the forward pass over a batch of rows and the pass driver for token strings.  Everything here has internal
// linkage; each translation unit compiles the helpers it uses.
#pragma once
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
  size_t o_attn_o, o_attn_ml, o_topp, o_pjobs, o_aplan;
  size_t o_blocks, o_rows, o_seq, o_samp, o_out_tok, o_out_lp, o_out_ver, o_forced, o_scal, o_first_h, o_stage, o_maps, o_qscales;
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
    p.o_qscales = b.take((size_t)std::max<int64_t>({V, Q + 2 * KV, 2 * F, H}) * 4);   // the row scales of the matrix a quantised load is in
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
  p.o_aplan = b.take(fast_attention_plan_ints(pad_rows(d->max_seqs)) * 4);   // tile lists of the several-rows decode attention
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
  // a quantised blob (echo_load_policy_q8_begin): where its byte stream stands
  bool q8 = false;
  std::vector<std::pair<int64_t, int64_t>> tensors;   // (rows, K) in blob order, rows == 0: a vector
  size_t ti = 0, tb = 0, bf_off = 0;                  // tensor, byte inside its quantised form, its start in the bf16 blob
  std::vector<char> carry;                            // a vector or a row of codes cut by the end of a piece
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
  hipEvent_t vacated_ev[2] = {nullptr, nullptr};   // recorded on the compute stream behind the last launch that reads a slot a rollout has left
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
  std::vector<hipGraphExec_t> retired_graphs;   // replaced while replays of them may still be queued; destroyed once the stream is idle
  // kernel timing (time_kernels)
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_attn, ev_gemm;
  bool timing = false;
  std::vector<float> step_ms;   // per-step durations of the last rollout run with time_steps
  bool attn_plain = false;   // cross-check switch of the running rollout (echo_rollout_opts.attn_plain)
  int attn_mode = 0;         // echo_rollout_opts.prefix_kernel of the running rollout
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

// The rollout stops using weight slot `s` (call with c->mu held, outside stream capture): decode steps that read the slot
// may still be queued on the compute stream, so whatever the copy stream does from now on -- the next install writes
// into this slot -- starts behind them.  The wait is placed here, by the rollout's thread, and not by the installing
// thread: the runtime refuses a cross-stream wait on an event of a stream that is capturing at that moment, and the
// rollout captures its next step graph right after a switch.
hipError_t leave_slot(echo_ctx *c, int s) {
  hipError_t e = hipEventRecord(c->vacated_ev[s], c->cs);
  if (e == hipSuccess) e = hipStreamWaitEvent(c->ks, c->vacated_ev[s], 0);
  return e;
}

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
  if (g.lds == 3 || g.lds == 2) g.nsplit = fast_gemm_even_split(Kp, g.nsplit);
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
  // decode attention over several rows per workgroup: the tile lists are the same for every layer
  const int att_rows = n_prefill_blocks == 0 && use_splitk_attn && c->px.n_jobs == 0 ? fast_attention_rows_per_group(M, Hq, Hkv, c->attn_mode) : 1;
  if (n_prefill_blocks == 0 && use_splitk_attn) { c->st.attn_rows_per_workgroup = att_rows; c->st.attn_prefix_jobs = c->px.n_jobs; }
  if (att_rows > 1) fast_attention_rows_plan(at<int32_t>(c, p.o_aplan), c->rows, M, Hq, Hkv, c->attn_mode, st);
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
      else if (att_rows > 1)
        fast_attention_rows(xatt, q16, at<int32_t>(c, p.o_aplan), c->rows, c->kv, l, M, Mp, Hq, Hkv, c->attn_mode, st);
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
  bool splitk = !c->attn_plain, causal_blocks = c->p.fast && splitk;
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

}  // namespace
