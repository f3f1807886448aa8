// Host engine behind the C ABI: arena planning, context set-up and tear-down, teacher-forced scoring, the learner-side
// tensors, statistics.  (Snapshot install: echo_install.hip; rollouts: echo_rollout.hip.)
#include "echo_engine_impl.h"

int echo_static_scratch_resolve(int device);   // echo_noalloc.hip: looks up this GPU's copy of the library's static scratch

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
  for (int s = 0; s < 2; ++s)
    if ((e = hipEventCreateWithFlags(&c->vacated_ev[s], hipEventDisableTiming)) != hipSuccess) return bail("hipEventCreate", e);
  if (int se = echo_static_scratch_resolve(device)) return bail("hipGetSymbolAddress(static scratch)", (hipError_t)se);
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

int echo_step_times(echo_ctx *c, float *out_ms, int32_t cap) {
  if (!c) return ECHO_EINVAL;
  if (cap < 0 || (cap > 0 && !out_ms)) return fail(c, ECHO_EINVAL, "bad argument");
  std::lock_guard<std::mutex> lk(c->mu);
  if (c->rollout_running) return fail(c, ECHO_ESTATE, "a rollout is running on this context");
  for (size_t i = 0; i < c->step_ms.size() && i < (size_t)cap; ++i) out_ms[i] = c->step_ms[i];
  return (int)c->step_ms.size();
}

const char *echo_last_error(const echo_ctx *c) { return c ? c->err.c_str() : g_init_error.c_str(); }

void echo_destroy(echo_ctx *c) {
  if (!c) return;
  hipSetDevice(c->device);
  hipStreamSynchronize(c->cs);
  hipStreamSynchronize(c->ks);
  if (c->graph) hipGraphExecDestroy(c->graph);
  for (hipGraphExec_t g : c->retired_graphs) hipGraphExecDestroy(g);
  if (c->staged_ev) hipEventDestroy(c->staged_ev);
  for (int s = 0; s < 2; ++s) if (c->vacated_ev[s]) hipEventDestroy(c->vacated_ev[s]);
  if (c->own_cs) hipStreamDestroy(c->cs);
  if (c->own_ks) hipStreamDestroy(c->ks);
  delete c;
}

}  // extern "C"
