// The rollout entry points behind the C ABI: echo_rollout (all sequences start together, one HIP graph per snapshot
// replayed per generation step) and echo_rollout_continuous (refill, compaction), with the planning of the shared-prompt
// attention jobs and the argument checks they share.
#include "echo_engine_impl.h"

namespace {

int capture_step(echo_ctx *c, const Slot &S, int N, int max_new, float temperature, uint64_t seed, bool unfused, const int32_t *forced,
                 int eos, float top_p, int per_row = 0) {
  if (c->graph) { c->retired_graphs.push_back(c->graph); c->graph = nullptr; }
  hipGraph_t g = nullptr;
  HIPCHK(c, hipStreamBeginCapture(c->cs, hipStreamCaptureModeThreadLocal));
  forward_layers(c, S, N, !c->attn_plain);
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
                     int max_ptiles, int grid_jobs, int prefix_kernel /* echo_rollout_opts.prefix_kernel */) {
  const int grp = c->d.n_q_heads / c->d.n_kv_heads, per_job = std::max(1, 32 / grp);
  const int cap = pad_rows(c->d.max_seqs) / 2 + 1;
  c->px = PrefixPlan{at<PrefixJob>(c, c->p.o_pjobs), 0, 0, 1};
  for (int r = 0; r < R; ++r) ptiles[r] &= ~ATT_PREFIX_DONE;
  if (!c->p.fast || max_ptiles < 1 || fast_attention_splits(R, c->d.n_kv_heads, c->p.attn_max_splits) != 1 || prefix_kernel == 1) return 0;
  if (fast_attention_rows_per_group(R, c->d.n_q_heads, c->d.n_kv_heads, c->attn_mode) > 1) return 0;   // the decode kernel shares the tiles itself
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
  // The extra launch costs more than it saves at 64 rows x 16 tiles (measured: -7 % there; -2 % at a draining 128 x 32,
  // +5 % at 256 x 32), so small batches with short prompts keep reading their shared tiles in the decode kernel.  A
  // batch that is refilled as sequences end (grid_jobs > 0) keeps 256 rows of unequal lengths in flight: +9 % at 256 x 15.
  int64_t covered = 0, min_covered = prefix_kernel == 2 ? 0 : grid_jobs > 0 ? 3584 : 6144;
  for (const PrefixJob &jb : jobs) covered += (int64_t)jb.nrows * jb.ptiles;
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
  if (o->prefix_kernel < 0 || o->prefix_kernel > 3) return fail(c, ECHO_EINVAL, "prefix_kernel must be 0, 1, 2 or 3");
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
    if (!c->retired_graphs.empty()) {   // step graphs replaced at a snapshot switch or a compaction
      hipStreamSynchronize(c->cs);
      for (hipGraphExec_t g : c->retired_graphs) hipGraphExecDestroy(g);
      c->retired_graphs.clear();
    }
    std::lock_guard<std::mutex> lk(c->mu);
    c->rollout_running = false;
    c->attn_plain = false;
    c->attn_mode = 0;
    c->ids = DrawIds{c->d_step, nullptr, nullptr};
    c->px.n_jobs = 0;
    if (c->staged >= 0) {   // (a rollout that failed half-way may have left work queued on the old slot)
      leave_slot(c, c->active);
      c->active = c->staged; c->staged = -1; c->st.active_version = c->slots[c->active].version; c->st.staged_version = -1;
    }
  }
};

}  // namespace

// =================================================================================================== C ABI
extern "C" {

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
  c->attn_plain = o.attn_plain != 0;
  c->attn_mode = o.prefix_kernel;
  const bool share_prefix = p.fast && !o.own_prompt_copy && !o.attn_plain;
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
  std::vector<int32_t> ident(N);   // (a vector of its own: the copy above may still be reading `map`)
  for (int n = 0; n < N; ++n) ident[n] = n;
  HIPCHK(c, hipMemcpyAsync(c->rows.slot, ident.data(), N * 4, hipMemcpyHostToDevice, st));
  // decode attention reads the whole tiles of a group's prompt from the group's first slot
  std::vector<int32_t> pslot(N), ptiles(N), stream(N);
  int max_ptiles = 0;
  {
    std::vector<int32_t> live(N, 1);
    for (int n = 0; n < N; ++n) {
      pslot[n] = n / G * G;
      ptiles[n] = share_prefix ? prompt_lens[n / G] / 32 : 0;
      max_ptiles = std::max(max_ptiles, ptiles[n]);
      stream[n] = n;
    }
    if ((rc = plan_prefix_jobs(c, ptiles, pslot, live, N, max_ptiles, 0, o.prefix_kernel))) return rc;
    HIPCHK(c, hipMemcpyAsync(c->rows.pslot, pslot.data(), N * 4, hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(c->rows.ptiles, ptiles.data(), N * 4, hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(c->d_stream, stream.data(), N * 4, hipMemcpyHostToDevice, st));
    HIPCHK(c, hipStreamSynchronize(st));
  }
  c->ids = DrawIds{c->d_step, nullptr, c->d_stream};   // a row's draws are keyed by its sequence, wherever the row moves
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
  int Rc = N;   // rows of the batch now (row r serves sequence row_seq[r]; rows are moved up when the batch has drained enough)
  std::vector<int> row_seq(N);
  for (int n = 0; n < N; ++n) row_seq[n] = n;
  std::vector<int32_t> lens_host(N, 0);
  auto book = [&](int slot) {
    launch_bookkeeping(Rc, max_new, 0, c->d_step, c->d_samp_tok, c->d_samp_lp, d_forced, c->d_limit, o.eos_id, c->slots[slot].version,
                       c->d_prompt_len_seq, c->d_gen_len, c->rows, at<int32_t>(c, p.o_out_tok), at<float>(c, p.o_out_lp),
                       at<int64_t>(c, p.o_out_ver), c->d_n_active, st);
  };
  book(cur);
  launch_kv_replicate(c->kv, c->d_plen_p, P, G, st);
  HIPCHK(c, hipStreamSynchronize(st));
  auto t1 = std::chrono::steady_clock::now();

  // ---- decode
  c->timing = want_timing;
  std::vector<hipEvent_t> step_ev;   // time_steps: one event per step boundary
  auto mark_step = [&]() -> int {
    if (!o.time_steps) return 0;
    hipEvent_t e;
    HIPCHK(c, hipEventCreate(&e));
    step_ev.push_back(e);
    HIPCHK(c, hipEventRecord(e, st));
    return 0;
  };
  if ((rc = mark_step())) return rc;
  double swap_wait = 0;
  int next_swap = 0, decode_steps = 0;
  bool have_graph = false;
  bool splitk = !o.attn_plain;
  const bool may_compact = !o.debug_logits && !o.no_compaction;   // (returned logits are in sequence order)
  for (int s = 1; s < steps; ++s) {
    if (next_swap < o.n_swaps && o.swap_at_step[next_swap] == s) {
      auto w0 = std::chrono::steady_clock::now();
      std::unique_lock<std::mutex> lk(c->mu);
      int tmo = o.swap_timeout_ms > 0 ? o.swap_timeout_ms : 10000;
      if (!c->cv.wait_for(lk, std::chrono::milliseconds(tmo), [&] { return c->staged >= 0; }))
        return fail(c, ECHO_ESTATE, "no snapshot was staged for the swap at step %d within %d ms", s, tmo);
      HIPCHK(c, leave_slot(c, cur));   // before the lock is released: an install that finds the old slot free starts behind its readers
      cur = c->staged; c->active = cur; c->staged = -1;
      c->st.active_version = c->slots[cur].version; c->st.staged_version = -1;
      lk.unlock();
      HIPCHK(c, hipStreamWaitEvent(st, c->staged_ev, 0));
      swap_wait += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - w0).count();
      have_graph = false;
      ++next_swap;
    }
    int live_now = Rc;   // sequences that take part in pass s, as far as the host knows
    if (o.eos_id >= 0) {
      if ((s % 16) == 0) {  // sequences may have ended early: look at the active count
        int32_t na = 0;
        HIPCHK(c, hipMemcpyAsync(&na, c->d_n_active, 4, hipMemcpyDeviceToHost, st));
        HIPCHK(c, hipStreamSynchronize(st));
        if (na == 0) break;
        live_now = na;
      }
    } else {
      live_now = 0;
      for (int r = 0; r < Rc; ++r) live_now += limit[row_seq[r]] > s;
    }
    // A draining batch: once the sequences still generating fit a smaller padded batch their rows are moved to the
    // front (cache slots and records stay where they are) and the step is captured again for fewer rows.  With stop
    // lengths only, the host knows who is still generating; with an end-of-sequence token it looks every 16 steps.
    if (may_compact && pad_rows(std::max(1, live_now)) < pad_rows(Rc) && live_now > 0) {
      std::vector<int32_t> tok(Rc), pos(Rc), act(Rc), gen(Rc);
      HIPCHK(c, hipMemcpyAsync(tok.data(), c->rows.token, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
      HIPCHK(c, hipMemcpyAsync(pos.data(), c->rows.pos, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
      HIPCHK(c, hipMemcpyAsync(act.data(), c->rows.active, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
      HIPCHK(c, hipMemcpyAsync(gen.data(), c->d_gen_len, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
      HIPCHK(c, hipStreamSynchronize(st));
      std::vector<int32_t> slot2, pslot2, ptiles2, plen2, lim2, stream2, tok2, pos2, act2, gen2, live2;
      std::vector<int> seq2;
      for (int r = 0; r < Rc; ++r) {
        const int n = row_seq[r];
        if (!act[r]) { lens_host[n] = gen[r]; continue; }
        tok2.push_back(tok[r]); pos2.push_back(pos[r]); act2.push_back(1); gen2.push_back(gen[r]); slot2.push_back(n);
        pslot2.push_back(pslot[r]); ptiles2.push_back(ptiles[r]); plen2.push_back(plen_seq[n]); lim2.push_back(limit[n]);
        stream2.push_back(n); seq2.push_back(n); live2.push_back(1);
      }
      const int w = (int)seq2.size();
      if (w > 0 && pad_rows(w) < pad_rows(Rc)) {
        if ((rc = plan_prefix_jobs(c, ptiles2, pslot2, live2, w, max_ptiles, 0, o.prefix_kernel))) return rc;
        struct { int32_t *dst; std::vector<int32_t> *src; } cp[] = {
            {c->rows.token, &tok2}, {c->rows.pos, &pos2}, {c->rows.active, &act2}, {c->rows.slot, &slot2}, {c->rows.pslot, &pslot2},
            {c->rows.ptiles, &ptiles2}, {c->d_prompt_len_seq, &plen2}, {c->d_gen_len, &gen2}, {c->d_limit, &lim2}, {c->d_stream, &stream2}};
        for (auto &x : cp) HIPCHK(c, hipMemcpyAsync(x.dst, x.src->data(), (size_t)w * 4, hipMemcpyHostToDevice, st));
        launch_fill_i32(c->rows.active + w, 0, Rc - w, st);   // the rows given up
        HIPCHK(c, hipStreamSynchronize(st));
        pslot = pslot2; ptiles = ptiles2; row_seq = seq2;
        Rc = w;
        have_graph = false;
      }
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
        if ((rc = capture_step(c, c->slots[cur], Rc, max_new, temperature, seed, unfused, d_forced, o.eos_id, o.top_p))) return rc;
        have_graph = true;
      }
      HIPCHK(c, hipGraphLaunch(c->graph, st));
    } else {
      forward_layers(c, c->slots[cur], Rc, splitk);
      sample_rows(c, c->slots[cur], Rc, temperature, seed, unfused, nullptr, o.top_p);
      if ((rc = grab_logits(s))) return rc;
      book(cur);
    }
    c->timing = time_this;
    ++decode_steps;
    if ((rc = mark_step())) return rc;
  }
  HIPCHK(c, hipStreamSynchronize(st));
  auto t2 = std::chrono::steady_clock::now();
  if (o.time_steps) {
    c->step_ms.clear();
    for (size_t i = 1; i < step_ev.size(); ++i) {
      float t = 0;
      if (hipEventElapsedTime(&t, step_ev[i - 1], step_ev[i]) == hipSuccess) c->step_ms.push_back(t);
    }
    for (hipEvent_t e : step_ev) hipEventDestroy(e);
  }

  // ---- results
  HIPCHK(c, hipMemcpyAsync(out_tokens, at<int32_t>(c, p.o_out_tok), outn * 4, hipMemcpyDeviceToHost, st));
  HIPCHK(c, hipMemcpyAsync(out_logprobs, at<float>(c, p.o_out_lp), outn * 4, hipMemcpyDeviceToHost, st));
  if (out_versions) HIPCHK(c, hipMemcpyAsync(out_versions, at<int64_t>(c, p.o_out_ver), outn * 8, hipMemcpyDeviceToHost, st));
  {
    std::vector<int32_t> gen(Rc);
    HIPCHK(c, hipMemcpyAsync(gen.data(), c->d_gen_len, (size_t)Rc * 4, hipMemcpyDeviceToHost, st));
    HIPCHK(c, hipStreamSynchronize(st));
    for (int r = 0; r < Rc; ++r) lens_host[row_seq[r]] = gen[r];
    memcpy(out_lens, lens_host.data(), (size_t)N * 4);
  }
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
  if (o.n_swaps || o.debug_logits || o.time_kernels || o.time_steps)
    return fail(c, ECHO_EINVAL, "a continuous rollout takes no pinned swaps (it switches when a snapshot is staged), no debug_logits, no time_kernels and no time_steps");
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
  c->attn_plain = o.attn_plain != 0;
  // rows of unequal lengths: workgroups of several rows, one per compute unit, would finish at very different times
  // (measured 22.7 k tokens/s against 25.5 k with the once-per-group kernel at 256 rows), so unless asked for that form is
  // taken only while the live rows sit at about the same position (decided whenever the rows change, below)
  c->attn_mode = o.prefix_kernel == 0 ? 1 : o.prefix_kernel;
  const bool share_prefix = p.fast && !o.own_prompt_copy && !o.attn_plain;
  const bool splitk = !o.attn_plain;
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
        int pos_lo = INT32_MAX, pos_hi = 0;
        for (int r = 0; r < Rc; ++r) {
          live[r] = row_seq[r] >= 0 && act[r];
          if (live[r]) { pos_lo = std::min(pos_lo, pos[r]); pos_hi = std::max(pos_hi, pos[r]); }
        }
        if (o.prefix_kernel == 0) {   // several rows per decode-attention workgroup only while their lengths are within an eighth
          const int mode = pos_hi >= pos_lo && (pos_hi - pos_lo) * 8 <= pos_hi ? 0 : 1;
          if (mode != c->attn_mode) { c->attn_mode = mode; have_graph = false; }
        }
        const PrefixPlan was = c->px;
        if ((rc = plan_prefix_jobs(c, ptiles, pslot, live, Rc, share_prefix ? (max_pl - 1) / 32 : 0, Rc / 2 + 1, o.prefix_kernel))) return rc;
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
        HIPCHK(c, leave_slot(c, cur));   // the steps queued so far still read the old slot
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

}  // extern "C"
