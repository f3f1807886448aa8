// Snapshot install behind the C ABI: the blob as a list of byte ranges, fed whole or in pieces through the staging
// buffer into the inactive weight slot on the copy stream (echo_load_policy and its begin / chunk / commit / abort form).
#include "echo_engine_impl.h"

namespace {

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

// Bytes [lo, lo + n) of the blob are replaced by `data` in a slot that already holds a whole snapshot: plain ranges are
// copied over, spans of a matrix go through the staging buffer and are re-packed element by element.
int patch_segments(echo_ctx *c, std::vector<BlobSeg> &segs, const char *data, size_t lo, size_t n) {
  const size_t hi = lo + n, elt = c->p.elt;
  for (BlobSeg &g : segs) {
    size_t a = std::max(lo, g.off), b = std::min(hi, g.off + g.bytes);
    if (a >= b) continue;
    const char *src = data + (a - lo);
    if (g.rows == 0) {
      HIPCHK(c, hipMemcpyAsync(g.dst + (a - g.off), src, b - a, hipMemcpyHostToDevice, c->ks));
      continue;
    }
    const int Np = (int)round_up(g.rows * g.stride, 32), Kp = (int)round_up(g.K, GEMM_K_PAD);
    const size_t half_stage = c->p.stage_bytes / 2;
    for (size_t o = a; o < b; o += half_stage) {
      const size_t len = std::min(half_stage, b - o);
      char *stg = c->arena + c->p.o_stage + (c->stage_flip ? half_stage : 0);
      c->stage_flip ^= 1;
      HIPCHK(c, hipMemcpyAsync(stg, data + (o - lo), len, hipMemcpyHostToDevice, c->ks));
      fast_pack_span(g.dst, stg, (int64_t)((o - g.off) / elt), (int64_t)(len / elt), g.dst_row0, g.stride, g.K, Kp, Np, c->ks);
    }
  }
  return 0;
}

// Bytes [lo, lo + n) of the bf16 blob sit at device address `dev` (whole rows of every matrix they touch): copy or pack
// them into every segment they cover, on the copy stream.
int feed_device(echo_ctx *c, std::vector<BlobSeg> &segs, const char *dev, size_t lo, size_t n) {
  const size_t hi = lo + n;
  for (BlobSeg &g : segs) {
    size_t a = std::max(lo, g.off), b = std::min(hi, g.off + g.bytes);
    if (a >= b) continue;
    const char *src = dev + (a - lo);
    if (g.rows == 0) {
      HIPCHK(c, hipMemcpyAsync(g.dst + (a - g.off), src, b - a, hipMemcpyDeviceToDevice, c->ks));
      continue;
    }
    const size_t row_bytes = (size_t)g.K * 2;
    if ((a - g.off) % row_bytes || (b - a) % row_bytes) return fail(c, ECHO_EINVAL, "internal: a device piece cuts a matrix row");
    const int Np = (int)round_up(g.rows * g.stride, 32), Kp = (int)round_up(g.K, GEMM_K_PAD);
    fast_pack_weight(g.dst, src, g.dst_row0 + (int64_t)((a - g.off) / row_bytes) * g.stride, g.stride, (int64_t)((b - a) / row_bytes), g.K, Kp, Np, c->ks);
  }
  return 0;
}

// The tensors of a blob in order: (rows, K), rows == 0 for a vector of K elements.
std::vector<std::pair<int64_t, int64_t>> blob_tensors(const echo_model_desc &d) {
  const int64_t H = d.hidden, hd = d.head_dim, Q = (int64_t)d.n_q_heads * hd, KV = (int64_t)d.n_kv_heads * hd, F = d.ffn, V = d.vocab;
  std::vector<std::pair<int64_t, int64_t>> t;
  t.push_back({V, H});
  for (int l = 0; l < d.n_layers; ++l) {
    t.push_back({0, H}); t.push_back({Q, H}); t.push_back({KV, H}); t.push_back({KV, H});
    if (d.qk_norm) { t.push_back({0, hd}); t.push_back({0, hd}); }
    t.push_back({H, Q}); t.push_back({0, H}); t.push_back({F, H}); t.push_back({F, H}); t.push_back({H, F});
  }
  t.push_back({0, H});
  if (!d.tie_embeddings) t.push_back({V, H});
  return t;
}

// The next n bytes of a quantised blob have arrived at `data` (host).  Vectors and rows of codes move whole: what a piece
// cuts waits in the carry buffer.  A matrix's scales go to their device buffer as they come; its codes are staged in batches
// of rows, turned into bf16 rows next to them and fed on as the bytes of the bf16 blob they stand for.  Everything runs on
// the copy stream, which is in order: a half of the staging buffer is free again when the copy that refills it is reached.
int feed_q8(echo_ctx *c, const char *data, size_t n) {
  Loading &L = c->load;
  const size_t half = c->p.stage_bytes / 2;
  auto stage = [&]() { char *p = c->arena + c->p.o_stage + (c->stage_flip ? half : 0); c->stage_flip ^= 1; return p; };
  char *d_scales = c->arena + c->p.o_qscales;
  // rows r0 .. r0 + nr - 1 of the current matrix, their codes at host address src
  auto rows_in = [&](const char *src, int64_t r0, int64_t nr, int64_t K) -> int {
    const int64_t per = std::max<int64_t>(1, (int64_t)((half - 256) / (size_t)(3 * K)));
    for (int64_t r = 0; r < nr; r += per) {
      const int64_t m = std::min(per, nr - r);
      char *stg = stage(), *d_codes = stg + round_up(m * K * 2, 256);
      HIPCHK(c, hipMemcpyAsync(d_codes, src + r * K, (size_t)(m * K), hipMemcpyHostToDevice, c->ks));
      fast_dequant_q8(stg, d_codes, d_scales + (r0 + r) * 4, m, (int)K, c->ks);
      int rc = feed_device(c, L.segs, stg, L.bf_off + (size_t)((r0 + r) * K * 2), (size_t)(m * K * 2));
      if (rc) return rc;
    }
    return 0;
  };
  while (n > 0) {
    if (L.ti >= L.tensors.size()) return fail(c, ECHO_EINVAL, "bytes past the end of the quantised blob");
    const int64_t rows = L.tensors[L.ti].first, K = L.tensors[L.ti].second;
    const size_t q_bytes = rows == 0 ? (size_t)K * 2 : (size_t)rows * 4 + (size_t)rows * K;
    size_t take = 0;
    if (rows == 0) {   // a vector: whole, through the carry buffer
      take = std::min(n, q_bytes - L.tb);
      L.carry.insert(L.carry.end(), data, data + take);
      if (L.carry.size() == q_bytes) {
        char *stg = stage();
        HIPCHK(c, hipMemcpyAsync(stg, L.carry.data(), q_bytes, hipMemcpyHostToDevice, c->ks));
        int rc = feed_device(c, L.segs, stg, L.bf_off, q_bytes);
        if (rc) return rc;
        HIPCHK(c, hipStreamSynchronize(c->ks));   // the carry buffer is reused
        L.carry.clear();
      }
    } else if (L.tb < (size_t)rows * 4) {   // scales, cut anywhere
      take = std::min(n, (size_t)rows * 4 - L.tb);
      HIPCHK(c, hipMemcpyAsync(d_scales + L.tb, data, take, hipMemcpyHostToDevice, c->ks));
    } else {   // codes
      const size_t cb = L.tb - (size_t)rows * 4;   // position inside the codes; a partial row is in the carry buffer
      if (!L.carry.empty()) {
        take = std::min(n, (size_t)K - L.carry.size());
        L.carry.insert(L.carry.end(), data, data + take);
        if ((int64_t)L.carry.size() == K) {
          int rc = rows_in(L.carry.data(), (int64_t)((cb - (L.carry.size() - take)) / K), 1, K);
          if (rc) return rc;
          HIPCHK(c, hipStreamSynchronize(c->ks));
          L.carry.clear();
        }
      } else {
        take = std::min(n, q_bytes - L.tb);
        const int64_t whole = (int64_t)(take / K);
        if (whole) {
          int rc = rows_in(data, (int64_t)(cb / K), whole, K);
          if (rc) return rc;
        }
        L.carry.assign(data + whole * K, data + take);
      }
    }
    data += take; n -= take; L.tb += take;
    if (L.tb == q_bytes) {   // the tensor is complete
      L.bf_off += rows == 0 ? (size_t)K * 2 : (size_t)(rows * K * 2);
      L.tb = 0;
      ++L.ti;
    }
  }
  return 0;
}

// The snapshot in slot `target` is complete on the copy stream: make it the active or the staged one.
int commit_slot(echo_ctx *c, int target, int64_t version) {
  HIPCHK(c, hipEventRecord(c->staged_ev, c->ks));
  HIPCHK(c, hipStreamSynchronize(c->ks));
  std::lock_guard<std::mutex> lk(c->mu);
  c->slots[target].version = version;
  c->newest_version = version;
  if (c->rollout_running) {
    c->staged = target;
    c->st.staged_version = version;
  } else {
    c->active = target;
    c->st.active_version = version;
  }
  c->load.open = false;
  c->load.segs.clear();
  c->cv.notify_all();
  return ECHO_OK;
}

}  // namespace

// =================================================================================================== C ABI
extern "C" {

int echo_load_policy_delta(echo_ctx *c, int64_t base_version, int64_t version, int32_t n_ranges, const uint64_t *offsets,
                           const uint64_t *sizes, const void *host_data) {
  if (!c) return ECHO_EINVAL;
  if (n_ranges < 0 || (n_ranges > 0 && (!offsets || !sizes || !host_data))) return fail(c, ECHO_EINVAL, "bad argument");
  const size_t blob = echo_blob_bytes(&c->d), elt = c->p.elt;
  size_t total = 0, prev_end = 0;
  for (int i = 0; i < n_ranges; ++i) {
    if (sizes[i] == 0 || offsets[i] % elt || sizes[i] % elt) return fail(c, ECHO_EINVAL, "range %d is empty or not a whole number of %zu-byte elements", i, elt);
    if (offsets[i] < prev_end || offsets[i] > blob || sizes[i] > blob - offsets[i])
      return fail(c, ECHO_EINVAL, "range %d overlaps its predecessor, is out of order or runs past the blob of %zu bytes", i, blob);
    prev_end = offsets[i] + sizes[i];
    total += sizes[i];
  }
  std::unique_lock<std::mutex> lk(c->mu);
  if (c->load.open) return fail(c, ECHO_ESTATE, "snapshot %lld is still arriving (commit or abort it first)", (long long)c->load.version);
  if (c->staged >= 0) return fail(c, ECHO_ESTATE, "a staged snapshot is still waiting to be switched in");
  if (c->active < 0 || base_version != c->newest_version)
    return fail(c, ECHO_ESTATE, "the delta is against version %lld, the newest installed snapshot is %lld", (long long)base_version, (long long)c->newest_version);
  if (version <= c->newest_version) return fail(c, ECHO_ESTATE, "version %lld does not advance past %lld", (long long)version, (long long)c->newest_version);
  const bool running = c->rollout_running;
  const int base = c->active;
  int target;
  if (c->d.n_weight_slots == 2) target = 1 - base;
  else if (!running) target = base;   // patched in place: nothing reads the only slot
  else return fail(c, ECHO_ESTATE, "installing during a rollout needs n_weight_slots = 2");
  c->load.open = true;
  c->load.version = version; c->load.target = target; c->load.received = 0; c->load.total = total;
  lk.unlock();
  auto undo = [&](int rc) {   // the target may hold part of two snapshots now
    hipStreamSynchronize(c->ks);
    std::lock_guard<std::mutex> g(c->mu);
    c->load.open = false;
    c->load.segs.clear();
    if (target == c->active) { c->active = -1; c->st.active_version = -1; }
    return rc;
  };
  if (hipSetDevice(c->device) != hipSuccess) return undo(fail(c, ECHO_EHIP, "hipSetDevice failed"));
  if (!running && hipStreamSynchronize(c->cs) != hipSuccess) return undo(fail(c, ECHO_EHIP, "hipStreamSynchronize failed"));
  if (target != base) {   // the other slot becomes a copy of the base first (behind whatever still reads it, see leave_slot)
    for (size_t o = 0; o < c->p.slot_bytes; o += (size_t)1 << 30) {
      size_t len = std::min((size_t)1 << 30, c->p.slot_bytes - o);
      if (hipMemcpyAsync(c->slots[target].base + o, c->slots[base].base + o, len, hipMemcpyDeviceToDevice, c->ks) != hipSuccess)
        return undo(fail(c, ECHO_EHIP, "copying the base snapshot failed"));
    }
  }
  c->load.segs = blob_segments(c, target);
  const char *data = (const char *)host_data;
  for (int i = 0; i < n_ranges; ++i) {
    int rc = patch_segments(c, c->load.segs, data, (size_t)offsets[i], (size_t)sizes[i]);
    if (rc) return undo(rc);
    data += sizes[i];
    if (hipStreamSynchronize(c->ks) != hipSuccess) return undo(fail(c, ECHO_EHIP, "hipStreamSynchronize failed"));   // staging halves are reused
  }
  int rc = commit_slot(c, target, version);
  return rc ? undo(rc) : ECHO_OK;
}

size_t echo_q8_blob_bytes(const echo_model_desc *desc) {
  if (!valid_desc(desc, nullptr) || desc->dtype != ECHO_BF16) return 0;
  size_t n = 0;
  for (auto &t : blob_tensors(*desc)) n += t.first == 0 ? (size_t)t.second * 2 : (size_t)t.first * 4 + (size_t)t.first * t.second;
  return n;
}

int echo_load_policy_q8_begin(echo_ctx *c, int64_t version, size_t nbytes) {
  if (!c) return ECHO_EINVAL;
  if (!c->p.fast) return fail(c, ECHO_EINVAL, "a quantised snapshot stands for bf16 weights and is unpacked through the MFMA path's staging buffer: the model dtype must be ECHO_BF16, without debug_naive");
  if (nbytes != echo_q8_blob_bytes(&c->d)) return fail(c, ECHO_EINVAL, "quantised blob has %zu bytes, this shape needs %zu", nbytes, echo_q8_blob_bytes(&c->d));
  int rc = echo_load_policy_begin(c, version, echo_blob_bytes(&c->d));
  if (rc) return rc;
  Loading &L = c->load;   // open: this thread's until commit or abort
  L.q8 = true;
  L.total = nbytes;
  L.tensors = blob_tensors(c->d);
  L.ti = 0; L.tb = 0; L.bf_off = 0;
  L.carry.clear();
  return ECHO_OK;
}

int echo_load_policy_q8(echo_ctx *c, int64_t version, const void *host_blob, size_t nbytes) {
  if (!c) return ECHO_EINVAL;
  if (!host_blob) return fail(c, ECHO_EINVAL, "host_blob is NULL");
  int rc = echo_load_policy_q8_begin(c, version, nbytes);
  if (rc) return rc;
  if ((rc = echo_load_policy_chunk(c, host_blob, nbytes)) || (rc = echo_load_policy_commit(c))) {
    std::string msg = c->err;
    echo_load_policy_abort(c);
    c->err = msg;
  }
  return rc;
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
  c->load.q8 = false;
  lk.unlock();
  auto undo = [&](int rc) { lk.lock(); c->load.open = false; if (target == c->active) { c->active = -1; c->st.active_version = -1; } return rc; };
  if (hipSetDevice(c->device) != hipSuccess) return undo(fail(c, ECHO_EHIP, "hipSetDevice failed"));
  if (!running && hipStreamSynchronize(c->cs) != hipSuccess) return undo(fail(c, ECHO_EHIP, "hipStreamSynchronize failed"));
  c->load.segs = blob_segments(c, target);
  // (A rollout that has just switched away from the target slot may still have decode steps queued that read it; the
  // rollout made the copy stream wait for them when it switched, see leave_slot.)
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
  int rc = c->load.q8 ? feed_q8(c, (const char *)data, nbytes) : feed_segments(c, c->load.segs, (const char *)data, c->load.received, nbytes);
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
  return commit_slot(c, c->load.target, c->load.version);
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

}  // extern "C"
