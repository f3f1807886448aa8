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

}  // namespace

// =================================================================================================== C ABI
extern "C" {

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

}  // extern "C"
