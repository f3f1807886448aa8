/*
 * echo.h -- C ABI of the MI355X rollout-generation library.
 *
 * The library is the GPU side of a rollout worker as ECHO-2 states the problem:
 * a worker holds a locally installed policy snapshot of some version, draws
 * responses y ~ pi_v(. | x) for prompts x, and emits them tagged with that version
 * (Sec. 4.1 "Versioned Execution and Bounded Staleness"; Algorithm 1, rollout-plane loop); the learner's
 * truncated importance ratio needs the sampler's own per-token probability
 * (App. "GRPO-Style Policy Gradient Objective"); a worker switches to a new
 * snapshot once it is completely installed (Sec. 4.2).  The policy is a dense
 * decoder-only transformer (RMSNorm, grouped-query attention with rotary
 * embeddings, SwiGLU, no biases); every step of the path runs in HIP kernels for
 * gfx950.  One context drives one GPU.  There is no CPU fallback.
 *
 * Conventions: all functions return 0 on success or a negative echo_status; they
 * never throw, abort or print.  "host" / "device" in a parameter comment says
 * where the pointer must live.  The caller owns every buffer it passes in.
 */
#ifndef ECHO_H_
#define ECHO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct echo_ctx echo_ctx; /* opaque, one per GPU */

typedef enum {
  ECHO_OK = 0,
  ECHO_EINVAL = -1, /* bad argument or shape */
  ECHO_ENOMEM = -2, /* arena too small / request exceeds max_seqs or max_ctx */
  ECHO_ESTATE = -3, /* no policy installed, version not increasing, swap never staged */
  ECHO_EHIP = -4    /* a HIP runtime call failed */
} echo_status;

enum { ECHO_F32 = 0, ECHO_BF16 = 1 };

/* Decoder shape and capacity.  dtype selects the storage type of weights and KV cache:
 * ECHO_BF16 (weights are bf16 values) runs the MFMA kernels: half-precision operands -- the weights converted
 * exactly, activations and the KV cache rounded to half -- fp32 accumulation, fp32 residual stream;
 * ECHO_F32 runs the all-fp32 debug kernels.  debug_naive = 1 with ECHO_BF16 keeps bf16
 * weights but runs the debug kernels on them (fp32 activations and KV cache).
 * Range of the half-precision operands (ECHO_BF16 without debug_naive): a value that is rounded to half -- a normed
 * activation, a query, a cached key or value, a SwiGLU output -- saturates at the largest finite half, +-65504, instead
 * of becoming infinite, so everything downstream stays finite (and differs from an unbounded evaluation from there on);
 * weights are held as halves of 256 times their value, exact for every bf16 weight of magnitude 2^-22 .. 255 and
 * saturating beyond (smaller magnitudes flush towards zero); accumulation and the residual stream are fp32. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rms_eps, rope_base;
  int32_t dtype;
  int32_t qk_norm;        /* 1: per-head RMSNorm on q and k before the rotary embedding */
  int32_t tie_embeddings; /* 1: lm_head is the embedding table (absent from the blob) */
  int32_t max_seqs;       /* KV-cache capacity in sequences (P*G of the largest rollout) */
  int32_t max_ctx;        /* KV-cache capacity in tokens per sequence (prompt + generated) */
  int32_t n_weight_slots; /* 1, or 2 to install a snapshot while another is decoding */
  int32_t debug_naive;
} echo_model_desc;

/* Optional rollout controls (a NULL opts means: none of them). */
typedef struct {
  const int32_t *stop_lens;    /* host [N] or NULL: sequence n ends after min(max_new, stop_lens[n]) tokens */
  int32_t eos_id;              /* >= 0: a sequence also ends after emitting this token (kept); -1: none */
  float top_p;                 /* in (0, 1]; 1.0: no truncation.  Below 1 (Sec. 5.1 runs rollouts at 0.95): sample from the
                                  shortest descending-probability prefix reaching top_p; out_logprobs are then renormalised
                                  over that kept set (the distribution actually sampled); logits are materialised per step */
  int32_t n_swaps;             /* snapshot switches pinned inside this rollout */
  const int32_t *swap_at_step; /* host [n_swaps], ascending, >= 1: from generation step k on, the forward
                                  passes use the snapshot staged by echo_load_policy (the call waits for it,
                                  at most swap_timeout_ms); the KV cache built so far is kept */
  int32_t swap_timeout_ms;     /* 0 = 10000 */
  const int32_t *forced_tokens; /* host [N, max_new] or NULL: teacher forcing -- the sampled token and its
                                   log-prob are still returned, the token fed back is the forced one */
  float *debug_logits;         /* host [N, max_new, vocab] or NULL: also return the raw logits (uses the
                                  unfused sampler; sizes the caller can afford only) */
  int32_t unfused_sampler;     /* 1: write logits to HBM and sample from them with the fp32 debug sampler */
  int32_t no_graph;            /* 1: launch decode steps kernel by kernel instead of replaying a HIP graph */
  int32_t time_kernels;        /* 1: bracket decode-attention and GEMM launches with HIP events (implies
                                  no_graph); durations are read back with echo_stats */
  int32_t time_steps;          /* 1 (echo_rollout only): a HIP event between every two decode steps (graph replays
                                  included); the per-step durations are read back with echo_step_times */
  int32_t no_compaction;       /* 1 (echo_rollout only): rows of sequences that have ended stay in the batch as inactive
                                  rows until the call ends, instead of the rows of a drained batch being moved together */
  /* Cross-check switches (0 = the default path; results differ from it by rounding order at most, see each): */
  int32_t attn_plain;          /* 1: decode and prompt attention by the plain kernel (one wavefront per (row, head), two
                                  passes, no key splitting, no sharing of prompt tiles) instead of the MFMA kernels */
  int32_t own_prompt_copy;     /* 1: every sequence reads its own replicated copy of its group's prompt K/V instead of
                                  the copy in the group's first cache slot (bit-identical results) */
  int32_t prefix_kernel;       /* who attends a group's shared whole prompt tiles: 0 = the planner decides by batch size,
                                  1 = always each row on its own in the decode kernel, 2 = always the once-per-group kernel
                                  where it applies (a row's keys not split over workgroups), 3 = always decode workgroups
                                  that take several neighbouring rows and their common prompt tiles once; the forms differ
                                  by summation order */
} echo_rollout_opts;

typedef struct {
  int64_t active_version, staged_version; /* -1 when none */
  int32_t decode_steps;                   /* decode forward passes of the last rollout */
  float prefill_ms, decode_ms, total_ms;  /* wall time of the last rollout, by phase */
  float swap_wait_ms;                     /* time the last rollout waited for staged snapshots */
  /* filled by a rollout run with time_kernels = 1 (sums over all timed launches): */
  int64_t attn_launches;
  double attn_ms, attn_bytes; /* decode attention: HIP-event time, K/V bytes it had to read (whole prompt tiles once per group) */
  int64_t gemm_launches;
  double gemm_ms, gemm_bytes; /* weight-streaming GEMMs: HIP-event time, weight bytes read */
  int32_t rollout_running;    /* 1 while echo_rollout is inside its loop on another thread (a snapshot installed
                                 now is staged, not activated) */
  int32_t attn_rows_per_workgroup; /* rows of the batch that one workgroup of the decode attention took in the last decode
                                 step that was launched or captured (1: a workgroup per row and KV head; see prefix_kernel) */
  int32_t attn_prefix_jobs;   /* jobs of the once-per-group prompt kernel in that step (0: the kernel did not run) */
} echo_stats_t;

/* Bytes of device memory a context of this shape needs (weights x slots, KV cache, activations);
 * 0 if the shape is invalid. */
size_t echo_arena_bytes(const echo_model_desc *desc);

/* Bytes of one policy blob for this shape (see echo_load_policy); 0 if the shape is invalid. */
size_t echo_blob_bytes(const echo_model_desc *desc);

/* Create a context on `device`.  dev_arena (device, >= echo_arena_bytes, 256-byte aligned) is owned by the
 * caller and must outlive the context; compute_stream / copy_stream are hipStream_t handles of default
 * priority (the caller's; NULL = the null stream).  *out receives the context. */
int echo_init(const echo_model_desc *desc, int device, void *dev_arena, size_t arena_bytes,
              void *compute_stream, void *copy_stream, echo_ctx **out);

/* Install policy snapshot `version` (Sec. 4.1-4.2: immutable snapshots, versions only advance).
 * host_weights (host, nbytes = echo_blob_bytes) is a flat row-major [out,in] blob in the model dtype:
 *   embed[V,d]; per layer attn_norm[d], wq[Hq*hd,d], wk[Hkv*hd,d], wv[Hkv*hd,d], (q_norm[hd], k_norm[hd]),
 *   wo[d,Hq*hd], ffn_norm[d], w_gate[F,d], w_up[F,d], w_down[d,F]; final_norm[d]; lm_head[V,d] (if untied).
 * The blob is copied and repacked on the GPU (copy stream) into the inactive weight slot; it may be freed
 * when the call returns.  With no rollout running the snapshot becomes active at once; while a rollout runs
 * (call from another thread; needs n_weight_slots = 2) it is staged and becomes active at the rollout's next
 * pinned swap step, or when the rollout ends.  ECHO_ESTATE if version <= the newest installed version or if
 * a staged snapshot is still waiting. */
int echo_load_policy(echo_ctx *ctx, int64_t version, const void *host_weights, size_t nbytes);

/* The same install for a snapshot that arrives in pieces (Sec. 4.2: snapshots travel as chunks that a worker
 * forwards and consumes as they land, and generation under the new version starts once the last one is in).
 *   echo_load_policy_begin(version, nbytes)  opens the load: same checks, same choice of weight slot and same
 *                                            errors as echo_load_policy; nbytes = echo_blob_bytes
 *   echo_load_policy_chunk(data, nbytes)     the next nbytes of the blob (host), in blob order, any sizes, cut at any
 *                                            byte; copied and repacked on the copy stream while a rollout keeps
 *                                            decoding; data may be freed when the call returns.  After an error
 *                                            the load must be aborted
 *   echo_load_policy_commit()                all bytes are in (ECHO_ESTATE otherwise): the snapshot becomes active
 *                                            or staged exactly as after echo_load_policy
 *   echo_load_policy_abort()                 drops the load; the version may be offered again
 * The calls of one load come from one thread at a time; a rollout may run, start and end meanwhile, except that
 * with n_weight_slots = 1 the load overwrites the active snapshot: echo_rollout and echo_logprobs return
 * ECHO_ESTATE until the commit, and after an abort no snapshot is installed.  The result is bit for bit the
 * one echo_load_policy leaves for the same bytes. */
int echo_load_policy_begin(echo_ctx *ctx, int64_t version, size_t nbytes);
int echo_load_policy_chunk(echo_ctx *ctx, const void *data, size_t nbytes);
int echo_load_policy_commit(echo_ctx *ctx);
int echo_load_policy_abort(echo_ctx *ctx);

/* Install snapshot `version` as a delta against the newest installed snapshot (Sec. 4.2 ships whole snapshots in chunks;
 * the "Limitations and Future Work" section names delta updates as the way to cut that traffic): the new blob is the
 * blob of base_version with n_ranges byte ranges replaced.
 *   offsets, sizes  host [n_ranges]: byte ranges of the blob, ascending and non-overlapping, whole elements of the model
 *                   dtype (they may start and end anywhere inside a tensor or a matrix row, and span tensors)
 *   host_data       host: the new bytes of all ranges, concatenated in range order
 * With n_weight_slots = 2 the inactive slot first becomes a device-side copy of the base snapshot, then the ranges are
 * copied in and re-packed on the copy stream, while a rollout may keep decoding; with one slot the active snapshot is
 * patched in place (no rollout may be running).  The result is bit for bit the snapshot a full echo_load_policy of the
 * patched blob leaves, and it becomes active or staged exactly as there.  ECHO_ESTATE if base_version is not the
 * newest installed snapshot, if version does not advance, if another load is open or a staged snapshot is waiting;
 * ECHO_EINVAL for a bad range list.  After a failure half-way a slot that was patched in place holds no snapshot. */
int echo_load_policy_delta(echo_ctx *ctx, int64_t base_version, int64_t version, int32_t n_ranges, const uint64_t *offsets,
                           const uint64_t *sizes, const void *host_data);

/* Install snapshot `version` from a quantised blob (the "Limitations and Future Work" section names quantised updates,
 * next to delta updates, as the way to cut snapshot traffic; it gives no format, this is the library's): the tensors of
 * the echo_load_policy blob in the same order; a vector (norm gain) as bf16, unchanged; a matrix [rows, K] as `rows`
 * little-endian fp32 scales followed by rows * K int8 codes, row-major.  The weight a code stands for is the bf16 value
 * nearest (ties to even) to float(code) * scale of its row, one fp32 product.  host_blob (host, nbytes =
 * echo_q8_blob_bytes: about half the bf16 blob) may be freed when the call returns.  Codes and scales are copied to the
 * GPU as they are, turned into bf16 rows and packed on the copy stream, so the PCIe traffic is that of the quantised
 * blob; the result is bit for bit the snapshot echo_load_policy leaves for the dequantised bf16 blob, and it becomes
 * active or staged exactly as there, with the same errors.  Needs dtype = ECHO_BF16 without debug_naive (ECHO_EINVAL
 * otherwise, and for a wrong size); echo_q8_blob_bytes returns 0 for an invalid shape or another dtype. */
size_t echo_q8_blob_bytes(const echo_model_desc *desc);
int echo_load_policy_q8(echo_ctx *ctx, int64_t version, const void *host_blob, size_t nbytes);
/* The same for a quantised blob that arrives in pieces (Sec. 4.2): echo_load_policy_q8_begin opens the load (nbytes =
 * echo_q8_blob_bytes; checks, slot choice and errors as echo_load_policy_begin), then echo_load_policy_chunk takes the
 * bytes of the quantised blob in order, in pieces of any size cut at any byte, and echo_load_policy_commit /
 * echo_load_policy_abort end the load as for a bf16 blob.  Bit for bit the snapshot of the one-call form. */
int echo_load_policy_q8_begin(echo_ctx *ctx, int64_t version, size_t nbytes);

/* Generate G samples for each of n_prompts prompts (sequence n = p*G + g) by ancestral sampling from
 * softmax(logits / temperature) (Algorithm 1, "sample and generate y ~ pi(.|x)"), up to max_new tokens each.
 * The draw for vocabulary entry i of sequence n at step s is the Gumbel-max rule on a counter-based uniform
 * keyed by (seed; n, s, i), so a sequence's result does not depend on what else is in the batch.
 *   prompt_tokens  host [n_prompts, prompt_stride]; prompt_lens host [n_prompts], each in 1..prompt_stride
 *   out_tokens     host [N, max_new], pad -1        out_logprobs host [N, max_new], pad 0
 *   out_lens       host [N]                         out_versions host [N, max_new], pad -1 (nullable)
 * out_logprobs[n][s] = log softmax(logits/temperature)[out_tokens[n][s]].
 * ECHO_ENOMEM if N > max_seqs or prompt_len + max_new > max_ctx; ECHO_ESTATE without a policy. */
int echo_rollout(echo_ctx *ctx, const int32_t *prompt_tokens, int32_t prompt_stride, const int32_t *prompt_lens,
                 int32_t n_prompts, int32_t G, int32_t max_new, float temperature, uint64_t seed,
                 const echo_rollout_opts *opts, int32_t *out_tokens, float *out_logprobs, int32_t *out_lens,
                 int64_t *out_versions);

/* The same rollout for more prompts than the KV cache holds at once: the worker's generate-continuously loop
 * (Algorithm 1, rollout side).  max_seqs / G groups decode together; when all G sequences of a group have
 * ended its records are handed over and the next waiting prompt takes its cache slots, so the batch stays
 * full until the prompts run out.  Arguments, output layout (sequence n = p*G + g over ALL n_prompts), sampling
 * rule and per-sequence results are those of echo_rollout -- the draw of sequence n at its own step s is keyed
 * (seed; n, s, i) whenever it runs -- with these differences:
 *   - n_prompts * G may exceed max_seqs (G may not: ECHO_ENOMEM); prompt_len + max_new <= max_ctx as before;
 *   - a snapshot staged by echo_load_policy / _commit while the call runs is switched in between two decode
 *     steps as soon as it is there (out_versions tags every token); pinned swaps (n_swaps), debug_logits and
 *     time_kernels are refused with ECHO_EINVAL;
 *   - echo_stats: prefill_ms is the time spent admitting prompts, decode_ms the rest. */
int echo_rollout_continuous(echo_ctx *ctx, const int32_t *prompt_tokens, int32_t prompt_stride,
                            const int32_t *prompt_lens, int32_t n_prompts, int32_t G, int32_t max_new,
                            float temperature, uint64_t seed, const echo_rollout_opts *opts, int32_t *out_tokens,
                            float *out_logprobs, int32_t *out_lens, int64_t *out_versions);

/* Teacher-forced scoring under the active snapshot (the learner-side pi(y_t | x, y_<t) of the importance
 * ratio): out[n][t] = log softmax(logits_{t-1}/temperature)[tokens[n][t]] for 1 <= t < lens[n], else 0.
 *   tokens host [n_seqs, stride]; lens host [n_seqs]; out host [n_seqs, stride]. */
int echo_logprobs(echo_ctx *ctx, const int32_t *tokens, int32_t stride, const int32_t *lens, int32_t n_seqs,
                  float temperature, float *out_logprobs);

/* Learner-side tensors of a batch of finished records (App. "Turn-Aware Masking", App. "Outcome-Based Returns and
 * Group-wise Normalization"), computed on the GPU; sequence n belongs to group n / G.
 *   c[n][t]          = number of k <= t with tokens[n][k] == turn_start_id         (turn index)
 *   out_mask[n][t]   = 1 if t < lens[n], c > 1 and c odd, else 0                   (response tokens)
 *   out_adv[n]       = (rewards[n] - mean) / (std + eps), mean and std over the group's G returns, std the
 *                      sample standard deviation (divisor G - 1), sums in f64, result rounded to f32
 *   out_adv_tok[n][t] = out_adv[n] * out_mask[n][t]                                (nullable)
 *   tokens host [n_seqs, stride]; lens host [n_seqs], each in 0..stride; rewards host [n_seqs];
 *   out_mask host u8 [n_seqs, stride]; out_adv host [n_seqs]; out_adv_tok host [n_seqs, stride].
 * Needs no policy.  ECHO_EINVAL if G < 2, n_seqs is not a positive multiple of G or eps < 0; ECHO_ENOMEM if one
 * group of G rows does not fit the context's staging buffer (9 bytes per token); ECHO_ESTATE during a rollout. */
int echo_grpo_tensors(echo_ctx *ctx, const int32_t *tokens, int32_t stride, const int32_t *lens, int32_t n_seqs,
                      int32_t G, int32_t turn_start_id, const float *rewards, float eps, uint8_t *out_mask,
                      float *out_adv, float *out_adv_tok);

/* echo_grpo_tensors for callers that cannot allocate device memory and whose context has no arena to lend (tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same kernels and bit-identical results, but the records are
 * staged in a fixed array of ECHO_STATIC_SCRATCH_BYTES that the library itself holds on every GPU it runs on (from
 * echo_init of the first context on that GPU until the process ends) instead of in the context's arena.  The call
 * allocates nothing: no hipMalloc / hipFree, no allocating library routine.  All records of a call must fit the
 * array at once -- 9 bytes per token of n_seqs * stride plus 12 per record, each part rounded up to 16 -- or the call
 * returns ECHO_ENOMEM and says how much was asked for; unlike echo_grpo_tensors it does not run in passes.  Other
 * errors as echo_grpo_tensors (ECHO_ESTATE during a rollout on the same context).  Every call on a GPU, whatever its
 * context, uses that GPU's one array, which keeps the previous call's contents (nothing in it needs to start from
 * zero): calls that overlap in time on one GPU race; serialise them. */
#define ECHO_STATIC_SCRATCH_BYTES (32u << 20)
int echo_grpo_tensors_static(echo_ctx *ctx, const int32_t *tokens, int32_t stride, const int32_t *lens, int32_t n_seqs,
                             int32_t G, int32_t turn_start_id, const float *rewards, float eps, uint8_t *out_mask,
                             float *out_adv, float *out_adv_tok);

/* Raw 32-bit draws of the sampler's generator for (seed; n, s, i = i0..i0+count-1), computed on the GPU
 * (out: host [count]).  Exists so that the generator can be compared bit for bit with its definition. */
int echo_debug_draw_bits(echo_ctx *ctx, uint64_t seed, uint32_t n, uint32_t s, uint32_t i0, int32_t count,
                         uint32_t *out_bits);

int echo_stats(echo_ctx *ctx, echo_stats_t *out);

/* Durations in milliseconds of the decode steps of the last echo_rollout that ran with time_steps = 1, in step order
 * (entry k: decode step k + 1, i.e. the pass that produced generated token k + 1): out_ms host [cap].  Returns the
 * number of steps that were timed (which may exceed cap; only cap entries are written), or a negative echo_status. */
int echo_step_times(echo_ctx *ctx, float *out_ms, int32_t cap);

/* Message for the last error on this context (ctx-owned, valid until the next call); "" if none.
 * With ctx == NULL: the message of the last failed echo_init on this thread. */
const char *echo_last_error(const echo_ctx *ctx);

void echo_destroy(echo_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* ECHO_H_ */
