// Internal launcher interface between the engine and the HIP kernels (not part of the C ABI).
// Every launcher enqueues on `st` and returns; shapes are validated by the engine before the call.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace echo {

// ------------------------------------------------------------------------------------------------
// Layouts of the MFMA path (model dtype bf16; MFMA operands are half precision, see echo_device.h).
//   packed weight  Wp: rows padded to 32, K padded to GEMM_K_PAD.  Element (r,k) lives at
//       ((((r/32)*(Kp/8) + k/8)*32 + r%32)*8 + k%8)            -- one 32-row block is contiguous over K,
//       and a wavefront's MFMA A-operand load (32 rows x 16 k) is one contiguous 1 KiB read.
//   packed activation Xp ("K8", halves): M padded to 32.  Element (m,k) lives at ((k/8)*Mp + m)*8 + k%8.
//   split-K partials P: [split][Mp][Np] fp32, row-major.
// ------------------------------------------------------------------------------------------------
static inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

struct RowState {        // device arrays, one entry per row of the current batch of rows
  int32_t *token;        // token fed at this row (-1: padding row)
  int32_t *slot;         // KV-cache sequence slot of the row
  int32_t *pos;          // position of the token inside its sequence
  int32_t *active;       // 0: row is skipped (finished sequence or padding)
  int32_t *pslot;        // slot whose first ptiles key tiles equal this row's (its group's prompt); read by the split-K
  int32_t *ptiles;       //   attention kernel only, which takes those tiles from pslot so that a group shares them in cache
};

struct KvGeom {          // KV cache, plain form: [slot][layer][K|V][kv_head][max_ctx][head_dim]
  void *base;
  int32_t n_layers, n_kv_heads, max_ctx, head_dim, elt_bytes;
  int32_t tiled;         // 1: the MFMA path's form (same size, max_ctx a multiple of 32), see below
  __host__ __device__ int64_t head_stride() const { return (int64_t)max_ctx * head_dim; }
  __host__ __device__ int64_t kv_stride() const { return head_stride() * n_kv_heads; }
  __host__ __device__ int64_t layer_stride() const { return kv_stride() * 2; }
  __host__ __device__ int64_t slot_stride() const { return layer_stride() * n_layers; }
  // Tiled form: [slot][layer][kv_head][tile of 32 keys][K tile | V tile].  Both tiles are stored in the order the
  // attention kernel's MFMA operands want them, so a wavefront reads a tile as head_dim/16 contiguous 1 KiB loads
  // per operand, straight into registers.  In 16-byte units (8 halves):
  //   K tile: unit (dim/8)*32 + key%32 holds dims 8*(dim/8).. of one key            (A operand of K Q^T)
  //   V tile: unit (((key%32)/16 * (hd/32) + dim/32)*2 + (key%16)/8)*32 + dim%32 holds 8 keys of one dim (A operand of V^T P^T)
  __host__ __device__ int64_t tiled_head_off(int slot, int layer, int kvh) const {
    return (int64_t)slot * slot_stride() + (int64_t)layer * layer_stride() + (int64_t)kvh * 2 * head_stride();
  }
  __host__ __device__ int64_t tiled_k_off(int key, int dim) const {
    return (int64_t)(key >> 5) * 64 * head_dim + ((dim >> 3) * 32 + (key & 31)) * 8 + (dim & 7);
  }
  __host__ __device__ int64_t tiled_v_off(int key, int dim) const {
    int k = key & 31;
    return (int64_t)(key >> 5) * 64 * head_dim + 32 * head_dim +
           ((((k >> 4) * (head_dim >> 5) + (dim >> 5)) * 2 + ((k >> 3) & 1)) * 32 + (dim & 31)) * 8 + (k & 7);
  }
};

// ---- shared small kernels (both paths) -----------------------------------------------------------
void launch_rope_table(float *cs /*[M][hd/2][2]*/, const int32_t *pos, int M, int hd, float base, hipStream_t st);
void launch_bookkeeping(int N, int max_new, int per_row /*1: a row's step is its gen_len*/, int32_t *d_step, const int32_t *samp_tok, const float *samp_lp,
                        const int32_t *forced, const int32_t *limit, int eos, int64_t version,
                        const int32_t *prompt_len, int32_t *gen_len, RowState rows, int32_t *out_tok,
                        float *out_lp, int64_t *out_ver, int32_t *n_active, hipStream_t st);
void launch_kv_replicate(KvGeom kv, const int32_t *prompt_len /*[P]*/, int P, int G, hipStream_t st);
void launch_draw_bits(uint32_t *out, uint64_t seed, uint32_t n, uint32_t s, uint32_t i0, int count, hipStream_t st);
// quads: device [n_quads][4] = (src slot, dst slot, begin, end); copies keys [begin, end) (plain cache) or whole tiles
// of 32 keys [begin, end) (tiled cache) of every layer and head from the source slot to the destination slot.
void launch_kv_copy_ranges(KvGeom kv, const int32_t *quads, int n_quads, hipStream_t st);
void launch_fill_i32(int32_t *p, int32_t v, int64_t n, hipStream_t st);
// Which draw of the generator a row takes (the step and stream words of its counter).  In a rollout whose sequences
// all start together every row sits at the step *d_step and row m is stream m; with row_step / row_stream set the
// two are read per row (sequences that join a running batch).
struct DrawIds {
  const int32_t *d_step;      // device scalar
  const int32_t *row_step;    // device [rows], or null
  const int32_t *row_stream;  // device [rows], or null
};
// Learner-side tensors of n_seqs records in groups of G (n_seqs a multiple of G, G >= 2): adv[n] from rewards[n],
// mask[n][t] and adv_tok[n][t] (nullable) from tokens[n][t], lens[n].  tokens, adv_tok 16-byte aligned, mask 4-byte.
void launch_grpo_tensors(uint8_t *mask, float *adv, float *adv_tok, const int32_t *tokens, const int32_t *lens, const float *rewards,
                         int n_seqs, int G, int stride, int32_t turn_start, float eps, hipStream_t st);
void launch_gather_rows_f32(float *dst, const float *src, const int32_t *src_row /*[n_dst], -1 = skip*/,
                            int n_dst, int width, hipStream_t st);

// ---- debug path: row-major weights (fp32 or bf16), fp32 activations, fp32 KV cache ------------------
void dbg_embed(float *h, const void *embed, int w_bf16, const int32_t *token, int M, int d, hipStream_t st);
void dbg_rmsnorm(float *x, const float *h, const void *gain, int w_bf16, int M, int d, float eps, hipStream_t st);
// Y[m][n] (+)= sum_k X[m][k] * W[n][k]
void dbg_gemm(float *Y, const float *X, const void *W, int w_bf16, int M, int N, int K, int accumulate, hipStream_t st);
void dbg_qkv_post(float *qkv /*[M][(Hq+2Hkv)*hd], q rotated in place*/, const void *q_gain, const void *k_gain,
                  int w_bf16, int qk_norm, float eps, const float *rope_cs, RowState rows, KvGeom kv, int layer,
                  int M, int Hq, int Hkv, hipStream_t st);
void dbg_attention(float *out /*[M][Hq*hd]*/, const float *qkv, RowState rows, KvGeom kv, int layer, int M, int Hq,
                   int Hkv, hipStream_t st);
void dbg_swiglu(float *ff /*[M][F]*/, const float *gu /*[M][2F] = gate | up*/, int M, int F, hipStream_t st);
// Unfused sampler over materialised logits [M][ld]: Gumbel-max token and its log-softmax, in fp32.
void dbg_sample(int32_t *tok, float *lp, const float *logits, int64_t ld, int M, int V, float temperature,
                uint64_t seed, DrawIds ids, const int32_t *row_active, hipStream_t st);
// log softmax(logits/T)[target[m]] per row (teacher-forced scoring).
void dbg_target_logprob(float *lp, const float *logits, int64_t ld, int M, int V, float temperature,
                        const int32_t *target, hipStream_t st);

// ---- MFMA path -------------------------------------------------------------------------------
// Repack a row-major bf16 chunk `src` [n_rows][K] into the packed weight `dst` (halves, scaled by W_SCALE): source row i goes to
// destination row dst_row0 + i*dst_row_stride (stride 2 interleaves gate and up rows).  K % 8 == 0.
void fast_pack_weight(void *dst, const void *src, int64_t dst_row0, int dst_row_stride, int64_t n_rows, int K, int Kp,
                      int Np, hipStream_t st);
// The same for a span of elements [e0, e0 + n) of the row-major matrix (src holds those n values only): a delta install.
void fast_pack_span(void *dst, const void *src, int64_t e0, int64_t n, int64_t dst_row0, int dst_row_stride, int K, int Kp, int Np,
                    hipStream_t st);
// rows x K int8 codes with one fp32 scale per row -> row-major bf16 [rows][K] (any path; out, codes, scales on the device).
void fast_dequant_q8(void *out_bf16, const void *codes, const void *scales, int64_t rows, int K, hipStream_t st);
// h = embed[token] (first layer) or h += sum_s P[s] (+0); then x = rmsnorm(h)*gain -> Xp (half K8).
void fast_resid_norm(float *h, const void *embed_bf16, const int32_t *token, const float *partials, int nsplit,
                     int Np, void *Xp, const void *gain_bf16, int M, int Mp, int d, float eps, hipStream_t st);
enum GemmEpilogue { EPI_PARTIAL = 0, EPI_SWIGLU = 1 };
// out = Xp[Mp x Kp] * Wp[Np x Kp]^T.  EPI_PARTIAL: fp32 partials [nsplit][Mp][Np];
// EPI_SWIGLU (rows alternate gate_f, up_f): silu(gate)*up -> half K8 [Mp][Np/2]; nsplit must be 1.
struct GemmShape { int nsplit, waves_k, waves_n, nbw, lds, stages; };   // launch shape, see fast_gemm_pick
constexpr int REDUCE_MAX_SPLIT = 12;   // most grid splits over K whose partials the reducing kernels sum
constexpr int GEMM_K_PAD = 128;   // packed weights and K8 activations pad K to this (whole LDS chunks of 8 k-steps)
void fast_gemm(void *out, const void *Xp, const void *Wp, int Mp, int Np, int Kp, GemmShape g, GemmEpilogue epi,
               hipStream_t st);
int fast_gemm_even_split(int Kp, int nsplit);
void fast_gemm_pick(int Np, int Kp, int Mp, int full_k, GemmShape *g);
void fast_qkv_post(const float *partials, int nsplit, int Np, int Mp, void *q_h16 /*[M][Hq][hd]*/,
                   const void *q_gain, const void *k_gain, int qk_norm, float eps, const float *rope_cs,
                   RowState rows, KvGeom kv, int layer, int M, int Hq, int Hkv, hipStream_t st);
// Plain one-wavefront-per-(row, head) attention over the half-precision KV cache (cross-check of the split-K kernel).
void fast_attention_simple(void *Xp_out, const void *q_h16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq,
                           int Hkv, hipStream_t st);
// Split-K decode attention over the half-precision KV cache + combine; writes Xp (half K8 [Mp][Hq*hd]).
// The shared prompt of a group is attended once for all its sequences by a kernel of its own: a job is up to 32 / (Hq/Hkv)
// rows of one group (rows with RowState.ptiles >= 1 that read the prompt tiles of cache slot pslot).  Rows covered by a
// job carry ATT_PREFIX_DONE in RowState.ptiles; the decode kernel then starts after the shared tiles and folds the job's
// partials in.  np chunk slots per (row, head) in the partial buffers, tiles_per_chunk whole tiles per chunk
// (np * tiles_per_chunk >= the longest job's ptiles); n_jobs = 0: no such kernel, every row reads its shared tiles itself.
constexpr int ATT_PREFIX_DONE = 0x40000000;
struct PrefixJob { int32_t pslot, ptiles, nrows; int32_t rows[32]; };
struct PrefixPlan { const PrefixJob *jobs; int n_jobs, np, tiles_per_chunk; };
// nsplit = fast_attention_splits(M, Hkv, capacity); partial buffers hold M*Hq*max(nsplit, px.np)*(hd + 2) floats.
// With px.n_jobs > 0 and nsplit == 1, fast_attention_prefix must have run first on the same stream, partial buffers and q.
void fast_attention(void *Xp_out, const void *q_h16, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq,
                    int Hkv, int nsplit, float *part_o, float *part_ml, PrefixPlan px, hipStream_t st);
void fast_attention_prefix(const void *q_h16, KvGeom kv, int layer, int Hq, int Hkv, float *part_o, float *part_ml, PrefixPlan px,
                           hipStream_t st);
int fast_attention_splits(int M, int Hkv, int max_splits);
// Decode attention with several rows of the batch per workgroup (at most R, R * Hq/Hkv <= 32): the whole prompt tiles
// that neighbouring rows of one group have in common are loaded and multiplied once per workgroup.  No key splitting and no
// partial buffers.  fast_attention_rows_per_group gives R (1: use fast_attention) -- mode 0: a workgroup for every compute
// unit, and at least two rows for each; 1, 2: never; 3: as many rows as the MFMA columns hold.  fast_attention_rows_plan
// deals the generating rows to the workgroups and writes every workgroup's tile list (fast_attention_plan_ints(rows of
// the largest batch) ints) from the row state, once per decode step and before the first fast_attention_rows of that
// step on the same stream, with the same M and mode.
int fast_attention_rows_per_group(int M, int Hq, int Hkv, int mode);
size_t fast_attention_plan_ints(int max_rows);
void fast_attention_rows_plan(int32_t *plan, RowState rows, int M, int Hq, int Hkv, int mode, hipStream_t st);
void fast_attention_rows(void *Xp_out, const void *q_h16, const int32_t *plan, RowState rows, KvGeom kv, int layer, int M, int Mp, int Hq,
                         int Hkv, int mode, hipStream_t st);
// Causal attention for runs of consecutive positions (prefill, teacher-forced scoring).  A block is up to
// ATT_PREFILL_WAVES * ATT_PREFILL_COLS / (Hq/Hkv) rows m0 .. m0 + nrows - 1 holding positions pos0 .. of one cache
// slot, whose keys and values (positions 0 .. pos0 + nrows - 1) are already in the cache.  The blocks must cover
// every row once.
struct PrefillBlock { int32_t m0, nrows, slot, pos0; };
constexpr int ATT_PREFILL_COLS = 32;    // (row, query head) pairs of one KV head that one wavefront carries
constexpr int ATT_PREFILL_WAVES = 8;    // wavefronts of a workgroup, which share the block's K / V tiles
void fast_attention_prefill(void *Xp_out, const void *q_h16, const PrefillBlock *blocks, int nblocks, KvGeom kv, int layer,
                            int Mp, int Hq, int Hkv, hipStream_t st);
// lm_head with the sampler fused into the epilogue (partials per workgroup) + the combine kernel.  With `target` set
// (scoring) only target_lp is meaningful: no noise is drawn and tok / lp describe the plain argmax.
void fast_lmhead_sample(int32_t *tok, float *lp, float *target_lp, const void *Xp, const void *Wp, int Mp, int M,
                        int V, int Np, int Kp, float temperature, uint64_t seed, DrawIds ids,
                        const int32_t *row_active, const int32_t *target, float *partials, hipStream_t st);
size_t fast_lmhead_partial_floats(int Np, int Mp);
// Nucleus sampling over fp32 logits [M][ld] (top_p < 1): finds every row's cut and leaves the sampler's partials of
// TOPP_CHUNKS vocabulary slices per row in scratch (fast_topp_scratch_floats(Mp) floats), in the layout that
// fast_sample_combine merges into the token and its log-prob under the renormalised kept set.
constexpr int TOPP_CHUNKS_PER_ROW = 16;
size_t fast_topp_scratch_floats(int Mp);
void fast_topp_cut_and_draw(float *scratch, const float *logits, int64_t ld, int M, int Mp, int V, float temperature, float top_p,
                            uint64_t seed, DrawIds ids, const int32_t *row_active, hipStream_t st);
void fast_sample_combine(int32_t *tok, float *lp, const float *part, int n_parts, int M, int Mp, const int32_t *row_active, hipStream_t st);
// lm_head writing fp32 logits [Mp][ld] row-major (debug / unfused sampler).
void fast_lmhead_logits(float *logits, int64_t ld, const void *Xp, const void *Wp, int Mp, int Np, int Kp, int V,
                        hipStream_t st);

}  // namespace echo
