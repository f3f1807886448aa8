// echo_grpo_tensors for callers that cannot allocate: the staging of the records (device memory beyond the caller's inputs
// and outputs, which echo_grpo_tensors borrows from the context's arena) lives in a file-scope device array of the
// library.  Every GPU the library runs on holds its own copy of the array until the process ends; its address there is
// looked up once per device, at echo_init, and only that address is ever handed to copies and kernels.
#include "echo_engine_impl.h"

static __device__ __align__(256) unsigned char scratch[ECHO_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[MAX_DEVICES] = {};   // per device: where that GPU's copy of `scratch` lives
}  // namespace

// Called by echo_init with `device` current.  0, or the HIP error of the lookup.
int echo_static_scratch_resolve(int device) {
  if (device < 0 || device >= MAX_DEVICES) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[device]) return 0;
  unsigned char *ptr = nullptr;
  hipError_t e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return (int)e;
  if (!ptr) return (int)hipErrorInvalidSymbol;
  g_scratch_ptr[device] = ptr;
  return 0;
}

extern "C" int echo_grpo_tensors_static(echo_ctx *c, const int32_t *tokens, int32_t stride, const int32_t *lens, int32_t n_seqs, int32_t G,
                                        int32_t turn_start_id, const float *rewards, float eps, uint8_t *out_mask, float *out_adv,
                                        float *out_adv_tok) {
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
  // tokens i32 [n, stride] | adv_tok f32 [n, stride] | mask u8 [n, stride] | lens i32 [n] | rewards f32 [n] | adv f32 [n]
  auto up16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
  const size_t ns = (size_t)n_seqs, cells = ns * (size_t)stride;
  const size_t need = 2 * up16(cells * 4) + up16(cells) + 3 * up16(ns * 4);
  if (need > (size_t)ECHO_STATIC_SCRATCH_BYTES)
    return fail(c, ECHO_ENOMEM, "%d x %d tokens need %zu bytes of staging, the static scratch holds %zu (use echo_grpo_tensors, or fewer records per call)",
                n_seqs, stride, need, (size_t)ECHO_STATIC_SCRATCH_BYTES);
  unsigned char *base;
  {
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    base = c->device < MAX_DEVICES ? g_scratch_ptr[c->device] : nullptr;
  }
  if (!base) return fail(c, ECHO_ESTATE, "the static scratch of device %d was not resolved at echo_init", c->device);
  HIPCHK(c, hipSetDevice(c->device));
  hipStream_t st = c->cs;
  int32_t *d_tok = (int32_t *)base;
  float *d_at = (float *)(base + up16(cells * 4));
  uint8_t *d_mask = (uint8_t *)(base + 2 * up16(cells * 4));
  int32_t *d_len = (int32_t *)((unsigned char *)d_mask + up16(cells));
  float *d_rew = (float *)((unsigned char *)d_len + up16(ns * 4));
  float *d_adv = (float *)((unsigned char *)d_rew + up16(ns * 4));
  // (nothing in the scratch has to start at zero: every byte that is read back below is written by this call first)
  HIPCHK(c, hipMemcpyAsync(d_tok, tokens, cells * 4, hipMemcpyHostToDevice, st));
  HIPCHK(c, hipMemcpyAsync(d_len, lens, ns * 4, hipMemcpyHostToDevice, st));
  HIPCHK(c, hipMemcpyAsync(d_rew, rewards, ns * 4, hipMemcpyHostToDevice, st));
  launch_grpo_tensors(d_mask, d_adv, out_adv_tok ? d_at : nullptr, d_tok, d_len, d_rew, n_seqs, G, stride, turn_start_id, eps, st);
  HIPCHK(c, hipGetLastError());
  HIPCHK(c, hipMemcpyAsync(out_mask, d_mask, cells, hipMemcpyDeviceToHost, st));
  HIPCHK(c, hipMemcpyAsync(out_adv, d_adv, ns * 4, hipMemcpyDeviceToHost, st));
  if (out_adv_tok) HIPCHK(c, hipMemcpyAsync(out_adv_tok, d_at, cells * 4, hipMemcpyDeviceToHost, st));
  HIPCHK(c, hipStreamSynchronize(st));
  return ECHO_OK;
}
