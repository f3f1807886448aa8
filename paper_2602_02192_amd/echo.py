"""ctypes binding of the C-ABI library (include/echo.h).  Argument marshalling only: every step of
the rollout runs in the library's HIP kernels.  PyTorch provides the device arena and the streams.

Importing this module loads paper_2602_02192_amd/libecho_hip.so and raises if it is missing:
there is no CPU fallback."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch  # noqa: F401  -- first: the library must bind to the HIP runtime PyTorch has already loaded,
#                              so that the arena and the streams belong to the runtime its kernels run on

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libecho_hip.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2602_02192_amd.build` "
                      "(the rollout path has no fallback without the HIP library)")
lib = C.CDLL(_LIB_PATH)

ECHO_OK, ECHO_EINVAL, ECHO_ENOMEM, ECHO_ESTATE, ECHO_EHIP = 0, -1, -2, -3, -4
ECHO_F32, ECHO_BF16 = 0, 1


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("dtype", C.c_int32), ("qk_norm", C.c_int32), ("tie_embeddings", C.c_int32),
                ("max_seqs", C.c_int32), ("max_ctx", C.c_int32), ("n_weight_slots", C.c_int32),
                ("debug_naive", C.c_int32)]


class RolloutOpts(C.Structure):
    _fields_ = [("stop_lens", C.c_void_p), ("eos_id", C.c_int32), ("top_p", C.c_float),
                ("n_swaps", C.c_int32), ("swap_at_step", C.c_void_p), ("swap_timeout_ms", C.c_int32),
                ("forced_tokens", C.c_void_p), ("debug_logits", C.c_void_p),
                ("unfused_sampler", C.c_int32), ("no_graph", C.c_int32), ("time_kernels", C.c_int32), ("time_steps", C.c_int32), ("no_compaction", C.c_int32),
                ("attn_plain", C.c_int32), ("own_prompt_copy", C.c_int32), ("prefix_kernel", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("active_version", C.c_int64), ("staged_version", C.c_int64),
                ("decode_steps", C.c_int32), ("prefill_ms", C.c_float), ("decode_ms", C.c_float),
                ("total_ms", C.c_float), ("swap_wait_ms", C.c_float),
                ("attn_launches", C.c_int64), ("attn_ms", C.c_double), ("attn_bytes", C.c_double),
                ("gemm_launches", C.c_int64), ("gemm_ms", C.c_double), ("gemm_bytes", C.c_double),
                ("rollout_running", C.c_int32), ("attn_rows_per_workgroup", C.c_int32), ("attn_prefix_jobs", C.c_int32)]


EXPORTS = ["echo_arena_bytes", "echo_blob_bytes", "echo_init", "echo_load_policy", "echo_load_policy_begin",
           "echo_load_policy_chunk", "echo_load_policy_commit", "echo_load_policy_abort", "echo_load_policy_delta", "echo_q8_blob_bytes", "echo_load_policy_q8", "echo_load_policy_q8_begin", "echo_rollout", "echo_rollout_continuous",
           "echo_logprobs", "echo_grpo_tensors", "echo_grpo_tensors_static", "echo_debug_draw_bits", "echo_stats", "echo_step_times", "echo_last_error", "echo_destroy"]

lib.echo_arena_bytes.restype = C.c_size_t
lib.echo_arena_bytes.argtypes = [C.POINTER(ModelDesc)]
lib.echo_blob_bytes.restype = C.c_size_t
lib.echo_blob_bytes.argtypes = [C.POINTER(ModelDesc)]
lib.echo_init.argtypes = [C.POINTER(ModelDesc), C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p,
                          C.POINTER(C.c_void_p)]
lib.echo_load_policy.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t]
lib.echo_load_policy_begin.argtypes = [C.c_void_p, C.c_int64, C.c_size_t]
lib.echo_load_policy_chunk.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
lib.echo_load_policy_commit.argtypes = [C.c_void_p]
lib.echo_load_policy_abort.argtypes = [C.c_void_p]
lib.echo_q8_blob_bytes.restype = C.c_size_t
lib.echo_q8_blob_bytes.argtypes = [C.POINTER(ModelDesc)]
lib.echo_load_policy_q8.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t]
lib.echo_load_policy_q8_begin.argtypes = [C.c_void_p, C.c_int64, C.c_size_t]
lib.echo_load_policy_delta.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
lib.echo_rollout.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                             C.c_float, C.c_uint64, C.POINTER(RolloutOpts), C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_void_p]
lib.echo_rollout_continuous.argtypes = lib.echo_rollout.argtypes
lib.echo_logprobs.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_float, C.c_void_p]
lib.echo_grpo_tensors.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
lib.echo_grpo_tensors_static.argtypes = lib.echo_grpo_tensors.argtypes
STATIC_SCRATCH_BYTES = 32 << 20
lib.echo_debug_draw_bits.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int32,
                                     C.c_void_p]
lib.echo_stats.argtypes = [C.c_void_p, C.POINTER(Stats)]
lib.echo_step_times.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
lib.echo_last_error.restype = C.c_char_p
lib.echo_last_error.argtypes = [C.c_void_p]
lib.echo_destroy.argtypes = [C.c_void_p]


class EchoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"echo error {code}: {msg}")
        self.code = code


def desc_from_shape(shape, max_seqs: int, max_ctx: int, n_weight_slots: int = 1,
                    debug_naive: bool = False) -> ModelDesc:
    return ModelDesc(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                     shape.ffn, shape.vocab, shape.rms_eps, shape.rope_base,
                     ECHO_F32 if shape.dtype == "fp32" else ECHO_BF16, int(shape.qk_norm),
                     int(shape.tie_embeddings), max_seqs, max_ctx, n_weight_slots, int(debug_naive))


def arena_bytes(desc: ModelDesc) -> int:
    return int(lib.echo_arena_bytes(C.byref(desc)))


def blob_bytes(desc: ModelDesc) -> int:
    return int(lib.echo_blob_bytes(C.byref(desc)))


def q8_blob_bytes(desc: ModelDesc) -> int:
    return int(lib.echo_q8_blob_bytes(C.byref(desc)))


def _ptr(a: Optional[np.ndarray]):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


class Context:
    """echo_init / echo_destroy plus the calls of include/echo.h with numpy marshalling."""

    def __init__(self, desc: ModelDesc, device: int = 0, compute_stream=None, copy_stream=None):
        need = arena_bytes(desc)
        if need == 0:
            h = C.c_void_p()
            rc = lib.echo_init(C.byref(desc), device, None, 0, None, None, C.byref(h))
            raise EchoError(rc, lib.echo_last_error(None).decode())
        self.desc = desc
        self.device = device
        self.arena = torch.empty(need + 256, dtype=torch.uint8, device=f"cuda:{device}")
        base = (self.arena.data_ptr() + 255) // 256 * 256
        self._streams = (compute_stream, copy_stream)
        cs = compute_stream.cuda_stream if compute_stream is not None else None
        ks = copy_stream.cuda_stream if copy_stream is not None else None
        h = C.c_void_p()
        rc = lib.echo_init(C.byref(desc), device, C.c_void_p(base), need, cs, ks, C.byref(h))
        if rc != 0:
            raise EchoError(rc, lib.echo_last_error(None).decode())
        self.h = h

    def _chk(self, rc: int) -> None:
        if rc != 0:
            raise EchoError(rc, lib.echo_last_error(self.h).decode())

    def close(self) -> None:
        if getattr(self, "h", None):
            lib.echo_destroy(self.h)
            self.h = None
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def load_policy(self, version: int, blob) -> None:
        """blob: host torch tensor or numpy array holding the flat weights in the model dtype."""
        if isinstance(blob, torch.Tensor):
            if blob.device.type != "cpu":
                raise ValueError("echo_load_policy takes a host blob")
            blob = blob.contiguous()
            ptr, nbytes = blob.data_ptr(), blob.numel() * blob.element_size()
        else:
            blob = np.ascontiguousarray(blob)
            ptr, nbytes = blob.ctypes.data, blob.nbytes
        self._chk(lib.echo_load_policy(self.h, version, C.c_void_p(ptr), nbytes))

    def load_policy_chunked(self, version: int, blob, chunk_sizes, between=None) -> None:
        """The same blob handed over in pieces of the given byte sizes (cycled until the blob ends); `between`,
        if given, is called after every piece."""
        if isinstance(blob, torch.Tensor):
            blob = blob.contiguous()
            ptr, nbytes = blob.data_ptr(), blob.numel() * blob.element_size()
        else:
            blob = np.ascontiguousarray(blob)
            ptr, nbytes = blob.ctypes.data, blob.nbytes
        self._chk(lib.echo_load_policy_begin(self.h, version, nbytes))
        try:
            off, k = 0, 0
            while off < nbytes:
                n = min(int(chunk_sizes[k % len(chunk_sizes)]), nbytes - off)
                self._chk(lib.echo_load_policy_chunk(self.h, C.c_void_p(ptr + off), n))
                off += n
                k += 1
                if between is not None:
                    between()
            self._chk(lib.echo_load_policy_commit(self.h))
        except Exception:
            lib.echo_load_policy_abort(self.h)
            raise

    def load_policy_delta(self, base_version: int, version: int, offsets, sizes, data) -> None:
        """data: the new bytes of the ranges, concatenated (numpy uint8 array or bytes)."""
        offsets = np.ascontiguousarray(offsets, np.uint64)
        sizes = np.ascontiguousarray(sizes, np.uint64)
        data = np.ascontiguousarray(np.frombuffer(data, np.uint8) if isinstance(data, (bytes, bytearray)) else data, np.uint8)
        assert offsets.shape == sizes.shape and data.size == int(sizes.sum())
        self._chk(lib.echo_load_policy_delta(self.h, base_version, version, offsets.size, _ptr(offsets), _ptr(sizes), _ptr(data)))

    def load_policy_q8(self, version: int, blob) -> None:
        """blob: numpy uint8 array in the quantised layout (per-row fp32 scales and int8 codes for every matrix)."""
        blob = np.ascontiguousarray(blob, np.uint8)
        self._chk(lib.echo_load_policy_q8(self.h, version, C.c_void_p(blob.ctypes.data), blob.nbytes))

    def load_policy_q8_chunked(self, version: int, blob, chunk_sizes) -> None:
        """The quantised blob handed over in pieces of the given byte sizes (cycled until the blob ends)."""
        blob = np.ascontiguousarray(blob, np.uint8)
        self._chk(lib.echo_load_policy_q8_begin(self.h, version, blob.nbytes))
        try:
            off, k = 0, 0
            while off < blob.nbytes:
                n = min(int(chunk_sizes[k % len(chunk_sizes)]), blob.nbytes - off)
                self._chk(lib.echo_load_policy_chunk(self.h, C.c_void_p(blob.ctypes.data + off), n))
                off += n
                k += 1
            self._chk(lib.echo_load_policy_commit(self.h))
        except Exception:
            lib.echo_load_policy_abort(self.h)
            raise

    def load_policy_begin(self, version: int, nbytes: int) -> None:
        self._chk(lib.echo_load_policy_begin(self.h, version, nbytes))

    def load_policy_chunk(self, data: np.ndarray) -> None:
        data = np.ascontiguousarray(data)
        self._chk(lib.echo_load_policy_chunk(self.h, C.c_void_p(data.ctypes.data), data.nbytes))

    def load_policy_commit(self) -> None:
        self._chk(lib.echo_load_policy_commit(self.h))

    def load_policy_abort(self) -> None:
        self._chk(lib.echo_load_policy_abort(self.h))

    def rollout(self, prompts, prompt_lens, G: int, max_new: int, temperature: float, seed: int,
                stop_lens=None, eos_id: int = -1, top_p: float = 1.0, swap_at_step: Sequence[int] = (),
                swap_timeout_ms: int = 0, forced=None, want_logits: bool = False, unfused_sampler: bool = False,
                no_graph: bool = False, time_kernels: bool = False, continuous: bool = False, attn_plain: bool = False,
                own_prompt_copy: bool = False, prefix_kernel: int = 0, time_steps: bool = False,
                no_compaction: bool = False) -> dict:
        prompts = np.ascontiguousarray(prompts, np.int32)
        prompt_lens = np.ascontiguousarray(prompt_lens, np.int32)
        P = prompts.shape[0]
        N = P * G
        o = RolloutOpts()
        o.eos_id, o.top_p = eos_id, top_p
        keep = []
        if stop_lens is not None:
            a = np.ascontiguousarray(stop_lens, np.int32)
            assert a.shape == (N,)
            keep.append(a)
            o.stop_lens = a.ctypes.data
        sw = np.ascontiguousarray(list(swap_at_step), np.int32)
        keep.append(sw)
        o.n_swaps = sw.size
        o.swap_at_step = sw.ctypes.data if sw.size else None
        o.swap_timeout_ms = swap_timeout_ms
        if forced is not None:
            f = np.ascontiguousarray(forced, np.int32)
            assert f.shape == (N, max_new)
            keep.append(f)
            o.forced_tokens = f.ctypes.data
        logits = None
        if want_logits:
            logits = np.zeros((N, max_new, self.desc.vocab), np.float32)
            o.debug_logits = logits.ctypes.data
        o.unfused_sampler, o.no_graph, o.time_kernels = int(unfused_sampler), int(no_graph), int(time_kernels)
        o.attn_plain, o.own_prompt_copy, o.prefix_kernel = int(attn_plain), int(own_prompt_copy), int(prefix_kernel)
        o.time_steps, o.no_compaction = int(time_steps), int(no_compaction)
        toks = np.empty((N, max_new), np.int32)
        lps = np.empty((N, max_new), np.float32)
        lens = np.empty(N, np.int32)
        vers = np.empty((N, max_new), np.int64)
        fn = lib.echo_rollout_continuous if continuous else lib.echo_rollout
        self._chk(fn(self.h, _ptr(prompts), prompts.shape[1], _ptr(prompt_lens), P, G, max_new,
                     temperature, seed, C.byref(o), _ptr(toks), _ptr(lps), _ptr(lens), _ptr(vers)))
        return dict(tokens=toks, logprobs=lps, lens=lens, versions=vers, logits=logits)

    def logprobs(self, tokens, lens, temperature: float = 1.0) -> np.ndarray:
        tokens = np.ascontiguousarray(tokens, np.int32)
        lens = np.ascontiguousarray(lens, np.int32)
        out = np.zeros(tokens.shape, np.float32)
        self._chk(lib.echo_logprobs(self.h, _ptr(tokens), tokens.shape[1], _ptr(lens), tokens.shape[0], temperature,
                                    _ptr(out)))
        return out

    def grpo_tensors(self, tokens, lens, G: int, turn_start_id: int, rewards, eps: float = 1e-6, per_token: bool = True,
                     static_scratch: bool = False):
        tokens = np.ascontiguousarray(tokens, np.int32)
        lens = np.ascontiguousarray(lens, np.int32)
        rewards = np.ascontiguousarray(rewards, np.float32)
        mask = np.empty(tokens.shape, np.uint8)
        adv = np.empty(tokens.shape[0], np.float32)
        adv_tok = np.empty(tokens.shape, np.float32) if per_token else None
        fn = lib.echo_grpo_tensors_static if static_scratch else lib.echo_grpo_tensors
        self._chk(fn(self.h, _ptr(tokens), tokens.shape[1], _ptr(lens), tokens.shape[0], G, turn_start_id,
                                        _ptr(rewards), eps, _ptr(mask), _ptr(adv), _ptr(adv_tok) if per_token else None))
        return mask, adv, adv_tok

    def draw_bits(self, seed: int, n: int, s: int, i0: int, count: int) -> np.ndarray:
        out = np.empty(count, np.uint32)
        self._chk(lib.echo_debug_draw_bits(self.h, seed, n, s, i0, count, _ptr(out)))
        return out

    def step_times(self) -> np.ndarray:
        """Per-step durations (ms) of the last rollout that ran with time_steps."""
        n = lib.echo_step_times(self.h, None, 0)
        if n < 0:
            self._chk(n)
        out = np.zeros(max(n, 0), np.float32)
        if n > 0:
            lib.echo_step_times(self.h, _ptr(out), n)
        return out

    def stats(self) -> Stats:
        st = Stats()
        self._chk(lib.echo_stats(self.h, C.byref(st)))
        return st


# ---- pool capacity and dissemination arithmetic (include/echo_capacity.h; host only) -------------------------
CAPACITY_EXPORTS = ["echo_mu_min", "echo_overlap_holds", "echo_staleness_bound", "echo_greedy_activate", "echo_peer_score",
                    "echo_n_chains", "echo_chain_assign"]
lib.echo_mu_min.restype = C.c_double
lib.echo_mu_min.argtypes = [C.c_double] * 4
lib.echo_overlap_holds.restype = C.c_int32
lib.echo_overlap_holds.argtypes = [C.c_double] * 5
lib.echo_staleness_bound.restype = C.c_int32
lib.echo_staleness_bound.argtypes = [C.c_int32, C.c_double, C.c_double, C.c_double, C.c_double]
lib.echo_greedy_activate.restype = C.c_int32
lib.echo_greedy_activate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
lib.echo_peer_score.restype = C.c_double
lib.echo_peer_score.argtypes = [C.c_double, C.c_double, C.c_int32, C.c_int32, C.c_double]
lib.echo_n_chains.restype = C.c_int32
lib.echo_n_chains.argtypes = [C.c_double, C.c_double]
lib.echo_chain_assign.restype = C.c_int32
lib.echo_chain_assign.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]


def mu_min(kappa, R, T_train, T_bcast) -> float:
    return lib.echo_mu_min(kappa, R, T_train, T_bcast)


def overlap_holds(kappa, R, T_train, T_bcast, mu_pool) -> int:
    return lib.echo_overlap_holds(kappa, R, T_train, T_bcast, mu_pool)


def staleness_bound(kappa: int, R, T_train, T_bcast, mu_pool) -> int:
    return lib.echo_staleness_bound(kappa, R, T_train, T_bcast, mu_pool)


def greedy_activate(mu, cost, mu_target, available=None):
    """(active flags, activated throughput, activated cost, return code of echo_greedy_activate)."""
    mu = np.ascontiguousarray(mu, np.float64)
    cost = np.ascontiguousarray(cost, np.float64)
    av = np.ascontiguousarray(available, np.int32) if available is not None else None
    active = np.zeros(mu.size, np.int32)
    got, paid = C.c_double(), C.c_double()
    rc = lib.echo_greedy_activate(_ptr(mu), _ptr(cost), _ptr(av), mu.size, mu_target, _ptr(active), C.addressof(got), C.addressof(paid))
    return active, got.value, paid.value, rc


def peer_score(avg_speed, success_rate, consecutive_failures: int, succ_count: int, elapsed_s) -> float:
    return lib.echo_peer_score(avg_speed, success_rate, consecutive_failures, succ_count, elapsed_s)


def n_chains(B0, Bw) -> int:
    return lib.echo_n_chains(B0, Bw)


def chain_assign(score, chains: int):
    score = np.ascontiguousarray(score, np.float64)
    chain = np.zeros(score.size, np.int32)
    hop = np.zeros(score.size, np.int32)
    rc = lib.echo_chain_assign(_ptr(score), score.size, chains, _ptr(chain), _ptr(hop))
    if rc != 0:
        raise ValueError("echo_chain_assign: bad arguments")
    return chain, hop
