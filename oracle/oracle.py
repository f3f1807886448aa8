"""ctypes access to the CPU oracle (test infrastructure; never imported by the
product package).  `load("f64")` is the parity reference, `load("f32")` the
all-fp32 build of the same source."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

from . import build as _build


class Desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("qk_norm", C.c_int32), ("tie_embeddings", C.c_int32)]


def desc_from_shape(s) -> Desc:
    return Desc(s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn, s.vocab,
                s.rms_eps, s.rope_base, int(s.qk_norm), int(s.tie_embeddings))


_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")


class Oracle:
    def __init__(self, precision: str = "f64"):
        path = _build.lib_path(precision)
        if os.environ.get("ORACLE_SANITIZE") == "1":     # the ASan + UBSan builds (oracle/build.py: build_sanitized)
            path = os.path.join(os.path.dirname(path), f"liboracle_{precision}_san.so")
            if not os.path.exists(path):
                raise RuntimeError(f"ORACLE_SANITIZE=1 needs {path} (oracle/build.py: build_sanitized)")
        elif not os.path.exists(path):
            _build.build(force=False)
        self.lib = L = C.CDLL(path)
        self.precision = precision
        L.orc_blob_numel.restype = C.c_int64
        L.orc_blob_numel.argtypes = [C.POINTER(Desc)]
        L.orc_draw_bits.restype = C.c_uint32
        L.orc_draw_bits.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_uniform.restype = C.c_float
        L.orc_uniform.argtypes = [C.c_uint32]
        L.orc_gumbel.restype = C.c_float
        L.orc_gumbel.argtypes = [C.c_float]
        L.orc_silu_d.restype = C.c_double
        L.orc_silu_d.argtypes = [C.c_double]
        L.orc_forward_cached.argtypes = [C.POINTER(Desc), _f32p, _i32p, C.c_int, _f64p]
        L.orc_forward_full.argtypes = [C.POINTER(Desc), _f32p, _i32p, C.c_int, _f64p]
        L.orc_logprobs.argtypes = [C.POINTER(Desc), _f32p, _i32p, C.c_int, C.c_float, _f64p]
        L.orc_rmsnorm_d.argtypes = [_f64p, _f64p, _f32p, C.c_int, C.c_float]
        L.orc_rope_d.argtypes = [_f64p, C.c_int, C.c_int, C.c_float]
        L.orc_attend_d.argtypes = [_f64p, _f64p, _f64p, _f64p, C.c_int, C.c_int]
        L.orc_log_softmax_d.argtypes = [_f64p, _f64p, C.c_int, C.c_float]
        L.orc_sample_d.argtypes = [_f64p, C.c_int, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                   C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_float)]
        L.orc_rollout.restype = C.c_int
        L.orc_set_threads.argtypes = [C.c_int]
        L.orc_set_progress_file.argtypes = [C.c_char_p]
        L.orc_get_threads.restype = C.c_int

    # -- primitives -------------------------------------------------------------------
    def philox(self, ctr: Sequence[int], key: Sequence[int]) -> np.ndarray:
        c = (C.c_uint32 * 4)(*ctr)
        k = (C.c_uint32 * 2)(*key)
        o = (C.c_uint32 * 4)()
        self.lib.orc_philox4x32(c, k, o)
        return np.array(list(o), dtype=np.uint32)

    def draw_bits(self, seed: int, n: int, s: int, i: int) -> int:
        return int(self.lib.orc_draw_bits(seed, n, s, i))

    def uniform(self, bits: int) -> float:
        return float(self.lib.orc_uniform(bits))

    def gumbel(self, u: float) -> float:
        return float(self.lib.orc_gumbel(u))

    def silu(self, x: float) -> float:
        return float(self.lib.orc_silu_d(x))

    def rmsnorm(self, x, g, eps: float) -> np.ndarray:
        x = np.ascontiguousarray(x, np.float64)
        y = np.empty_like(x)
        self.lib.orc_rmsnorm_d(y, x, np.ascontiguousarray(g, np.float32), x.size, eps)
        return y

    def rope(self, x, pos: int, base: float) -> np.ndarray:
        y = np.array(x, np.float64, copy=True)
        self.lib.orc_rope_d(y, y.size, pos, base)
        return y

    def attend(self, q, k, v) -> np.ndarray:
        q = np.ascontiguousarray(q, np.float64)
        k = np.ascontiguousarray(k, np.float64)
        v = np.ascontiguousarray(v, np.float64)
        o = np.empty_like(q)
        self.lib.orc_attend_d(o, q, k, v, k.shape[0], q.size)
        return o

    def log_softmax(self, logits, temperature: float = 1.0) -> np.ndarray:
        z = np.ascontiguousarray(logits, np.float64)
        o = np.empty_like(z)
        self.lib.orc_log_softmax_d(o, z, z.size, temperature)
        return o

    def sample(self, logits, temperature: float, seed: int, n: int, s: int):
        z = np.ascontiguousarray(logits, np.float64)
        tok, lp, gap = C.c_int32(), C.c_double(), C.c_float()
        self.lib.orc_sample_d(z, z.size, temperature, seed, n, s, C.byref(tok), C.byref(lp), C.byref(gap))
        return tok.value, lp.value, gap.value

    def sample_top_p(self, logits, temperature: float, top_p: float, seed: int, n: int, s: int):
        """(token, log-prob under the renormalised kept set, gap, size of the kept set, margin of the cut)."""
        z = np.ascontiguousarray(logits, np.float64)
        tok, lp, gap, kept, margin = C.c_int32(), C.c_double(), C.c_float(), C.c_int32(), C.c_double()
        self.lib.orc_sample_top_p_d.argtypes = [_f64p, C.c_int, C.c_float, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                                C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_float),
                                                C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        self.lib.orc_sample_top_p_d(z, z.size, temperature, top_p, seed, n, s, C.byref(tok), C.byref(lp), C.byref(gap),
                                    C.byref(kept), C.byref(margin))
        return tok.value, lp.value, gap.value, kept.value, margin.value

    # -- model-level --------------------------------------------------------------------
    def blob_numel(self, desc: Desc) -> int:
        return int(self.lib.orc_blob_numel(C.byref(desc)))

    def _check_blob(self, desc: Desc, blob: np.ndarray) -> np.ndarray:
        blob = np.ascontiguousarray(blob, np.float32)
        if blob.size != self.blob_numel(desc):
            raise ValueError(f"blob has {blob.size} elements, expected {self.blob_numel(desc)}")
        return blob

    def forward_cached(self, desc: Desc, blob, tokens) -> np.ndarray:
        blob = self._check_blob(desc, blob)
        tokens = np.ascontiguousarray(tokens, np.int32)
        out = np.empty((tokens.size, desc.vocab), np.float64)
        self.lib.orc_forward_cached(C.byref(desc), blob, tokens, tokens.size, out)
        return out

    def forward_full(self, desc: Desc, blob, tokens) -> np.ndarray:
        blob = self._check_blob(desc, blob)
        tokens = np.ascontiguousarray(tokens, np.int32)
        out = np.empty((tokens.size, desc.vocab), np.float64)
        self.lib.orc_forward_full(C.byref(desc), blob, tokens, tokens.size, out)
        return out

    def logprobs(self, desc: Desc, blob, tokens, temperature: float = 1.0) -> np.ndarray:
        blob = self._check_blob(desc, blob)
        tokens = np.ascontiguousarray(tokens, np.int32)
        out = np.zeros(tokens.size, np.float64)
        self.lib.orc_logprobs(C.byref(desc), blob, tokens, tokens.size, temperature, out)
        return out

    def rollout(self, desc: Desc, blobs, prompts, prompt_lens, G: int, max_new: int,
                temperature: float, seed: int, versions: Optional[Sequence[int]] = None,
                swap_at_step: Optional[Sequence[int]] = None, stop_lens=None, eos_id: int = -1,
                forced=None, want_logits: bool = False, top_p: float = 1.0) -> dict:
        if isinstance(blobs, np.ndarray):
            blobs = [blobs]
        blobs = [self._check_blob(desc, b) for b in blobs]
        nm = len(blobs)
        versions = np.ascontiguousarray(versions if versions is not None else range(nm), np.int64)
        swaps = np.ascontiguousarray(swap_at_step if swap_at_step is not None else [], np.int32)
        if swaps.size != nm - 1:
            raise ValueError("need one swap step per additional snapshot")
        prompts = np.ascontiguousarray(prompts, np.int32)
        prompt_lens = np.ascontiguousarray(prompt_lens, np.int32)
        P = prompts.shape[0]
        N = P * G
        toks = np.empty((N, max_new), np.int32)
        lps = np.empty((N, max_new), np.float64)
        lens = np.empty(N, np.int32)
        vers = np.empty((N, max_new), np.int64)
        gaps = np.zeros((N, max_new), np.float32)
        logits = np.zeros((N, max_new, desc.vocab), np.float64) if want_logits else None
        bp = (C.c_void_p * nm)(*[b.ctypes.data for b in blobs])
        vp = lambda a: a.ctypes.data_as(C.c_void_p) if a is not None else None
        stop = np.ascontiguousarray(stop_lens, np.int32) if stop_lens is not None else None
        frc = np.ascontiguousarray(forced, np.int32) if forced is not None else None
        if frc is not None and frc.shape != (N, max_new):
            raise ValueError("forced must be [N, max_new]")
        margins = np.ones((N, max_new), np.float64)
        self.lib.orc_rollout_top_p.argtypes = None
        self.lib.orc_rollout_top_p.restype = C.c_int
        rc = self.lib.orc_rollout_top_p(C.byref(desc), C.c_int(nm), bp, vp(versions), vp(swaps if swaps.size else np.zeros(1, np.int32)),
                                        vp(prompts), C.c_int(prompts.shape[1]), vp(prompt_lens), C.c_int(P), C.c_int(G),
                                        C.c_int(max_new), C.c_float(temperature), C.c_float(top_p), C.c_uint64(seed), vp(stop),
                                        C.c_int(eos_id), vp(frc), vp(toks), vp(lps), vp(lens), vp(vers), vp(logits), vp(gaps),
                                        vp(margins))
        if rc != 0:
            raise RuntimeError(f"orc_rollout_top_p failed: {rc}")
        return dict(tokens=toks, logprobs=lps, lens=lens, versions=vers, gaps=gaps, logits=logits, margins=margins)

    def grpo_tensors(self, tokens, lens, G: int, turn_start: int, rewards, eps: float = 1e-6):
        """(response mask uint8 [N, T], advantages [N], per-token advantages [N, T])."""
        tokens = np.ascontiguousarray(tokens, np.int32)
        lens = np.ascontiguousarray(lens, np.int32)
        rewards = np.ascontiguousarray(rewards, np.float64)
        N, T = tokens.shape
        mask = np.zeros((N, T), np.uint8)
        adv = np.zeros(N, np.float64)
        adv_tok = np.zeros((N, T), np.float64)
        vp = lambda a: a.ctypes.data_as(C.c_void_p)
        self.lib.orc_grpo_tensors.argtypes = None
        self.lib.orc_grpo_tensors.restype = C.c_int
        rc = self.lib.orc_grpo_tensors(vp(tokens), C.c_int(T), vp(lens), C.c_int(N), C.c_int(G), C.c_int32(turn_start), vp(rewards),
                                       C.c_double(eps), vp(mask), vp(adv), vp(adv_tok))
        if rc != 0:
            raise ValueError("orc_grpo_tensors: bad arguments")
        return mask, adv, adv_tok

    def set_progress_file(self, path: Optional[str]) -> None:
        """Long calls append a line every 32 tokens to this file (None: off)."""
        self.lib.orc_set_progress_file(path.encode() if path else None)

    def set_threads(self, n: int) -> None:
        self.lib.orc_set_threads(n)

    def get_threads(self) -> int:
        return int(self.lib.orc_get_threads())


_cache = {}


def load(precision: str = "f64") -> Oracle:
    if precision not in _cache:
        _cache[precision] = Oracle(precision)
    return _cache[precision]
