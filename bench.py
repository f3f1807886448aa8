"""Rollout-generation benchmark on one MI355X.

A "step" is one whole rollout of the workload (prefill of the unique prompts, KV replication, every
decode step with fused sampling, result read-back), with the policy already installed in HBM.
Prints one JSON line: generated tokens/s, the HBM roofline of the decode-attention kernel measured
with HIP events inside the library, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the decode-attention kernel (profiles/pmc_traffic_*.md), scaled by the same
# counters on a plain 256 MiB copy: KiB fetched + written per launch over the KiB of the K/V tiles the launch touches
# (shared prompt tiles once per group, a sequence's last tile whole).  Taken at the same kernel and grid on a 2-layer
# model generating 64 tokens (the profiler crashes on the 36-layer process); set to None whenever attn_rows_kernel changes.
ATTN_TRAFFIC_OVER_TILE_BYTES = (29524.2 + 512.0) / (28608.0 + 512.0)
# The same kernel timed by rocprofv3 --kernel-trace inside the graph replays of this very command (config 2), in microseconds
# per launch (profiles/kernel_trace_dense4b-64x512+1024.md): the HIP events of the timed run bracket launches that are issued
# one by one and include the launch gap, so both figures go into the line.  None for any other workload, and whenever the
# kernel changes.
ATTN_KERNEL_TRACE_US = {"dense4b-64x512+1024": 31.39}


def attn_kv_bytes_per_launch(shape, gen_lens, prompt_len, group, steps, whole_tiles, shared_elsewhere=False):
    """K/V bytes one decode-attention launch (one layer) reads, averaged over the decode passes `steps`: the whole
    32-key tiles of a prompt once per group with an active sequence, everything else per active sequence.
    whole_tiles: count the tiles the kernel touches (a sequence's last tile is fetched whole) instead of the keys.
    shared_elsewhere: the groups' whole prompt tiles are attended by attn_prefix_kernel, not by this kernel."""
    gen = np.asarray(gen_lens, np.int64)
    shared = (prompt_len // 32) * 32 if group > 1 else 0
    group_len = gen.reshape(-1, group).max(axis=1)
    per_key = 2 * shape.n_kv_heads * shape.head_dim * 2
    tot = 0.0
    for st in steps:
        own = prompt_len - shared + st
        if whole_tiles:
            own = -(-own // 32) * 32
        tot += (int((group_len > st).sum()) * (0 if shared_elsewhere else shared) + int((gen > st).sum()) * own) * per_key
    return tot / max(1, len(steps))

WORKLOADS = {
    # name: shape, prompts, G, prompt_len, max_new [, stop = (lo, hi) per-sequence stop lengths, swap_every = decode
    # steps between snapshot swaps, score = teacher-forced log-prob pass over all generated strings afterwards]
    "tiny-fp32": dict(shape="TINY", P=4, G=2, plen=16, max_new=32),
    "dense4b-64x512+1024": dict(shape="DENSE_4B", P=8, G=8, plen=512, max_new=1024),
    # the same with the paper's sampling setting (Sec. 5.1: top-p 0.95): logits are materialised and cut per step
    "dense4b-64x512+1024-top_p0.95": dict(shape="DENSE_4B", P=8, G=8, plen=512, max_new=1024, top_p=0.95),
    "dense4b-kvheavy-256x1024+4096": dict(shape="DENSE_4B", P=32, G=8, plen=1024, max_new=4096, stop=(512, 4096)),
    "dense8b-128x512+2048-swap256": dict(shape="DENSE_8B", P=16, G=8, plen=512, max_new=2048, swap_every=256),
    # config 3's lengths with four times the prompts than the cache holds at once: finished groups are replaced by
    # waiting prompts (echo_rollout_continuous), 256 sequences decode together throughout
    "dense4b-kvheavy-512x1024+4096-continuous256": dict(shape="DENSE_4B", P=64, G=8, plen=1024, max_new=4096, stop=(512, 4096),
                                                        slots=256, continuous=True),
    # the paper's own sampling setting (Sec. 5.1: Qwen3-8B-class policy, 16 samples per prompt, temperature 1.0, top-p 0.95,
    # up to 8192 generated tokens); stop lengths stand in for EOS
    "dense8b-paper-128x1024+8192-top_p0.95": dict(shape="DENSE_8B", P=8, G=16, plen=1024, max_new=8192, top_p=0.95, stop=(1024, 8192)),
    # eight cache-fuls of shorter sequences, and one cache-ful of the same length mix through the ordinary rollout
    "dense4b-2048x512+1024-continuous256": dict(shape="DENSE_4B", P=256, G=8, plen=512, max_new=1024, stop=(128, 1024),
                                                slots=256, continuous=True),
    "dense4b-256x512+1024-ragged": dict(shape="DENSE_4B", P=32, G=8, plen=512, max_new=1024, stop=(128, 1024)),
    "dense32b-64x1024+4096-score": dict(shape="DENSE_32B", P=8, G=8, plen=1024, max_new=4096, score=True),
}


def algorithmic_bytes(shape, gen_lens, prompt_len, group=1, first_step=1, per_step_out=None):
    """HBM bytes the decode steps must move: all decode-read weights once per step, the K/V of every active
    sequence once per step, and the new K/V written.  gen_lens: tokens generated per sequence (prompt-major,
    `group` sequences per prompt).  The whole 32-key tiles of a prompt are read from one copy per group by the
    decode attention kernel, so they count once per group that still has an active sequence; group=1 gives the
    per-sequence figure (every sequence reads its own copy of everything).  first_step=0: the first token, too, comes
    out of a decode step (continuous rollouts); the K/V terms depend on each sequence's own steps only, not on when it ran.
    per_step_out: a list that receives the bytes of every decode pass, in step order."""
    e = 2 if shape.dtype == "bf16" else 4
    hd, H = shape.head_dim, shape.hidden
    per_layer = H * (shape.n_q_heads + 2 * shape.n_kv_heads) * hd + shape.n_q_heads * hd * H + 3 * H * shape.ffn
    w_dec = (shape.n_layers * per_layer + shape.vocab * H) * e
    kvb = 2 * shape.n_layers * shape.n_kv_heads * hd * e
    gen = np.asarray(gen_lens, np.int64)
    steps = int(gen.max())
    shared = (prompt_len // 32) * 32 if group > 1 else 0
    group_len = gen.reshape(-1, group).max(axis=1)
    s_idx = np.arange(first_step, steps, dtype=np.int64)
    active = np.array([(gen > s).sum() for s in range(first_step, steps)], np.int64)   # decode pass s serves sequences with gen > s
    groups = np.array([(group_len > s).sum() for s in range(first_step, steps)], np.int64)
    kv_read = groups * shared + active * (prompt_len - shared + s_idx)
    per_step = w_dec + kv_read * kvb + active * kvb
    if per_step_out is not None:
        per_step_out.extend(int(b) for b in per_step)
    total = int(per_step.sum())
    return total, w_dec, kvb


def cpu_baseline(shape, blob, wl):
    """The oracle (fp32 build, as it stands) on a bounded slice of the same workload.  The tiny workload: the whole
    rollout.  The large shapes: one sequence with the workload's prompt length (at most 512 tokens) and four generated
    tokens, all layers at full width -- the oracle's cost per token is the same at every step, so the slice fixes its
    rate; its prompt pass is inside the timed call as the GPU's prefill is inside the rollout."""
    from oracle import oracle
    from paper_2602_02192_amd import synth
    orc = oracle.load("f32")
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")))
    orc.set_threads(cores)
    if shape.n_layers <= 2:
        P, G, prompt_len, new = wl["P"], wl["G"], wl["plen"], wl["max_new"]
    else:
        P, G, prompt_len, new = 1, 1, min(512, wl["plen"]), 4
    prompts, lens = synth.make_prompts(shape.vocab, P, prompt_len, seed=1)
    b32 = synth.widen_to_f32(blob)
    t0 = time.perf_counter()
    r = orc.rollout(oracle.desc_from_shape(shape), b32, prompts, lens, G=G, max_new=new, temperature=1.0, seed=2)
    dt = time.perf_counter() - t0
    del b32
    n_gen = int(r["lens"].sum())
    n_fed = int(P * G * prompt_len + n_gen - P * G)
    return {"value": float(n_gen / dt), "unit": "generated tokens/s", "cores": orc.get_threads(),
            "kind": "oracle", "tokens_through_the_decoder_per_s": float(n_fed / dt),
            "sample": f"fp32 oracle, {P * G} sequence(s), prompt {prompt_len} + {new} new tokens, all "
            f"{shape.n_layers} layers at full width, {dt:.1f} s (prompt pass included; every token costs one pass through the decoder)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="dense4b-64x512+1024", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-step-timing", action="store_true")
    ap.add_argument("--ctx-pad", type=int, default=0, help="extra KV-cache tokens per sequence beyond prompt + max_new")
    ap.add_argument("--pageable-blob", action="store_true",
                    help="keep the host copy of the weights in pageable memory (a counter-collecting profiler crashed on the pinned copy)")
    ap.add_argument("--install-chunk-mb", type=int, default=0,
                    help="snapshot swaps inside a rollout hand the blob over in pieces of this size (0 = one call)")
    ap.add_argument("--continuous", action="store_true",
                    help="run the workload through echo_rollout_continuous (refill does not apply when everything fits the cache; "
                         "the rows of a draining batch are compacted)")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch decode steps kernel by kernel (counter collection cannot follow graph replays)")
    ap.add_argument("--prefix-kernel", type=int, default=0, choices=[0, 1, 2, 3],
                    help="echo_rollout_opts.prefix_kernel: who attends a group's shared prompt tiles (0 = the planner decides)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py measures one GPU: rollout workers are independent (data parallel over prompts) and "
                 "this build runs a single MI355X; run with --gpus 1")
    import torch
    from paper_2602_02192_amd import echo, synth

    wl = WORKLOADS[a.workload]
    name, P, G, plen, max_new = wl["shape"], wl["P"], wl["G"], wl["plen"], wl["max_new"]
    shape = getattr(synth, name)
    N = P * G
    torch.cuda.set_device(0)
    t_start = time.perf_counter()

    def host_blob(seed):
        dev = synth.make_weights(shape, seed, device="cuda")
        if a.pageable_blob:
            host = dev.cpu()
        else:
            host = torch.empty(dev.shape, dtype=dev.dtype, pin_memory=True)
            host.copy_(dev)
        del dev
        torch.cuda.empty_cache()
        return host

    blob = host_blob(0)
    swap_every = wl.get("swap_every")
    blob_b = host_blob(10) if swap_every else None
    prompts, lens = synth.make_prompts(shape.vocab, P, plen, seed=1)
    stop = synth.make_stop_lens(N, wl["stop"][0], wl["stop"][1], seed=3) if wl.get("stop") else None
    swaps = list(range(swap_every, max_new, swap_every)) if swap_every else []
    continuous = bool(wl.get("continuous")) or a.continuous
    if continuous:
        a.no_kernel_timing = True    # the continuous entry point takes no per-kernel event timing
    ctx = echo.Context(echo.desc_from_shape(shape, wl.get("slots", N), plen + max_new + a.ctx_pad, n_weight_slots=2 if swap_every else 1))
    t0 = time.perf_counter()
    ctx.load_policy(0, blob)
    load_s = time.perf_counter() - t0
    version = [0]

    def progress(msg):   # stage marks on stderr: the long workloads run minutes between two lines of output otherwise
        print(f"[bench] {msg} (+{time.perf_counter() - t_start:.1f} s)", file=sys.stderr, flush=True)

    progress(f"policy installed in {load_s:.2f} s")

    def rollout(seed, **kw):
        """One rollout; with a swap schedule a second thread installs the next snapshot (alternating two weight
        sets) as soon as the previous one has been switched in, as a worker's receiver thread would."""
        kw.setdefault("top_p", wl.get("top_p", 1.0))
        kw.setdefault("prefix_kernel", a.prefix_kernel)
        if not swaps:
            return ctx.rollout(prompts, lens, G, max_new, 1.0, seed, stop_lens=stop, no_graph=a.no_graph, continuous=continuous, **kw)
        import threading
        done = threading.Event()

        def feeder():
            for j in range(len(swaps)):
                while not done.is_set():
                    st = ctx.stats()
                    if st.rollout_running and st.staged_version < 0:
                        break
                    time.sleep(0.002)
                if done.is_set():
                    return
                version[0] += 1
                nxt = blob_b if version[0] % 2 else blob
                if a.install_chunk_mb > 0:
                    ctx.load_policy_chunked(version[0], nxt, [a.install_chunk_mb << 20])
                else:
                    ctx.load_policy(version[0], nxt)

        th = threading.Thread(target=feeder)
        th.start()
        try:
            return ctx.rollout(prompts, lens, G, max_new, 1.0, seed, stop_lens=stop, swap_at_step=swaps, swap_timeout_ms=60000,
                               no_graph=a.no_graph, **kw)
        finally:
            done.set()
            th.join()

    for _ in range(a.warmup):
        rollout(2)
        progress("warm-up rollout done")
    torch.cuda.synchronize()
    times, toks, decode_ms, prefill_ms, swap_wait_ms, steps_run = [], 0, [], [], [], []
    t_all = time.perf_counter()
    for k in range(a.steps):
        t0 = time.perf_counter()
        out = rollout(2 + k)
        times.append(time.perf_counter() - t0)
        toks += int(out["lens"].sum())
        st = ctx.stats()
        decode_ms.append(st.decode_ms)
        prefill_ms.append(st.prefill_ms)
        swap_wait_ms.append(st.swap_wait_ms)
        steps_run.append(st.decode_steps)
        progress(f"timed rollout {k + 1} of {a.steps} done")
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t_all
    value = toks / total_s

    bytes_decode, w_dec, kvb = algorithmic_bytes(shape, out["lens"], plen, G)
    step_frac = bytes_decode / (np.mean(decode_ms) * 1e-3) / (HBM_PEAK_GBS * 1e9)
    bytes_per_seq = algorithmic_bytes(shape, out["lens"], plen, 1)[0]   # every sequence reading a prompt copy of its own
    step_frac_per_seq = bytes_per_seq / (np.mean(decode_ms) * 1e-3) / (HBM_PEAK_GBS * 1e9)
    n_decode_steps = max(1, int(out["lens"].max()) - 1)
    if continuous:     # weights once per step actually run; every token, the first included, comes out of a decode step
        n_decode_steps = int(np.mean(steps_run))
        longest = int(out["lens"].max())
        bytes_decode = algorithmic_bytes(shape, out["lens"], plen, G, first_step=0)[0] + w_dec * (n_decode_steps - longest)
        bytes_per_seq = algorithmic_bytes(shape, out["lens"], plen, 1, first_step=0)[0] + w_dec * (n_decode_steps - longest)
        step_frac = bytes_decode / (np.mean(decode_ms) * 1e-3) / (HBM_PEAK_GBS * 1e9)
        step_frac_per_seq = bytes_per_seq / (np.mean(decode_ms) * 1e-3) / (HBM_PEAK_GBS * 1e9)

    # per-step roofline fractions: one more rollout (graph replay as timed above) with a HIP event between every two steps
    step_stats = {}
    if not continuous and not swaps and not a.no_step_timing:
        rollout(2 + a.steps - 1, time_steps=True)
        progress("rollout with per-step event timing done")
        sm = ctx.step_times().astype(np.float64)
        strict, per_seq = [], []
        algorithmic_bytes(shape, out["lens"], plen, G, per_step_out=strict)
        algorithmic_bytes(shape, out["lens"], plen, 1, per_step_out=per_seq)
        n = min(len(sm), len(strict))
        if n > 0:
            fs = np.array(strict[:n]) / (sm[:n] * 1e-3) / (HBM_PEAK_GBS * 1e9)
            fp = np.array(per_seq[:n]) / (sm[:n] * 1e-3) / (HBM_PEAK_GBS * 1e9)
            step_stats = {"steps_timed": int(n), "step_ms_p10_median_p90": [float(np.percentile(sm[:n], q)) for q in (10, 50, 90)],
                          "hbm_frac_p10": float(np.percentile(fs, 10)), "hbm_frac_median": float(np.percentile(fs, 50)),
                          "hbm_frac_p90": float(np.percentile(fs, 90)),
                          "hbm_frac_if_every_sequence_read_its_own_prompt_copy_p10_median_p90":
                              [float(np.percentile(fp, q)) for q in (10, 50, 90)]}

    score = None
    if wl.get("score"):       # teacher-forced log-probs of every generated string (prompt + response) under the active snapshot
        full = np.concatenate([np.repeat(prompts, G, axis=0), np.maximum(out["tokens"], 0)], axis=1)
        flen = (plen + out["lens"]).astype(np.int32)
        t0 = time.perf_counter()
        lp = ctx.logprobs(full, flen, 1.0)
        score_s = time.perf_counter() - t0
        progress("scoring pass done")
        hd, H = shape.head_dim, shape.hidden
        per_layer = H * (shape.n_q_heads + 2 * shape.n_kv_heads) * hd + shape.n_q_heads * hd * H + 3 * H * shape.ffn
        rows = int((flen - 1).sum())
        flops = 2.0 * rows * (shape.n_layers * per_layer + shape.vocab * H)
        m = np.arange(max_new)[None, :] < out["lens"][:, None]
        dev = float(np.abs(lp[:, plen:][m] - out["logprobs"][m]).max())
        score = {"rows": rows, "seconds": score_s, "gemm_tflops": flops / score_s / 1e12, "mfma_frac_of_2.5PFLOPs": flops / score_s / 2.5e15,
                 "max_abs_diff_vs_sampler_logprobs": dev}

    roofline = None
    if not a.no_kernel_timing:
        rollout(2, time_kernels=True)
        progress("rollout with per-kernel event timing done")
        st = ctx.stats()
        if st.attn_launches:
            per_launch_bytes = st.attn_bytes / st.attn_launches
            per_launch_s = st.attn_ms * 1e-3 / st.attn_launches
            ach = per_launch_bytes / per_launch_s / 1e9
            timed = [t for t in range(1, int(out["lens"].max())) if t % 16 == 1]   # the passes the library times
            # which accounting the library used tells whether the shared prompt tiles went through the prefix kernel
            models = {se: attn_kv_bytes_per_launch(shape, out["lens"], plen, G, timed, whole_tiles=False, shared_elsewhere=se)
                      for se in (True, False)}
            prefix_kernel = abs(models[True] - per_launch_bytes) < abs(models[False] - per_launch_bytes)
            traffic = None
            # (the counters were taken with the kernel reading its shared tiles itself; with the prefix kernel it also reads
            # that kernel's partials, which the factor does not cover; they were taken on the two-rows-per-workgroup form)
            rows_per_wg = int(st.attn_rows_per_workgroup)
            if (ATTN_TRAFFIC_OVER_TILE_BYTES and not prefix_kernel and rows_per_wg == 2
                    and abs(models[False] - per_launch_bytes) <= 1e-3 * per_launch_bytes):
                traffic = attn_kv_bytes_per_launch(shape, out["lens"], plen, G, timed, whole_tiles=True,
                                                   shared_elsewhere=prefix_kernel) * ATTN_TRAFFIC_OVER_TILE_BYTES
            kname = (f"attn_rows_kernel (decode attention, one launch per layer, {rows_per_wg} neighbouring rows and their common prompt tiles per workgroup)"
                     if rows_per_wg > 1 else
                     "attn_splitk_kernel (decode attention, one launch per layer" +
                     ("; the groups' shared prompt tiles are attended by attn_prefix_kernel before it)" if prefix_kernel else ")"))
            roofline = {"bound": "hbm", "kernel": kname,
                        "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                        "traffic": traffic,
                        "traffic_unit": "bytes per launch: whole K/V tiles of the timed launches x 1.0315 (FETCH_SIZE + WRITE_SIZE over "
                                        "whole-tile bytes, same kernel and grid, profiles/pmc_traffic_*.md)",
                        "launches_timed": int(st.attn_launches),
                        "avg_launch_us": per_launch_s * 1e6, "bytes_per_launch": per_launch_bytes}
            if ATTN_KERNEL_TRACE_US.get(a.workload) and not prefix_kernel:
                t_us = ATTN_KERNEL_TRACE_US[a.workload]
                mean_bytes = attn_kv_bytes_per_launch(shape, out["lens"], plen, G, range(1, int(out["lens"].max())), whole_tiles=False)
                roofline["kernel_trace"] = {"avg_launch_us": t_us, "bytes_per_launch": mean_bytes, "achieved": mean_bytes / t_us / 1e3,
                                            "frac": mean_bytes / t_us / 1e3 / HBM_PEAK_GBS,
                                            "source": "profiles/kernel_trace_dense4b-64x512+1024.md (rocprofv3 --kernel-trace of this command, all decode steps, inside graph replays)"}
            if st.gemm_launches:
                g = st.gemm_bytes / (st.gemm_ms * 1e-3) / 1e9
                roofline["gemm_weight_stream"] = {"achieved": g, "frac": g / HBM_PEAK_GBS,
                                                  "avg_launch_us": st.gemm_ms * 1e3 / st.gemm_launches,
                                                  "launches_timed": int(st.gemm_launches)}
    cpu = None
    if not a.no_cpu_baseline and blob.numel() < 6e9:   # the oracle needs an fp32 copy of the weights: 4B-class and smaller
        cpu = cpu_baseline(shape, blob, wl)
    ctx.close()
    line = {
        "metric": "rollout generated tokens/s on 1 MI355X", "value": value, "unit": "generated tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": 1e3 * total_s / a.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 MFMA operands, f32 accumulate (bf16 weights)" if shape.dtype == "bf16" else "f32", "data": "synthetic (random N(0,0.02) weights, uniform random prompt tokens)",
        "config": {"workload": a.workload, "decoder_shape": name, "sequences": N, "prompts": P, "group": G,
                   "prompt_len": plen, "max_new": max_new, "temperature": 1.0, "top_p": wl.get("top_p", 1.0),
                   "stop_lens": list(wl["stop"]) if wl.get("stop") else None,
                   "sequences_decoding_together": wl.get("slots", N), "continuous": continuous},
        "decode_step": {"mean_ms": float(np.mean(decode_ms)) / n_decode_steps,
                        "hbm_frac_of_8TBps": step_frac, "algorithmic_bytes_per_rollout": bytes_decode,
                        "hbm_frac_if_every_sequence_read_its_own_prompt_copy": step_frac_per_seq,
                        "prefill_ms": float(np.mean(prefill_ms)), "policy_install_s": load_s,
                        "swaps_per_rollout": len(swaps), "install_chunk_mb": a.install_chunk_mb, "swap_wait_ms": float(np.mean(swap_wait_ms)),
                        **step_stats},
        "scoring_pass": score,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
