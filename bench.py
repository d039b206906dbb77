#!/usr/bin/env python3
"""Decode throughput of the LazyEviction hot path on one MI355X.

A "step" is one decode step of the whole model: for every layer one lazyev_decode_step
(append, attention, recurrence tracking) and, when t is a multiple of W, the eviction of every
layer (score, select, compact: lazyev_evict_all, or one lazyev_evict per layer with
--evict-per-layer).  The run replays the workload from its prompt: W warm-up steps on a
throw-away pass, the state is reset, then exactly K steps are timed between two
synchronisations.  Inputs (prompt K/V and every step's q, k_new, v_new) are generated on the
GPU beforehand and are resident in HBM when the clock starts.

Prints one JSON line: whole-job steps/s (value), tokens/s, the HBM roofline of the attention
split kernel measured with HIP events inside the timed region, and the CPU oracle timed on the
host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

# HBM bytes per launch of the attention split kernel at the steady-state cache length, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script (summaries under profiles/; the
# counters are scaled by what they read for the plain copy kernel of --calibrate-copy-mb).
MEASURED_TRAFFIC_BYTES = {"cfg3": 2 * 68540 * 1024 + 2545 * 1024,      # 137.4 MB algorithmic at N = 2080.5
                          "cfg4": 2 * 38180 * 1024 + 5776 * 1024,      # 72.4 MB at N = 1088.5 (every logit kept)
                          "cfg5": 2 * 134900 * 1024 + 4395 * 1024}     # 271.5 MB at N = 4128.5


def algorithmic_bytes_decode(cfg, n1: int) -> int:
    """Bytes one layer's decode step must move with n1 cached entries (after the append):
    every K and V row once, q and out once, the appended rows (read + write)."""
    esz = 4 if cfg.dtype == "fp32" else 2
    kv = 2 * cfg.batch * cfg.n_kv_heads * n1 * cfg.head_dim * esz
    qo = 2 * cfg.batch * cfg.n_q_heads * cfg.head_dim * esz
    app = 2 * 2 * cfg.batch * cfg.n_kv_heads * cfg.head_dim * esz
    return kv + qo + app


def algorithmic_bytes_move(cfg, rows_moved_per_event: float) -> float:
    """What a stable in-place compaction must move: every surviving entry that changes slot
    (counted by the library, summed over the layer's units) has its K row and its V row read
    and written once."""
    esz = 4 if cfg.dtype == "fp32" else 2
    return 2 * 2 * rows_moved_per_event * cfg.head_dim * esz


def _oracle_worker(job):
    """Steady-state sample for the CPU baseline: one oracle unit with B entries runs W decode
    steps and the eviction that follows."""
    name, seed = job
    import numpy as np
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(1)
    except Exception:                                   # pragma: no cover
        limiter = None
    from oracle.lazyev_oracle import OracleUnit
    from paper_2506_15969_amd.workload import CONFIGS
    cfg = CONFIGS[name]
    rng = np.random.default_rng(seed)
    G, d, B, W = cfg.group, cfg.head_dim, cfg.budget, cfg.window
    u = OracleUnit(rng.standard_normal((B, d)), rng.standard_normal((B, d)), G, B, W, cfg.alpha)
    qs = rng.standard_normal((W, G, d))
    ks = rng.standard_normal((W, d))
    vs = rng.standard_normal((W, d))
    t0 = time.perf_counter()
    for t in range(1, W + 1):
        u.decode_step(t, qs[t - 1], ks[t - 1], vs[t - 1])
        u.evict(t)
    dt = time.perf_counter() - t0
    assert len(u) == B
    del limiter
    return W, dt


def cpu_baseline(cfg, target_seconds: float = 15.0) -> dict:
    import multiprocessing as mp
    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    ctx = mp.get_context("spawn")
    with ctx.Pool(cores) as pool:
        w, dt = pool.map(_oracle_worker, [(cfg.name, 0)])[0]          # calibrate on one unit
        per_unit = max(dt, 1e-3)
        rounds = max(1, int(target_seconds / per_unit))
        jobs = [(cfg.name, 1 + i) for i in range(cores * rounds)]
        t0 = time.perf_counter()
        res = pool.map(_oracle_worker, jobs, chunksize=1)
        wall = time.perf_counter() - t0
    unit_steps = sum(r[0] for r in res)
    unit_steps_per_s = unit_steps / wall
    units_per_model = cfg.n_layers * cfg.batch * cfg.n_kv_heads
    return {"value": unit_steps_per_s / units_per_model, "unit": "steps/s", "cores": cores,
            "kind": "oracle",
            "unit_steps_per_s": unit_steps_per_s,
            "sample": "%d oracle units x (%d decode steps at N=%d..%d + 1 eviction), one "
                      "process per core; value = unit-steps/s / (L*S*Hkv=%d), extrapolated"
                      % (len(jobs), cfg.window, cfg.budget + 1, cfg.budget + cfg.window,
                         units_per_model)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed decode steps (0: the config's)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--chunk", type=int, default=0, help="split-block size override")
    ap.add_argument("--input-steps", type=int, default=0,
                    help="steps of inputs kept in HBM (0: all timed steps if they fit in "
                         "--input-gb, else as many as fit; later steps reuse them cyclically)")
    ap.add_argument("--input-gb", type=float, default=150.0)
    ap.add_argument("--profile-every", type=int, default=16,
                    help="time one layer call with HIP events every this many steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prompt-len", type=int, default=-1,
                    help="override the workload's prompt length (prompt = budget puts the cache "
                         "in its steady state from the first step; used for short profiling runs)")
    ap.add_argument("--variant", type=int, default=-1, help="attention kernel override (lazyev_set_variant)")
    ap.add_argument("--calibrate-copy-mb", type=int, default=0,
                    help="after the timed region, run one plain copy kernel of this many MiB "
                         "(a known traffic to scale hardware byte counters with)")
    ap.add_argument("--window", type=int, default=0,
                    help="override the observation window W (1 = an eviction after every step, "
                         "the schedule of the greedy methods the paper compares against)")
    ap.add_argument("--evict-per-layer", action="store_true",
                    help="one lazyev_evict call per layer instead of lazyev_evict_all")
    ap.add_argument("--no-evict", action="store_true",
                    help="full-cache baseline: budget covers prompt + all steps")
    ap.add_argument("--ragged", action="store_true",
                    help="per-sequence timing (lazyev_admit): sequence s takes its first step at "
                         "global step 1 + s %% W, so the sequences' evictions fall on different steps")
    ap.add_argument("--target-blocks", type=int, default=0,
                    help="blocks per decode launch, taken literally (lazyev_set_target_blocks)")
    ap.add_argument("--progress", type=int, default=0,
                    help="write a line to stderr every this many submitted steps (long runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path has no cross-GPU part "
              "(every (layer, sequence, KV head) unit is independent). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_15969_amd import binding
    from paper_2506_15969_amd.workload import CONFIGS, Workload

    cfg = CONFIGS[args.config]
    K = args.steps or cfg.steps
    if args.prompt_len >= 0:
        cfg = cfg.scaled(prompt_len=args.prompt_len, name="%s-prompt%d" % (cfg.name, args.prompt_len))
    if args.window > 0:
        cfg = cfg.scaled(window=args.window, name="%s-window%d" % (cfg.name, args.window))
    if args.ragged:
        cfg = cfg.scaled(name=cfg.name + "-ragged")
    if args.no_evict:
        # (alpha stays the workload's: it is defined from the budget, and a budget of the whole
        # generation would put the threshold below the weight of an average entry)
        full = cfg.prompt_len + K
        cfg = cfg.scaled(budget=full, name=cfg.name + "-fullkv",
                         alpha_numer=cfg.alpha_numer * (full + cfg.window) / (cfg.budget + cfg.window))
    wl = Workload(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L, S, Hq, Hkv, d, W = cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window
    esz = 4 if cfg.dtype == "fp32" else 2

    try:
        eng = binding.LazyEviction(L, S, Hq, Hkv, d, cfg.budget, W, cfg.prompt_len, cfg.alpha,
                                   dtype=cfg.torch_dtype, device=dev)
    except binding.LazyevError as e:
        print("bench.py: configuration rejected by the library: %s" % e, file=sys.stderr)
        sys.exit(2)

    def reset_state():
        for l in range(L):
            k, v = wl.prompt_kv(l, device=dev)
            eng.load_prompt(l, k, v)
        eng.init()
        if args.chunk:
            eng.set_chunk(args.chunk)
        if args.variant >= 0:
            eng.set_variant(args.variant)
        if args.target_blocks:
            eng.set_target_blocks(args.target_blocks)
        if args.ragged:
            for sq in range(S):                     # (the prompt rows are in the caches already)
                eng.admit(sq, cfg.prompt_len, sq % W)

    # ---- inputs resident in HBM
    per_step = L * S * (Hq + 2 * Hkv) * d * esz
    R = args.input_steps or K
    R = max(1, min(R, K, int(args.input_gb * 1e9 // per_step)))
    t_gen = time.perf_counter()
    q_all = torch.empty((R, L, S, Hq, d), dtype=cfg.torch_dtype, device=dev)
    k_all = torch.empty((R, L, S, Hkv, d), dtype=cfg.torch_dtype, device=dev)
    v_all = torch.empty((R, L, S, Hkv, d), dtype=cfg.torch_dtype, device=dev)
    GEN = 128
    for t0 in range(1, R + 1, GEN):
        t1 = min(R + 1, t0 + GEN)
        for l in range(L):
            q, kn, vn = wl.step_inputs(l, t0, t1, device=dev)
            q_all[t0 - 1:t1 - 1, l] = q
            k_all[t0 - 1:t1 - 1, l] = kn
            v_all[t0 - 1:t1 - 1, l] = vn
    out = torch.empty((L, S, Hq, d), dtype=cfg.torch_dtype, device=dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    lib, ctx = binding.lib, None
    q_base, k_base, v_base, o_base = q_all.data_ptr(), k_all.data_ptr(), v_all.data_ptr(), out.data_ptr()
    q_sz, kv_sz = S * Hq * d * esz, S * Hkv * d * esz
    decode, evict = lib.lazyev_decode_step, lib.lazyev_evict

    # cache length (after the append) seen by the decode call of step t: closed form of the
    # saw-tooth, used to attach algorithmic bytes to the profiled calls
    first = (max(cfg.budget - cfg.prompt_len, 0) // W + 1) * W     # first step with P + t > B, t = kW

    def n1_ragged(t, sq):
        """Entries of sequence sq after the append of global step t (0: it has not started)."""
        tau = t - sq % W
        if tau < 1:
            return 0
        return lib.lazyev_cached_before_step(cfg.prompt_len, tau, cfg.budget, W) + 1

    def bytes_at(t):
        """Algorithmic bytes of one layer call at step t."""
        if not args.ragged:
            return algorithmic_bytes_decode(cfg, n1_at(t))
        one = cfg.scaled(batch=1)
        return sum(algorithmic_bytes_decode(one, n1_ragged(t, sq)) for sq in range(S) if n1_ragged(t, sq))

    def n1_at(t):
        if t <= first:
            return cfg.prompt_len + t
        last_ev = (t - 1) // W * W
        return cfg.budget + (t - last_ev)

    def run(n_steps, profile_every=0):
        """n_steps decode steps from t = 1; one layer call is event-timed every
        `profile_every` steps (the layer rotates)."""
        ctx = eng._ctx
        for t in range(1, n_steps + 1):
            r = (t - 1) % R
            prof_layer = (t // profile_every) % L if profile_every and t % profile_every == 0 else -1
            for l in range(L):
                i = r * L + l
                if l == prof_layer:
                    lib.lazyev_profile_arm(ctx, 1)
                rc = decode(ctx, l, t, q_base + i * q_sz, k_base + i * kv_sz, v_base + i * kv_sz,
                            o_base + l * q_sz, None, None)
                if rc:
                    raise binding.LazyevError(rc, "lazyev_decode_step(layer %d, t %d), HIP error %d"
                                              % (l, t, lib.lazyev_last_hip_error(ctx)))
            if args.ragged:                                  # the library knows which sequences are due
                rc = lib.lazyev_evict_all(ctx, t, None)
                if rc:
                    raise binding.LazyevError(rc, "lazyev_evict_all(t %d)" % t)
            elif t % W == 0:
                due = n1_at(t) > cfg.budget
                if args.evict_per_layer:
                    for l in range(L):
                        if l == prof_layer and due:
                            lib.lazyev_profile_arm(ctx, 1)
                        rc = evict(ctx, l, t, None)
                        if rc:
                            raise binding.LazyevError(rc, "lazyev_evict(layer %d, t %d)" % (l, t))
                else:                                        # all layers in one launch pair
                    if prof_layer >= 0 and due:
                        lib.lazyev_profile_arm(ctx, 1)
                    rc = lib.lazyev_evict_all(ctx, t, None)
                    if rc:
                        raise binding.LazyevError(rc, "lazyev_evict_all(t %d)" % t)
            if args.progress and t % args.progress == 0:
                print("bench.py: step %d of %d submitted" % (t, n_steps), file=sys.stderr, flush=True)

    # ---- warm-up on a throw-away pass, then the timed pass from the prompt
    reset_state()
    run(args.warmup)
    torch.cuda.synchronize()
    reset_state()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    run(K, args.profile_every)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    if args.calibrate_copy_mb:
        nbytes = args.calibrate_copy_mb << 20
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        lib.lazyev_stream_probe(dst.data_ptr(), src.data_ptr(), nbytes, 2048,
                                torch.cuda.current_stream(dev).cuda_stream)
        torch.cuda.synchronize()
        del src, dst
    # what a plain streaming read reaches on this machine (1 GiB, non-temporal loads, two blocks per
    # compute unit): the second denominator beside the published peak
    probe_bytes = 1 << 30
    probe_src = torch.empty(probe_bytes, dtype=torch.uint8, device=dev).random_(0, 255)
    probe_sink = torch.zeros(4, dtype=torch.int32, device=dev)
    stream_ptr = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    lib.lazyev_stream_read_probe(probe_src.data_ptr(), probe_bytes, 512, probe_sink.data_ptr(), stream_ptr)
    ev0.record()
    for _ in range(5):
        lib.lazyev_stream_read_probe(probe_src.data_ptr(), probe_bytes, 512, probe_sink.data_ptr(), stream_ptr)
    ev1.record()
    torch.cuda.synchronize()
    read_probe_gbs = 5 * probe_bytes / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del probe_src
    prof = eng.profile_read()
    st = eng.stats()
    # what a pair of HIP events adds to the kernel it brackets (empty kernel, same stream)
    ov = C.c_double(0.0)
    lib.lazyev_event_overhead(200, C.c_void_p(torch.cuda.current_stream(dev).cuda_stream), C.byref(ov))
    ov_ms = ov.value
    # bytes of the profiled decode calls
    prof_steps = [t for t in range(1, K + 1) if args.profile_every and t % args.profile_every == 0]
    dec_bytes = sum(bytes_at(t) for t in prof_steps)
    ev_steps = [t for t in prof_steps if t % W == 0 and n1_at(t) > cfg.budget]
    split_ms, split_n = prof["split"]
    comb_ms, comb_n = prof["combine"]
    sel_ms, sel_n = prof["select"]
    mov_ms, mov_n = prof["move"]
    assert split_n == len(prof_steps), (split_n, len(prof_steps))

    steps_per_s = K / elapsed
    result = {
        "metric": "decode steps/s at batch %d, budget %d (incl. eviction); tokens/s = value x batch"
                  % (S, cfg.budget),
        "value": steps_per_s, "unit": "steps/s", "tokens_per_s": steps_per_s * S,
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": 1e3 * elapsed / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": L, "batch": S, "q_heads": Hq, "kv_heads": Hkv,
                   "head_dim": d, "prompt_len": cfg.prompt_len, "budget": cfg.budget,
                   "window": W, "alpha": cfg.alpha, "input_steps_resident": R,
                   "evictions_per_layer": st["n_evict_events"][0],
                   "activations_per_unit_step": sum(st["n_activations"]) / (K * L * S * Hkv)},
        "input_generation_s": t_gen,
    }
    # which attention kernel the library picks for this shape (see lazyev_set_variant)
    fused = cfg.dtype == "bf16" and d == 128 and args.variant in (-1, 1, 4)
    if split_n:
        # event intervals minus the fixed cost of the event pair itself
        split_k = split_ms - ov_ms * split_n
        call_k = split_ms + comb_ms - 2 * ov_ms * split_n
        ach = dec_bytes / (split_k * 1e-3) / 1e9
        result["roofline"] = {
            "kernel": ("decode_fused_kernel (the one kernel of lazyev_decode_step)"
                       if fused else "first of the two kernels of lazyev_decode_step (split; "
                                     "decode_call covers split + merge)"),
            "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name),
            "plain_read_on_this_box": {"GB/s": read_probe_gbs, "frac_of_it": ach / read_probe_gbs,
                                       "what": "1 GiB read once with non-temporal loads, grid-stride, 512 blocks of 256 threads (the fastest of 512..65536 blocks: 7.0 TB/s; 1024..16384 blocks reach 5.6-6.2)"},
            "avg_us": 1e3 * split_k / split_n, "avg_us_between_events": 1e3 * split_ms / split_n,
            "event_pair_overhead_us": 1e3 * ov_ms, "launches_timed": split_n,
            "algorithmic_bytes_per_launch": dec_bytes / split_n,
            "decode_call": {"avg_us": 1e3 * call_k / split_n,
                            "achieved": dec_bytes / (call_k * 1e-3) / 1e9,
                            "frac": dec_bytes / (call_k * 1e-3) / 1e9 / HBM_PEAK_GBS},
        }
        if mov_n:
            events = sum(st["n_evict_events"])
            # bytes of one launch of the row-move kernel: one layer's, or all layers' at once
            mb = algorithmic_bytes_move(cfg, sum(st["n_rows_moved"]) / max(events, 1)) * (1 if args.evict_per_layer else L)
            mov_k = mov_ms - ov_ms * mov_n
            result["roofline"]["compaction"] = {
                "kernel": "evict_move_kernel", "layers_per_launch": 1 if args.evict_per_layer else L,
                "avg_us": 1e3 * mov_k / mov_n,
                "select_avg_us": 1e3 * (sel_ms - ov_ms * sel_n) / sel_n, "launches_timed": mov_n,
                "algorithmic_bytes_per_launch": mb,
                "rows_moved_per_unit_event": sum(st["n_rows_moved"]) / max(events, 1) / (S * Hkv),
                "achieved": mb / (mov_k / mov_n * 1e-3) / 1e9,
                "frac": mb / (mov_k / mov_n * 1e-3) / 1e9 / HBM_PEAK_GBS}
        # whole-step view: all algorithmic decode bytes of the run over the wall time
        tot = sum(bytes_at(t) for t in range(1, K + 1)) * L
        result["roofline"]["whole_run_frac"] = tot / elapsed / 1e9 / HBM_PEAK_GBS
    if not args.no_cpu_baseline:
        eng.close()
        del q_all, k_all, v_all
        result["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
