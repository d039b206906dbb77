#!/usr/bin/env python3
"""Decode throughput of the LazyEviction hot path on one MI355X.

A "step" is one decode step of the whole model: for every layer one lazyev_decode_step
(append, attention, recurrence tracking) and, when t is a multiple of W, the eviction of every
layer (score, select, compact: lazyev_evict_all, or one lazyev_evict per layer with
--evict-per-layer).  Two ways to place the K timed steps:

  from the prompt   (K reaches the workload's first eviction, e.g. the default K = all 16384
                    steps): the run replays the workload from its prompt.
  steady state      (a short K, e.g. --steps 20): the metric is quoted on a cache AT its budget
                    with evictions running, which a short run from a 256-token prompt never
                    reaches.  The prompt is then as long as the budget, TS / MRI start from the
                    prompt's own attention (lazyev_prefill_track), an untimed pre-roll brings the
                    cache to the step where the K timed steps straddle an eviction (they lie
                    around t = W), and the K steps are timed from there.

In both, --warmup steps run first on a throw-away pass, the state is rebuilt, and exactly K steps
are timed between two synchronisations.  Inputs (prompt K/V and every step's q, k_new, v_new)
are generated on the GPU beforehand and are resident in HBM when the clock starts.

Prints one JSON line: whole-job steps/s (value), tokens/s, the HBM roofline of the attention
kernel measured with HIP events inside the timed region (one event pair around the L layer calls
of a step: interval / L, nothing subtracted), and the CPU oracle timed on the host cores on a
bounded sample of the same workload.
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

# HBM bytes per launch of the attention kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# of this script in the steady state (summaries under profiles/decode_fused_<cfg>_steady.txt; the
# counters are scaled by what they read for the plain copy kernel of --calibrate-copy-mb):
# (mean entries per unit after the append in that profile, bytes).  Printed as roofline.traffic
# only when the timed steps of this run have the same mean cache length.
PROFILED_TRAFFIC = {"cfg3": (2080.5, 2 * 68000 * 1024 + 2325 * 1024),      # 136.9 MB algorithmic
                    "cfg4": (1088.5, 2 * 36080 * 1024 + 1987 * 1024),      # 71.9 MB
                    "cfg5": (4128.5, 2 * 134300 * 1024 + 3988 * 1024)}     # 271.0 MB


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
    from dataclasses import replace
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(1)
    except Exception:                                   # pragma: no cover
        limiter = None
    from oracle.lazyev_oracle import OracleUnit
    from paper_2506_15969_amd.workload import CONFIGS
    base, _, over = name.partition("|")               # "cfg3" or "cfg3|budget=..,window=.."
    cfg = CONFIGS[base]
    if over:
        cfg = replace(cfg, **{k: int(v) for k, v in (kv.split("=") for kv in over.split(","))})
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
    pool = ctx.Pool(cores)
    try:
        key = "%s|budget=%d,window=%d" % (cfg.name.split("-")[0], cfg.budget, cfg.window)
        w, dt = pool.map(_oracle_worker, [(key, 0)])[0]               # calibrate on one unit
        per_unit = max(dt, 1e-3)
        rounds = max(1, int(target_seconds / per_unit))
        jobs = [(key, 1 + i) for i in range(cores * rounds)]
        t0 = time.perf_counter()
        res = pool.map(_oracle_worker, jobs, chunksize=1)
        wall = time.perf_counter() - t0
    finally:
        pool.close()                                    # let the workers exit by themselves
        pool.join()
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


MFMA_BF16_PEAK_TFLOPS = 2500.0


def prefill_track_mode(args):
    """--prefill-track: times lazyev_prefill_track (the tracking loop of Alg. 1 and Eq. 1 over the
    prompt's own causal attention) on one layer of the workload with a prompt of --prompt-len
    (default 2048) positions, and prints one JSON line: milliseconds per layer and the rate of
    the two causal Q K^T passes against the dense bf16 MFMA peak."""
    import torch
    from paper_2506_15969_amd import binding
    from paper_2506_15969_amd.workload import CONFIGS, Workload
    P = args.prompt_len if args.prompt_len > 0 else 2048
    reps = args.steps or 5
    cfg = CONFIGS[args.config].scaled(n_layers=1, prompt_len=P, steps=8)
    wl = Workload(cfg)
    eng = binding.LazyEviction(1, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.budget,
                               cfg.window, P, cfg.alpha, dtype=cfg.torch_dtype)
    eng.load_prompt(0, *wl.prompt_kv(0, device="cuda"))
    eng.init()
    q = wl.prompt_queries(0, device="cuda")
    eng.prefill_track(0, q)                                   # warm-up
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(reps):
        eng.prefill_track(0, q)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / reps
    units = cfg.batch * cfg.n_kv_heads
    # 2 flops per multiply-add, causal triangle incl. the diagonal, G heads, two passes
    flops = 2.0 * 2.0 * units * cfg.group * (P * (P + 1) / 2.0) * cfg.head_dim
    st = eng.stats()
    print(json.dumps({
        "metric": "prompt_tracking_ms_per_layer", "value": ms, "unit": "ms", "higher_is_better": False,
        "config": {"workload": "%s-prompt%d" % (cfg.name, P), "batch": cfg.batch, "prompt_len": P,
                   "n_q_heads": cfg.n_q_heads, "n_kv_heads": cfg.n_kv_heads, "alpha": cfg.alpha},
        "prompt_tokens_per_s": cfg.batch * P / (ms * 1e-3), "dtype": "bf16", "data": "synthetic",
        "activations_per_call": st["n_activations"][0] // (reps + 1),
        "roofline": {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "flops_per_call": flops}}))
    eng.close()


def timeline_mode(args):
    """--timeline: where the time of one decode launch goes.  Runs the workload's shapes (4 layers,
    prompt = budget, so the cache is at its budget) on the instrumented build of the library
    (liblazyev_timeline.so: every block of the fused decode kernel leaves time stamps of the
    100 MHz counter) and prints, over the blocks of the sampled launches, when the stream, the
    ticket and the block end fall, counted from the start of the launch's first block."""
    os.environ["LAZYEV_LIBRARY"] = "liblazyev_timeline.so"
    import numpy as np
    import torch
    from paper_2506_15969_amd import binding
    from paper_2506_15969_amd.workload import CONFIGS, Workload
    base = CONFIGS[args.config]
    L, steps = 4, max(args.steps or 40, 24)
    P = args.prompt_len if args.prompt_len >= 0 else base.budget
    cfg = base.scaled(n_layers=L, prompt_len=P, steps=steps)
    wl = Workload(cfg)
    eng = binding.LazyEviction(L, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.budget,
                               cfg.window, cfg.prompt_len, cfg.alpha, dtype=cfg.torch_dtype)
    for l in range(L):
        eng.load_prompt(l, *wl.prompt_kv(l, device="cuda"))
    eng.init()
    if args.target_blocks:
        eng.set_target_blocks(args.target_blocks)
    ins = [wl.step_inputs(l, 1, steps + 1, device="cuda") for l in range(L)]
    out = torch.empty((L, cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
    read = binding.lib.lazyev_timeline_read
    read.restype = C.c_int
    NB = 2048
    buf = (C.c_uint64 * (NB * 8))()
    samples = []
    for t in range(1, steps + 1):
        for l in range(L):
            q, kn, vn = ins[l]
            eng.decode_step(l, t, q[t - 1], kn[t - 1], vn[t - 1], out[l])
        if t > steps // 2:                            # the stamps of the step's last launch
            torch.cuda.synchronize()
            assert read(buf, NB * 8) == 0
            a = np.frombuffer(buf, dtype=np.uint64).reshape(NB, 8).astype(np.int64)
            live = a[:, 0] > 0
            stream = live & (a[:, 3] >= a[:, 0]) & (a[:, 2] >= a[:, 0])
            if stream.any():
                origin = a[stream, 0].min()
                trk = a[live & ~stream]
                trk = trk[trk[:, 5] >= trk[:, 0]]
                samples.append(((a[stream][:, :6] - origin) / 100.0, a[stream][:, 7],
                                (trk[:, [0, 5]] - origin) / 100.0, a[stream][:, 6],
                                np.nonzero(stream)[0]))
        eng.evict_all(t)                              # (fires where the schedule says so)
    n1 = eng.stats()["len"][0]
    names = ["block start", "first sub-tile multiplied", "end of wave 0's stream", "all four waves done",
             "ticket taken", "block end"]

    def q(x):
        return {"min": round(float(np.min(x)), 2), "p50": round(float(np.median(x)), 2),
                "p90": round(float(np.percentile(x, 90)), 2), "max": round(float(np.max(x)), 2)}
    res = {"what": "in-kernel timeline of decode_fused_kernel, microseconds from the start of the launch's "
                   "first block, over the stream blocks of %d launches" % len(samples),
           "config": {"workload": "%s-prompt%d" % (base.name, P), "layers": L, "entries_per_unit_at_the_end": n1,
                      "stream_blocks_per_launch": int(samples[0][0].shape[0])},
           "stamps": {n: dict(q(np.concatenate([s[0][:, i] for s in samples])),
                              mean_of_per_launch_max=round(float(np.mean([s[0][:, i].max() for s in samples])), 2),
                              mean_of_per_launch_min=round(float(np.mean([s[0][:, i].min() for s in samples])), 2))
                      for i, n in enumerate(names)},
           "finisher_tail_us (block end - end of its stream)":
               q(np.concatenate([(s[0][:, 5] - s[0][:, 2])[s[1] == 1] for s in samples])),
           # (the tracking blocks of the launch apply the PREVIOUS call's tracking; the first call of a
           # layer has none)
           "tracking_blocks": ({"start": q(np.concatenate([s[2][:, 0] for s in samples])),
                                "end": q(np.concatenate([s[2][:, 1] for s in samples]))}
                               if sum(len(s[2]) for s in samples) else {})}
    # Which blocks end their stream late: by the XCD they ran on, by their place among the unit's
    # blocks, and how far the blocks of one unit lie apart.
    end = np.concatenate([s[0][:, 2] for s in samples])
    xcd = np.concatenate([s[3] for s in samples])
    blk = np.concatenate([s[4] for s in samples])
    n_split = max(1, int(samples[0][0].shape[0]) // (cfg.batch * cfg.n_kv_heads))
    res["stream_end_by_xcd"] = {str(int(x)): {"blocks_per_launch": round(float((xcd == x).sum()) / len(samples), 1),
                                              "mean": round(float(end[xcd == x].mean()), 2)}
                                for x in np.unique(xcd)}
    res["stream_end_by_block_of_the_unit"] = {str(j): round(float(end[blk % n_split == j].mean()), 2)
                                              for j in range(n_split)}
    res["xcd_of_block_index_mod_8"] = {str(j): sorted(int(x) for x in np.unique(xcd[blk % 8 == j])) for j in range(8)}
    per_unit = [s[0][:, 2].reshape(-1, n_split) for s in samples]
    res["spread_of_a_unit's_blocks (latest - earliest stream end)"] = q(
        np.concatenate([u.max(axis=1) - u.min(axis=1) for u in per_unit]))
    fin = np.concatenate([s[1] == 1 for s in samples])
    st = np.concatenate([s[0] for s in samples])
    res["finishing_blocks"] = {"partials complete - all four waves done": q((st[:, 4] - st[:, 3])[fin]),
                               "block end - partials complete": q((st[:, 5] - st[:, 4])[fin]),
                               "stream end": q(st[fin, 2])}
    res["other_blocks"] = {"block end - all four waves done": q((st[:, 5] - st[:, 3])[~fin]),
                           "stream end": q(st[~fin, 2])}
    # the block that ends a launch: did it stream longest, or did it wait for another block's partial?
    last = [int(np.argmax(s[0][:, 5])) for s in samples]
    res["last_block_of_a_launch"] = {
        "is_the_block_whose_stream_ended_last": round(float(np.mean([int(i == int(np.argmax(s[0][:, 2]))) for i, s in zip(last, samples)])), 2),
        "finishes_its_unit": round(float(np.mean([float(s[1][i] == 1) for i, s in zip(last, samples)])), 2),
        "stream end": q(np.array([s[0][i, 2] for i, s in zip(last, samples)])),
        "partials complete - all four waves done": q(np.array([s[0][i, 4] - s[0][i, 3] for i, s in zip(last, samples)])),
        "block end - end of its stream": q(np.array([s[0][i, 5] - s[0][i, 2] for i, s in zip(last, samples)]))}
    res["per_launch"] = {"stream_end_sigma": round(float(np.mean([s[0][:, 2].std() for s in samples])), 2),
                         "mean_stream_end": round(float(np.mean([s[0][:, 2].mean() for s in samples])), 2),
                         "latest_stream_end": round(float(np.mean([s[0][:, 2].max() for s in samples])), 2)}
    print(json.dumps(res))
    eng.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed decode steps (0: the config's)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--chunk", type=int, default=0, help="split-block size override")
    ap.add_argument("--input-gb", type=float, default=150.0,
                    help="cap on the inputs kept in HBM; beyond it later steps reuse them cyclically")
    ap.add_argument("--profile-every", type=int, default=0,
                    help="bracket the layer calls of every this many steps with a HIP event pair "
                         "(0: every step up to 1024 timed steps, every 16th beyond)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--from-prompt", action="store_true",
                    help="time the K steps from the workload's own prompt even when K is too short "
                         "to reach the first eviction (the cache then stays below its budget)")
    ap.add_argument("--prompt-len", type=int, default=-1,
                    help="override the workload's prompt length and time from that prompt")
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
    ap.add_argument("--single-call-window", action="store_true",
                    help="after the timed region, run one more untimed window of W steps with ONE "
                         "layer call per step bracketed by the library's own events "
                         "(roofline.single_call)")
    ap.add_argument("--prefill-track", action="store_true",
                    help="time lazyev_prefill_track on one layer instead of the decode path "
                         "(--prompt-len positions, default 2048; --steps repetitions, default 5)")
    ap.add_argument("--timeline", action="store_true",
                    help="per-block timeline of the fused decode kernel from the instrumented build "
                         "of the library (liblazyev_timeline.so) instead of the throughput run")
    ap.add_argument("--progress", type=int, default=0,
                    help="write a line to stderr every this many submitted steps (long runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path has no cross-GPU part "
              "(every (layer, sequence, KV head) unit is independent). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)
    if args.prefill_track:
        prefill_track_mode(args)
        return
    if args.timeline:
        timeline_mode(args)
        return

    import torch
    from paper_2506_15969_amd import binding
    from paper_2506_15969_amd.workload import CONFIGS, Workload

    cfg = CONFIGS[args.config]
    K = args.steps or cfg.steps
    if args.window > 0:
        cfg = cfg.scaled(window=args.window, name="%s-window%d" % (cfg.name, args.window))
    W = cfg.window

    def first_eviction(c):
        """First step after which an eviction fires: the smallest t = kW with P + t > B."""
        return (max(c.budget - c.prompt_len, 0) // c.window + 1) * c.window

    # ---- where the K timed steps lie
    steady = (not args.from_prompt and args.prompt_len < 0 and not args.no_evict and not args.ragged
              and K < first_eviction(cfg) and cfg.dtype == "bf16" and cfg.head_dim == 128)
    pre = 0
    if steady:
        cfg = cfg.scaled(prompt_len=cfg.budget, name=cfg.name + "-steady")
        if K < W:
            pre = W - (K + 1) // 2                  # the timed steps pre+1 .. pre+K straddle t = W
    elif args.prompt_len >= 0:
        cfg = cfg.scaled(prompt_len=args.prompt_len, name="%s-prompt%d" % (cfg.name, args.prompt_len))
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
    L, S, Hq, Hkv, d = cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    esz = 4 if cfg.dtype == "fp32" else 2
    follow = W if args.single_call_window else 0    # untimed steps after the timed ones
    total_steps = pre + K + follow

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
        if steady:
            # TS / MRI of the budget-long prompt from the prompt's own attention, so that the
            # eviction ranks a varied state and not 2048 untouched entries
            for l in range(L):
                eng.prefill_track(l, wl.prompt_queries(l, device=dev))
        if args.ragged:
            for sq in range(S):                     # (the prompt rows are in the caches already)
                eng.admit(sq, cfg.prompt_len, sq % W)

    # ---- inputs resident in HBM
    per_step = L * S * (Hq + 2 * Hkv) * d * esz
    R = max(1, min(total_steps, int(args.input_gb * 1e9 // per_step)))
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

    lib = binding.lib
    q_base, k_base, v_base, o_base = q_all.data_ptr(), k_all.data_ptr(), v_all.data_ptr(), out.data_ptr()
    q_sz, kv_sz = S * Hq * d * esz, S * Hkv * d * esz
    decode, evict = lib.lazyev_decode_step, lib.lazyev_evict

    # cache length (after the append) seen by the decode call of step t: closed form of the
    # saw-tooth, used to attach algorithmic bytes to the bracketed calls
    first = first_eviction(cfg)

    def n1_at(t):
        if t <= first:
            return cfg.prompt_len + t
        last_ev = (t - 1) // W * W
        return cfg.budget + (t - last_ev)

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

    def due_at(t):
        return t % W == 0 and n1_at(t) > cfg.budget

    brackets = []                                    # (step, event before layer 0, event after layer L-1)

    def run(t_from, t_to, bracket_every=0, single_call=False):
        """Decode steps t_from .. t_to.  bracket_every: one event pair around the L layer calls
        of every bracket_every-th step (the due eviction comes after the closing event).
        single_call: the library brackets ONE layer call per step itself (the layer rotates)."""
        ctx = eng._ctx
        for t in range(t_from, t_to + 1):
            r = (t - 1) % R
            bracket = bracket_every and (t - t_from) % bracket_every == 0
            armed = t % L if single_call else -1
            if bracket:
                ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                ev[0].record()
            for l in range(L):
                i = r * L + l
                if l == armed:
                    lib.lazyev_profile_arm(ctx, 1)
                rc = decode(ctx, l, t, q_base + i * q_sz, k_base + i * kv_sz, v_base + i * kv_sz,
                            o_base + l * q_sz, None, None)
                if rc:
                    raise binding.LazyevError(rc, "lazyev_decode_step(layer %d, t %d), HIP error %d"
                                              % (l, t, lib.lazyev_last_hip_error(ctx)))
            if bracket:
                ev[1].record()
                brackets.append((t, ev[0], ev[1]))
            if args.ragged:                                  # the library knows which sequences are due
                rc = lib.lazyev_evict_all(ctx, t, None)
                if rc:
                    raise binding.LazyevError(rc, "lazyev_evict_all(t %d)" % t)
            elif t % W == 0:
                due = due_at(t)
                if args.evict_per_layer:
                    for l in range(L):
                        if l == 0 and due and bracket_every:
                            lib.lazyev_profile_arm(ctx, 1)
                        rc = evict(ctx, l, t, None)
                        if rc:
                            raise binding.LazyevError(rc, "lazyev_evict(layer %d, t %d)" % (l, t))
                else:                                        # all layers in one launch pair
                    if due and bracket_every:
                        lib.lazyev_profile_arm(ctx, 1)       # select and move kernels, timed apart
                    rc = lib.lazyev_evict_all(ctx, t, None)
                    if rc:
                        raise binding.LazyevError(rc, "lazyev_evict_all(t %d)" % t)
            if args.progress and t % args.progress == 0:
                print("bench.py: step %d of %d submitted" % (t, t_to), file=sys.stderr, flush=True)

    # ---- warm-up on a throw-away pass, then the state the timed steps start from
    reset_state()
    run(1, args.warmup)
    torch.cuda.synchronize()
    reset_state()
    run(1, pre)                                      # untimed pre-roll (steady state only)
    st0 = eng.stats()                                # (applies pending tracking, waits for the stream)
    eng.profile_read()                               # forget anything armed so far
    every = args.profile_every or (1 if K <= 1024 else 16)
    t_start = time.perf_counter()
    run(pre + 1, pre + K, every)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    prof = eng.profile_read()
    st = eng.stats()
    timed_evictions = sum(1 for t in range(pre + 1, pre + K + 1) if due_at(t)) if not args.ragged else None

    single = None
    if follow:
        run(pre + K + 1, pre + K + follow, 0, single_call=True)
        torch.cuda.synchronize()
        single = eng.profile_read()

    probes = binding.bench_lib()
    stream_ptr = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    if args.calibrate_copy_mb:
        nbytes = args.calibrate_copy_mb << 20
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        probes.lazyev_stream_probe(dst.data_ptr(), src.data_ptr(), nbytes, 2048, stream_ptr)
        torch.cuda.synchronize()
        del src, dst
    # what a plain streaming read reaches on this machine (1 GiB, non-temporal loads, two blocks per
    # compute unit): the second denominator beside the published peak
    probe_bytes = 1 << 30
    probe_src = torch.empty(probe_bytes, dtype=torch.uint8, device=dev).random_(0, 255)
    probe_sink = torch.zeros(4, dtype=torch.int32, device=dev)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    probes.lazyev_stream_read_probe(probe_src.data_ptr(), probe_bytes, 512, probe_sink.data_ptr(), stream_ptr)
    ev0.record()
    for _ in range(5):
        probes.lazyev_stream_read_probe(probe_src.data_ptr(), probe_bytes, 512, probe_sink.data_ptr(), stream_ptr)
    ev1.record()
    torch.cuda.synchronize()
    read_probe_gbs = 5 * probe_bytes / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del probe_src
    # what a pair of HIP events adds to the interval it brackets (empty kernel, same stream)
    ov = C.c_double(0.0)
    probes.lazyev_event_overhead(200, stream_ptr, C.byref(ov))
    ov_ms = ov.value

    timed_steps = list(range(pre + 1, pre + K + 1))
    n1s = [n1_at(t) for t in timed_steps] if not args.ragged else []
    steps_per_s = K / elapsed
    with_ev = bool(timed_evictions) or (args.ragged and sum(st["n_evict_events"]) > sum(st0["n_evict_events"]))
    result = {
        "metric": "decode steps/s at batch %d, budget %d (%s); tokens/s = value x batch"
                  % (S, cfg.budget, "incl. eviction" if with_ev else
                     "NO eviction fell into the timed steps: the cache is below its budget"),
        "value": steps_per_s, "unit": "steps/s", "tokens_per_s": steps_per_s * S,
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": 1e3 * elapsed / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": L, "batch": S, "q_heads": Hq, "kv_heads": Hkv,
                   "head_dim": d, "prompt_len": cfg.prompt_len, "budget": cfg.budget,
                   "window": W, "alpha": cfg.alpha, "input_steps_resident": R,
                   "placement": ("steady state: prompt = budget with TS/MRI from the prompt's own "
                                 "attention, %d untimed pre-roll steps, timed steps t = %d..%d"
                                 % (pre, pre + 1, pre + K)) if steady else
                                "from the prompt: timed steps t = 1..%d" % K,
                   "entries_per_unit_in_timed_steps": [min(n1s), max(n1s)] if n1s else None,
                   "mean_entries_per_unit": sum(n1s) / len(n1s) if n1s else None,
                   "evictions_in_timed_region": timed_evictions,
                   "evictions_per_layer": st["n_evict_events"][0] - st0["n_evict_events"][0],
                   "activations_per_unit_step": (sum(st["n_activations"]) - sum(st0["n_activations"]))
                                                / (K * L * S * Hkv)},
        "input_generation_s": t_gen,
    }
    if steady and K < W:
        # one eviction per K < W steps over-weights it; what a whole window of W such steps costs
        sel_ms, sel_n = prof["select"]
        mov_ms, mov_n = prof["move"]
        if sel_n and mov_n:
            ev_ms = (sel_ms + mov_ms) / sel_n
            dec_ms = (1e3 * elapsed - ev_ms * timed_evictions) / K
            result["config"]["steps_per_s_over_a_whole_window"] = 1e3 / (dec_ms + ev_ms / W)
    fused = cfg.dtype == "bf16" and d == 128 and args.variant in (-1, 1, 4, 5, 6)
    if brackets:
        group_ms = sum(a.elapsed_time(b) for _, a, b in brackets)
        n_launch = L * len(brackets)
        dec_bytes = sum(bytes_at(t) for t, _, _ in brackets) * L
        avg_us = 1e3 * group_ms / n_launch
        ach = dec_bytes / (group_ms * 1e-3) / 1e9
        roof = {
            "kernel": ("decode_fused_kernel (the one kernel of lazyev_decode_step)"
                       if fused else "the two kernels of lazyev_decode_step (split, merge)"),
            "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBS, "traffic": None,
            "avg_us": avg_us, "launches_timed": n_launch,
            "algorithmic_bytes_per_launch": dec_bytes / n_launch,
            "how": "one HIP event pair on the library's stream around the %d layer calls of a step, "
                   "interval / %d, nothing subtracted (the pair itself costs %.1f us per step, the "
                   "turn-around between two dependent launches is inside)" % (L, L, 1e3 * ov_ms),
            "plain_read_on_this_box": {"GB/s": read_probe_gbs, "frac_of_it": ach / read_probe_gbs,
                                       "what": "1 GiB read once with non-temporal loads, grid-stride, 512 blocks of 256 threads"},
        }
        prof_n1 = PROFILED_TRAFFIC.get(cfg.name.split("-")[0])
        mean_n1 = result["config"]["mean_entries_per_unit"]
        if fused and prof_n1 and mean_n1 and abs(mean_n1 - prof_n1[0]) <= 0.01 * prof_n1[0]:
            roof["traffic"] = prof_n1[1]
            roof["traffic_source"] = ("profiles/decode_fused_%s_steady.txt (FETCH_SIZE x 2 + WRITE_SIZE per "
                                      "launch at a mean of %.1f entries per unit; this run: %.1f); a "
                                      "profile constant, not a counter read in this run"
                                      % (cfg.name.split("-")[0], prof_n1[0], mean_n1))
        if single and single["split"][1]:
            s_ms, s_n = single["split"]
            c_ms, c_n = single["combine"]
            tf = range(pre + K + 1, pre + K + follow + 1)
            b1 = sum(bytes_at(t) for t in tf) / len(tf)
            k_us = 1e3 * (s_ms - ov_ms * s_n) / s_n
            roof["single_call"] = {
                "what": "untimed follow-up window of %d steps, ONE layer call per step between two events "
                        "recorded by the library, the cost of an empty event pair subtracted" % follow,
                "avg_us": k_us, "avg_us_between_events": 1e3 * s_ms / s_n,
                "event_pair_overhead_us": 1e3 * ov_ms, "launches_timed": s_n,
                "algorithmic_bytes_per_launch": b1, "frac": b1 / (k_us * 1e-6) / 1e9 / HBM_PEAK_GBS}
        sel_ms, sel_n = prof["select"]
        mov_ms, mov_n = prof["move"]
        if mov_n:
            events = sum(st["n_evict_events"]) - sum(st0["n_evict_events"])
            rows = sum(st["n_rows_moved"]) - sum(st0["n_rows_moved"])
            # bytes of one launch of the row-move kernel: one layer's, or all layers' at once
            mb = algorithmic_bytes_move(cfg, rows / max(events, 1)) * (1 if args.evict_per_layer else L)
            mov_k = mov_ms - ov_ms * mov_n
            roof["compaction"] = {
                "kernel": "evict_move_kernel", "layers_per_launch": 1 if args.evict_per_layer else L,
                "avg_us": 1e3 * mov_k / mov_n,
                "select_avg_us": 1e3 * (sel_ms - ov_ms * sel_n) / sel_n, "launches_timed": mov_n,
                "algorithmic_bytes_per_launch": mb,
                "rows_moved_per_unit_event": rows / max(events, 1) / (S * Hkv),
                "achieved": mb / (mov_k / mov_n * 1e-3) / 1e9,
                "frac": mb / (mov_k / mov_n * 1e-3) / 1e9 / HBM_PEAK_GBS}
        # whole-step view: all algorithmic decode bytes of the timed steps over the wall time
        tot = sum(bytes_at(t) for t in timed_steps) * L
        roof["whole_run_frac"] = tot / elapsed / 1e9 / HBM_PEAK_GBS
        result["roofline"] = roof
    if not args.no_cpu_baseline:
        eng.close()
        del q_all, k_all, v_all
        result["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
