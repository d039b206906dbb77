"""HIP library against the CPU oracle, through the C ABI, on the same seeded inputs."""
import itertools

import numpy as np
import pytest
import torch

from paper_2506_15969_amd.workload import CONFIGS

pytestmark = pytest.mark.gpu


def _all_units(cfg, layers=None):
    return [(l, s, h) for l in (layers or range(cfg.n_layers)) for s in range(cfg.batch)
            for h in range(cfg.n_kv_heads)]


def _report(name, stat):
    print("\n[%s] steps=%d decisions=%d near-threshold disagreements=%d evictions=%d "
          "max out err=%.3g max p err=%.3g" % (name, stat["steps"], stat["decisions"],
                                               stat["near_threshold"], stat["evictions"],
                                               stat["max_out_err"], stat["max_p_err"]), flush=True)


@pytest.mark.parametrize("mode", ["e2e", "oracle_p", "synthetic"])
def test_cfg1_fp32_every_unit_every_step(lazyev_lib, mode):
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg1"]
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode=mode)
    _report("cfg1/" + mode, stat)
    assert stat["evictions"] == 28                       # t = 80, 96, ..., 512
    if mode != "e2e":
        assert stat["near_threshold"] == 0
    else:
        assert stat["near_threshold"] <= 2
        # planted keys are still cached at the end, in every head
        from paper_2506_15969_amd.workload import Workload
        planted = set(Workload(cfg).planted.tolist())
        for u in stat["oracle_units"].values():
            assert planted <= set(u.pos.tolist())
    acts = sum(u.n_activations for u in stat["oracle_units"].values())
    assert stat["gpu_stats"]["n_activations"][0] == acts
    assert stat["gpu_stats"]["n_evict_events"][0] == 28
    assert stat["gpu_stats"]["n_evicted"][0] == 28 * 16
    assert stat["gpu_stats"]["n_rows_moved"][0] == stat["rows_moved"] > 0


@pytest.mark.parametrize("mode,variant,knob", [("e2e", 0, 128), ("e2e", 0, 64), ("oracle_p", 0, 128),
                                               ("synthetic", 0, 256),
                                               ("e2e", 4, 8), ("e2e", 4, 16), ("e2e", 4, 24),
                                               ("e2e", 4, 32), ("e2e", 4, 40),
                                               ("e2e", 4, 1000), ("oracle_p", 4, 32),
                                               ("synthetic", 4, 40)])
def test_cfg2_shapes_scaled_down(lazyev_lib, mode, variant, knob):
    """bf16, 28/4 heads, d=128; cache up to 170+32 entries (7 tiles of 32, ragged tail).
    variant 4 is the single-launch MFMA kernel, `knob` its target block count (8 units: 1, 2, 3,
    4, 5 blocks per unit: alone, partials handed over to the unit's last block, tickets; and as
    many as the cache length allows: waves with one or no sub-tile);
    variant 0 is the vector-ALU kernel, `knob` its chunk."""
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg2"].scaled(batch=2, prompt_len=100, steps=330, budget=170, window=32,
                                 interval_lo=20, interval_hi=120)
    kw = dict(target_blocks=knob) if variant == 4 else dict(chunk=knob)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode=mode, variant=variant, **kw)
    _report("cfg2-small/%s/variant%d/knob%d" % (mode, variant, knob), stat)
    assert stat["evictions"] == len([t for t in range(32, 331, 32) if 100 + t > 170])


@pytest.mark.parametrize("name,dtype,hq,hkv,d", [("g1-fp32-d128", "fp32", 2, 2, 128),
                                                 ("g5-bf16-d128", "bf16", 10, 2, 128),
                                                 ("g8-bf16-d64", "bf16", 8, 1, 64),
                                                 ("g2-fp32-d64", "fp32", 4, 2, 64)])
def test_other_head_shapes(lazyev_lib, name, dtype, hq, hkv, d):
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg2"].scaled(batch=2, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, dtype=dtype,
                                 prompt_len=70, steps=200, budget=150, window=20,
                                 interval_lo=20, interval_hi=80)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="e2e", chunk=64)
    _report(name, stat)
    assert stat["evictions"] > 0


@pytest.mark.parametrize("flags", [0, 1, 2, 2 | 16, 3 | 16])
def test_score_ablation_flags(lazyev_lib, flags):
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg1"].scaled(steps=200)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="oracle_p", score_flags=flags)
    assert stat["evictions"] > 0 and stat["near_threshold"] == 0


def test_mri_histogram_matches_the_oracle(lazyev_lib):
    """Every unit in the oracle: the library's MRI histogram of the layer equals the oracle's,
    bin by bin, overflow bin included; and the window derived from it is the oracle's."""
    from lockstep import run_lockstep
    from oracle.lazyev_oracle import window_from_mri
    cfg = CONFIGS["cfg2"].scaled(batch=2, prompt_len=64, steps=420, budget=484, window=32)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="e2e")      # full cache: no eviction
    assert stat["evictions"] == 0
    got, want = stat["gpu_mri_hist_layer"][0], stat["oracle_mri_hist_layer"][0]
    assert got == want and got == stat["gpu_mri_hist"]
    assert sum(got) == cfg.batch * cfg.n_kv_heads * 484 and got[-1] > 0 and sum(got[1:]) > 100
    eng = stat["engine"]
    all_mri = np.concatenate([u.MRI for u in stat["oracle_units"].values()])
    wide = eng.mri_histogram(0, 1024)
    assert lazyev_lib.window_from_histogram(wide) == window_from_mri(all_mri)
    assert lazyev_lib.window_from_histogram(wide, 0.5) == window_from_mri(all_mri, 0.5)
    with pytest.raises(lazyev_lib.LazyevError):
        eng.mri_histogram(0, 1)
    with pytest.raises(lazyev_lib.LazyevError):
        eng.mri_histogram(1, 16)
    # with eviction: same comparison on what is left in the cache
    cfg = CONFIGS["cfg1"]
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="e2e")
    assert stat["gpu_mri_hist_layer"][0] == stat["oracle_mri_hist_layer"][0]


@pytest.mark.parametrize("window", [1, 16])
def test_current_attention_ranking(lazyev_lib, window):
    """Score = the weight an entry received at the eviction's own step (the greedy baselines'
    rule): per step with W = 1, behind an observation window with W = 16.  The oracle ranks and
    thresholds the library's exported fp32 weights, so survivors and statistics are exact."""
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg2"].scaled(batch=2, prompt_len=150, steps=120, budget=128, window=window)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="gpu_p",
                        score_flags=lazyev_lib.SCORE_CURRENT_ATTENTION)
    _report("current attention, W=%d" % window, stat)
    assert stat["evictions"] == 120 // window            # the prompt is longer than the budget


def test_current_attention_ranking_needs_the_call_that_made_the_weights(lazyev_lib):
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import Workload
    cfg = CONFIGS["cfg2"].scaled(n_layers=2, batch=1, prompt_len=40, steps=4, budget=32, window=1)
    wl = Workload(cfg)
    eng = make_engine(lazyev_lib, cfg, wl, score_flags=lazyev_lib.SCORE_CURRENT_ATTENTION)
    out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
    ins = [wl.step_inputs(l, 1, 3, device="cuda") for l in range(2)]
    for l in range(2):
        eng.decode_step(l, 1, ins[l][0][0], ins[l][1][0], ins[l][2][0], out)
    with pytest.raises(lazyev_lib.LazyevError):           # layer 0's weights have been overwritten
        eng.evict(0, 1)
    assert eng.evict(1, 1) == 9                           # 41 entries -> 32
    assert eng.evict(1, 1) == 0                           # nothing is due any more
    eng.set_variant(0)                                    # a kernel that keeps no logits
    eng.decode_step(1, 2, ins[1][0][1], ins[1][1][1], ins[1][2][1], out)
    with pytest.raises(lazyev_lib.LazyevError):
        eng.evict(1, 2)
    assert eng.stats()["len"] == [41, 33]


def test_empty_prompt_and_window_of_one(lazyev_lib):
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg1"].scaled(prompt_len=0, planted_count_in_prompt=0, steps=90, budget=40,
                                 window=1)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="e2e")
    assert stat["evictions"] == 50                       # every step from t = 41 on


def test_prompt_longer_than_budget(lazyev_lib):
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg1"].scaled(prompt_len=300, steps=64, budget=64, window=16,
                                 planted_count_in_prompt=8)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="e2e")
    assert stat["evictions"] == 4                        # first one drops 252 entries at once


def test_budget_at_least_sequence_is_full_attention(lazyev_lib):
    """No eviction ever fires, the cache just grows: plain attention over all tokens so far."""
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg2"].scaled(batch=1, prompt_len=40, steps=300, budget=340, window=16)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="e2e", variant=0, chunk=64)
    assert stat["evictions"] == 0 and stat["gpu_stats"]["len"][0] == 340
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="e2e", variant=4, target_blocks=3)
    assert stat["evictions"] == 0 and stat["gpu_stats"]["len"][0] == 340


@pytest.mark.parametrize("variant", [0, 4, 6])
def test_two_runs_are_bitwise_identical(lazyev_lib, variant):
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import Workload
    cfg = CONFIGS["cfg2"].scaled(batch=2, prompt_len=100, steps=130, budget=170, window=32)
    wl = Workload(cfg)
    snaps = []
    for _ in range(2):
        eng = make_engine(lazyev_lib, cfg, wl, variant=variant)
        out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
        outs = []
        q, kn, vn = wl.step_inputs(0, 1, cfg.steps + 1, device="cuda")
        for t in range(1, cfg.steps + 1):
            eng.decode_step(0, t, q[t - 1], kn[t - 1], vn[t - 1], out)
            outs.append(out.clone())
            eng.evict(0, t)
        torch.cuda.synchronize()
        snaps.append((torch.stack(outs), eng.k_cache.clone(), eng.ts.clone(), eng.mri.clone(),
                      eng.pos.clone()))
    (out_a, *state_a), (out_b, *state_b) = snaps
    for x, y in zip(state_a, state_b):                   # caches and recurrence state: bitwise
        assert torch.equal(x, y)
    assert torch.equal(out_a, out_b)


def test_hand_over_of_partials_reports_a_wait_that_ends(lazyev_lib):
    """Units of 2..4 blocks: the unit's last block waits (bounded) for the other blocks' partials.
    With the limit at 0 a block gives up as soon as a look finds a partial missing; every kernel
    still ends, the next lazyev_stats says so once, and with the limit back the engine goes on
    and reports nothing."""
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import Workload
    cfg = CONFIGS["cfg2"].scaled(n_layers=1, batch=8, prompt_len=600, steps=60, budget=1024, window=32)
    wl = Workload(cfg)
    eng = make_engine(lazyev_lib, cfg, wl, variant=4, target_blocks=2 * cfg.batch * cfg.n_kv_heads)
    out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
    q, kn, vn = wl.step_inputs(0, 1, cfg.steps + 1, device="cuda")
    eng.set_spin_ticks(0)
    for t in range(1, 41):
        eng.decode_step(0, t, q[t - 1], kn[t - 1], vn[t - 1], out)
    torch.cuda.synchronize()
    with pytest.raises(lazyev_lib.LazyevError) as err:
        eng.stats()
    assert err.value.code == lazyev_lib.EEXCHANGE
    eng.set_spin_ticks(2000000)
    assert eng.stats()["len"][0] == 640                  # reported once
    for t in range(41, 61):
        eng.decode_step(0, t, q[t - 1], kn[t - 1], vn[t - 1], out)
    assert eng.stats()["len"][0] == 660
    eng.close()


@pytest.mark.parametrize("blocks", [8, 24, 1000])
def test_deferred_tracking_equals_immediate(lazyev_lib, blocks):
    """The single-launch kernel applies the tracking of a call with the NEXT launch (or at the
    next lazyev_evict / lazyev_stats) unless the caller asks for the weights.  All routes must
    leave identical state: one engine is driven with p_out (tracked at once, the route the
    lock-step tests check against the oracle), one without and with every logit stored
    (kernel 5), one without and with candidate lists only (kernel 6); two layers interleaved;
    one, three and as many blocks per unit as the cache allows."""
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import Workload
    cfg = CONFIGS["cfg2"].scaled(n_layers=2, batch=2, prompt_len=100, steps=140, budget=170, window=32)
    wl = Workload(cfg)
    runs = []
    for immediate, variant in ((True, 4), (False, 5), (False, 6)):
        eng = make_engine(lazyev_lib, cfg, wl, variant=variant, target_blocks=blocks)
        out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
        p_out = torch.zeros((cfg.batch, cfg.n_q_heads, cfg.capacity), dtype=torch.float32, device="cuda")
        ins = [wl.step_inputs(l, 1, cfg.steps + 1, device="cuda") for l in range(cfg.n_layers)]
        outs, n_ev = [], 0
        for t in range(1, cfg.steps + 1):
            for l in range(cfg.n_layers):
                q, kn, vn = ins[l]
                eng.decode_step(l, t, q[t - 1], kn[t - 1], vn[t - 1], out,
                                p_out=p_out if immediate else None)
                outs.append(out.clone())
            for l in range(cfg.n_layers):
                n_ev += 1 if eng.evict(l, t) else 0
        st = eng.stats()                                  # applies what is still pending
        runs.append((torch.stack(outs), eng.k_cache.clone(), eng.v_cache.clone(), eng.ts.clone(),
                     eng.mri.clone(), eng.pos.clone(), st, n_ev))
    a = runs[0]
    for b in runs[1:]:
        assert a[7] == b[7] == 2 * len([t for t in range(32, 141, 32) if 100 + t > 170])
        for x, y in zip(a[:6], b[:6]):
            assert torch.equal(x, y)
        assert a[6] == b[6] and sum(a[6]["n_activations"]) > 0


@pytest.mark.parametrize("window,budget,steps", [(1, 120, 50), (2, 121, 60), (5, 400, 43), (7, 130, 90)])
def test_activation_log_with_short_windows(lazyev_lib, window, budget, steps):
    """The tracking of calls that nobody asks the weights of is kept as one bit per entry and
    applied to TS / MRI later (before an eviction, by lazyev_stats, or when the log's min(W, 256)
    slots are full).  Windows of 1, 2 and 7 steps (a log of one slot; evictions after every or
    every other step; applications that fall between evictions) and a budget that is never
    reached (the log is only ever applied because it is full, and once at the end): the state
    must equal, bit for bit, that of an engine whose every call is tracked at once (p_out); a
    lazyev_stats call in the middle of a window must not change that either."""
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import Workload
    cfg = CONFIGS["cfg2"].scaled(n_layers=2, batch=2, prompt_len=100, steps=steps, budget=budget, window=window)
    wl = Workload(cfg)
    runs = []
    for immediate, stats_at in ((True, 0), (False, 0), (False, 17)):
        eng = make_engine(lazyev_lib, cfg, wl, variant=6 if not immediate else 4, target_blocks=16)
        out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
        p_out = torch.zeros((cfg.batch, cfg.n_q_heads, cfg.capacity), dtype=torch.float32, device="cuda")
        ins = [wl.step_inputs(l, 1, cfg.steps + 1, device="cuda") for l in range(cfg.n_layers)]
        outs, n_ev = [], 0
        for t in range(1, cfg.steps + 1):
            for l in range(cfg.n_layers):
                q, kn, vn = ins[l]
                eng.decode_step(l, t, q[t - 1], kn[t - 1], vn[t - 1], out,
                                p_out=p_out if immediate else None)
                outs.append(out.clone())
                if t == stats_at and l == 0:
                    eng.stats()
            n_ev += eng.evict_all(t)
        st = eng.stats()
        runs.append((torch.stack(outs), eng.k_cache.clone(), eng.v_cache.clone(), eng.ts.clone(),
                     eng.mri.clone(), eng.pos.clone(), st, n_ev))
        eng.close()
    a = runs[0]
    for b in runs[1:]:
        assert a[7] == b[7]
        for x, y in zip(a[:6], b[:6]):
            assert torch.equal(x, y)
        assert a[6] == b[6] and sum(a[6]["n_activations"]) > 0
    assert (a[7] > 0) == (budget < 100 + steps)


def test_long_runs_per_wave(lazyev_lib):
    """One block per unit over a cache of 1400..1532 entries: every wave owns 22-24 sub-tiles,
    more than it keeps logits for in LDS, so the logits go out in two instalments."""
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg2"].scaled(batch=2, prompt_len=1400, steps=70, budget=1500, window=32,
                                 interval_lo=10, interval_hi=40)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="e2e", variant=4, target_blocks=8)
    _report("cfg2-long-runs", stat)
    assert stat["evictions"] == 0 and stat["near_threshold"] <= 2
    cfg = cfg.scaled(budget=1416, steps=40)
    stat = run_lockstep(lazyev_lib, cfg, _all_units(cfg), mode="oracle_p", variant=4, target_blocks=8)
    assert stat["evictions"] == 1 and stat["near_threshold"] == 0


@pytest.mark.parametrize("variant", [4, 0])
def test_evicting_all_layers_at_once_equals_layer_by_layer(lazyev_lib, variant):
    """lazyev_evict_all (selection and row move of all layers in one launch each) against one
    lazyev_evict per layer: three layers, 140 steps, two evictions, everything bit for bit."""
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import Workload
    cfg = CONFIGS["cfg2"].scaled(n_layers=3, batch=2, prompt_len=100, steps=140, budget=170, window=32)
    wl = Workload(cfg)
    runs = []
    for together in (False, True):
        eng = make_engine(lazyev_lib, cfg, wl, variant=variant)
        out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
        ins = [wl.step_inputs(l, 1, cfg.steps + 1, device="cuda") for l in range(cfg.n_layers)]
        outs, n_ev = [], 0
        for t in range(1, cfg.steps + 1):
            for l in range(cfg.n_layers):
                q, kn, vn = ins[l]
                eng.decode_step(l, t, q[t - 1], kn[t - 1], vn[t - 1], out)
                outs.append(out.clone())
            if together:
                n = eng.evict_all(t)
                n_ev += cfg.n_layers if n else 0
                assert eng.evict_all(t) == 0                  # a second request finds nothing due
            else:
                n_ev += sum(1 if eng.evict(l, t) else 0 for l in range(cfg.n_layers))
        st = eng.stats()
        runs.append((torch.stack(outs), eng.k_cache.clone(), eng.v_cache.clone(), eng.ts.clone(),
                     eng.mri.clone(), eng.pos.clone(), st, n_ev))
    a, b = runs
    assert a[7] == b[7] == 3 * 2
    for x, y in zip(a[:6], b[:6]):
        assert torch.equal(x, y)
    assert a[6] == b[6] and sum(a[6]["n_rows_moved"]) > 0


def test_evict_all_falls_back_when_layers_differ(lazyev_lib):
    """Layers at different steps: lazyev_evict_all reports the order error of the per-layer call."""
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import Workload
    cfg = CONFIGS["cfg2"].scaled(n_layers=2, batch=1, prompt_len=40, steps=4, budget=60, window=8)
    wl = Workload(cfg)
    eng = make_engine(lazyev_lib, cfg, wl)
    out = torch.empty((1, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
    q, kn, vn = wl.step_inputs(0, 1, 2, device="cuda")
    eng.decode_step(0, 1, q[0], kn[0], vn[0], out)            # layer 1 has not taken step 1
    with pytest.raises(lazyev_lib.LazyevError):
        eng.evict_all(1)
