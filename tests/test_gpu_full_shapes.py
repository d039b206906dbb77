"""The HIP library against the oracle at the shapes the benchmark times (full batch, head
counts, capacity and block split of the five workloads), on a seeded sample of units: the
oracle follows only the sampled (layer, sequence, KV head) units, the library runs every unit.
Prompts are set to the budget so that the cache is in its steady state (eviction every W steps)
from the first step on; workload 2 is also run at its full length."""
import numpy as np
import pytest

from paper_2506_15969_amd.workload import CONFIGS

pytestmark = pytest.mark.gpu


def _sample(cfg, n, seed, layers):
    rng = np.random.default_rng(seed)
    units = set()
    while len(units) < n:
        units.add((int(rng.choice(layers)), int(rng.integers(cfg.batch)), int(rng.integers(cfg.n_kv_heads))))
    return sorted(units)


def _report(name, stat):
    print("\n[%s] steps=%d decisions=%d near-threshold disagreements=%d evictions=%d "
          "max out err=%.3g max p err=%.3g" % (name, stat["steps"], stat["decisions"],
                                               stat["near_threshold"], stat["evictions"],
                                               stat["max_out_err"], stat["max_p_err"]), flush=True)


@pytest.mark.parametrize("name,steps,n_units", [("cfg3", 130, 6), ("cfg4", 260, 6), ("cfg5", 130, 4)])
def test_benchmark_shapes_in_steady_state(lazyev_lib, name, steps, n_units):
    from lockstep import run_lockstep
    base = CONFIGS[name]
    cfg = base.scaled(n_layers=2, prompt_len=base.budget, steps=steps,
                      interval_lo=min(base.interval_lo, 16), interval_hi=min(base.interval_hi, 64),
                      schedule="uniform" if base.schedule == "bursty" else base.schedule)
    units = _sample(cfg, n_units, base.seed, [0, 1])
    stat = run_lockstep(lazyev_lib, cfg, units, mode="e2e")
    _report(name + "/steady", stat)
    per_layer = steps // cfg.window
    assert stat["evictions"] == per_layer * len({u[0] for u in units})
    assert stat["near_threshold"] <= max(4, stat["decisions"] // 20000)


def test_benchmark_shapes_weights_injected(lazyev_lib):
    """Identical weights on both sides: every decision and every survivor set must agree."""
    from lockstep import run_lockstep
    base = CONFIGS["cfg3"]
    cfg = base.scaled(n_layers=1, prompt_len=base.budget, steps=130, interval_lo=16, interval_hi=64)
    units = _sample(cfg, 4, 11, [0])
    for mode in ("oracle_p", "synthetic"):
        stat = run_lockstep(lazyev_lib, cfg, units, mode=mode)
        assert stat["evictions"] == 2 and stat["near_threshold"] == 0


def test_cfg2_full_length_on_sampled_units(lazyev_lib):
    """Workload 2 at its full length: 512-token prompt, 4096 steps, 112 evictions."""
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg2"]
    units = _sample(cfg, 2, 2, [0])
    from paper_2506_15969_amd.workload import Workload
    wl = Workload(cfg)
    early = {int(j) for j, tau in zip(wl.planted, wl.period) if j < cfg.prompt_len and 0 < tau <= 256}
    stat = run_lockstep(lazyev_lib, cfg, units, mode="e2e", watch=early)
    _report("cfg2/full", stat)
    assert stat["evictions"] == 112
    assert stat["near_threshold"] <= max(4, stat["decisions"] // 20000)
    # The survivor sets are the oracle's (compared above, exactly).  What Eq. 3 promises for the
    # recurring keys planted in the prompt: H1 falls below 2*sigmoid(-1) only once the time since
    # the last activation exceeds the longest interval seen so far, so such a key can only have
    # been dropped at an eviction where it was overdue by its own record (t - TS > MRI).  On this
    # workload background entries are activated by chance about every 33 steps, which cuts a
    # planted period of 150-250 steps into shorter recorded intervals: a few of the nine keys
    # are overdue in that sense at some eviction and go (the rest stay to the end).
    for u, lost in stat["evicted_watch"].items():
        for pos, t, ts, mri in lost:
            assert t - ts > mri, ("a recurring key dropped although it was not overdue", u, pos, t, ts, mri)
        kept = early & set(stat["oracle_units"][u].pos.tolist())
        assert kept == early - {x[0] for x in lost} and len(kept) >= 1


@pytest.mark.parametrize("name,prompt_len,budget,target_blocks,n_ev",
                         [("cfg3", 2048, 2048, None, 2), ("cfg5", 4096, 4096, None, 2),
                          # runs of 47 sub-tiles per wave: the lists are written segment by segment
                          ("cfg3", 6000, 6000, 256, 2),
                          # the cache grows across the change of split (4 -> 6 blocks per unit)
                          ("cfg3", 5080, 8000, None, 0),
                          # one block per unit and 100 sub-tiles per wave
                          ("cfg5", 6400, 8000, 128, 0)])
def test_candidate_lists_leave_the_same_state_as_all_logits(lazyev_lib, name, prompt_len, budget,
                                                            target_blocks, n_ev):
    """Benchmark shapes, two layers, 70 steps: the default (candidate lists for the deferred
    tracking at these cache lengths) against the same kernel keeping every logit: outputs,
    caches, TS / MRI / pos and counters bit for bit."""
    import torch
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import Workload
    base = CONFIGS[name]
    cfg = base.scaled(n_layers=2, prompt_len=prompt_len, budget=budget, steps=70)
    wl = Workload(cfg)
    runs = []
    for variant in (4, 5):
        eng = make_engine(lazyev_lib, cfg, wl, variant=variant, target_blocks=target_blocks)
        out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
        ins = [wl.step_inputs(l, 1, cfg.steps + 1, device="cuda") for l in range(cfg.n_layers)]
        acc = torch.zeros_like(out, dtype=torch.float32)
        n_ev = 0
        for t in range(1, cfg.steps + 1):
            for l in range(cfg.n_layers):
                q, kn, vn = ins[l]
                eng.decode_step(l, t, q[t - 1], kn[t - 1], vn[t - 1], out)
                acc += out.float() * (1 + (t + l) % 7)
            for l in range(cfg.n_layers):
                n_ev += 1 if eng.evict(l, t) else 0
        st = eng.stats()
        n = st["len"][0]
        runs.append((acc, eng.k_cache[:, :, :, :n].clone(), eng.ts[:, :, :, :n].clone(),
                     eng.mri[:, :, :, :n].clone(), eng.pos[:, :, :, :n].clone(), st, n_ev))
        eng.close()
    a, b = runs
    assert a[6] == b[6] == n_ev and a[5] == b[5] and sum(a[5]["n_activations"]) > 0
    for x, y in zip(a[:5], b[:5]):
        assert torch.equal(x, y)


@pytest.mark.parametrize("prompt_len,steps,budget", [(5200, 24, 4096), (8000, 24, 4096), (5100, 40, 4096),
                                                     (1780, 30, 2048)])
def test_long_prompt_with_the_default_block_split(lazyev_lib, prompt_len, steps, budget):
    """Caches beyond the benchmark budgets at cfg3's batch and head counts (full-cache decoding, or
    a prompt that exceeds the budget): the library then uses more blocks per unit so that a
    wave's run still fits on chip (6 and 9 per unit for 5200 and 8000 entries).  From 5100
    entries the cache grows across the length where the split changes from 4 to 6 blocks, so the
    tracking blocks of one call read the candidate lists of a call with another split; from 1780
    it grows across the length where candidate lists replace the full logits.  Sampled units
    against the oracle, with the eviction at the last step where one is due."""
    from lockstep import run_lockstep
    base = CONFIGS["cfg3"]
    cfg = base.scaled(n_layers=1, prompt_len=prompt_len, steps=steps, budget=budget, window=steps,
                      interval_lo=4, interval_hi=12, schedule="uniform")
    units = _sample(cfg, 3, prompt_len, [0])
    stat = run_lockstep(lazyev_lib, cfg, units, mode="e2e")
    _report("long-prompt-%d" % prompt_len, stat)
    due = prompt_len + steps > budget
    assert stat["evictions"] == (1 if due else 0) and stat["near_threshold"] <= 2
    for u in stat["oracle_units"].values():
        assert len(u) == (budget if due else prompt_len + steps)
