"""The path the benchmark times, compared with the oracle directly: lazyev_decode_step without
exported or injected weights (the tracking of a call rides with the next launch and reads
candidate lists) and lazyev_evict_all for all layers at once.
The oracle follows a seeded sample of (layer, sequence, KV head) units on its own fp64 weights;
the library runs the whole batch at the workload's shapes.  Three kinds of run:

  steady state   prompt = budget, two layers: the state the headline metric is quoted on;
  all layers     the workload unmodified (its own prompt, schedule and ALL its layers) from the
                 prompt through the growth of the cache and its first evictions;
  full length    the workload's own prompt, schedule and ALL its steps on two layers: every
                 eviction of the closed-form schedule (228 / 122 / 456 per layer).
"""
import numpy as np
import pytest

from paper_2506_15969_amd.workload import CONFIGS

pytestmark = pytest.mark.gpu


def _sample(cfg, n, seed):
    rng = np.random.default_rng(seed)
    units = set()
    while len(units) < n:
        units.add((int(rng.integers(cfg.n_layers)), int(rng.integers(cfg.batch)),
                   int(rng.integers(cfg.n_kv_heads))))
    return sorted(units)


def _logger(capsys, name, every):
    def log(msg):
        t = int(msg.split()[0][2:])
        if t % every < 32:
            with capsys.disabled():
                print("\n[%s] %s" % (name, msg[:160]), flush=True)
    return log


def _report(capsys, name, stat):
    with capsys.disabled():
        print("\n[%s] steps=%d calls checked=%d decisions=%d near-threshold disagreements=%d "
              "evictions=%d calls leaving candidate lists=%d max out err=%.3g"
              % (name, stat["steps"], stat["calls_checked"], stat["decisions"], stat["near_threshold"],
                 stat["evictions"], stat["compact_calls"], stat["max_out_err"]), flush=True)


def _first_eviction(cfg):
    return (max(cfg.budget - cfg.prompt_len, 0) // cfg.window + 1) * cfg.window


@pytest.mark.parametrize("name,n_units", [("cfg3", 6), ("cfg5", 4), ("cfg4", 6)])
def test_timed_path_in_steady_state(lazyev_lib, capsys, name, n_units):
    """Benchmark shapes, prompt = budget, the workload's own firing schedule, 2 layers, a bit
    over two windows: the kernel instance bench.py times (deferred tracking, candidate lists)
    against the oracle at every call."""
    from lockstep import run_timed_path
    base = CONFIGS[name]
    steps = 2 * base.window + 2
    cfg = base.scaled(n_layers=2, prompt_len=base.budget, steps=steps)
    stat = run_timed_path(lazyev_lib, cfg, _sample(cfg, n_units, base.seed))
    _report(capsys, name + "/timed-path/steady", stat)
    assert stat["evictions"] == 2 and stat["steps"] == steps
    assert stat["compact_calls"] == stat["calls_checked"]
    assert stat["near_threshold"] <= max(4, stat["decisions"] // 20000)


@pytest.mark.parametrize("name,extra_windows,n_units", [("cfg3", 3, 6), ("cfg4", 3, 6), ("cfg5", 2, 4)])
def test_unmodified_workload_all_layers_through_its_first_evictions(lazyev_lib, capsys, name,
                                                                    extra_windows, n_units):
    """The workload exactly as the benchmark runs it (own prompt, own schedule, all 28 / 36
    layers, lazyev_evict_all over 3584 / 4608 units in one launch pair) from the prompt through
    the growth of the cache and the first evictions; sampled units across the layers."""
    from lockstep import run_timed_path
    cfg = CONFIGS[name]
    steps = _first_eviction(cfg) + extra_windows * cfg.window + 3
    cfg = cfg.scaled(steps=steps)
    stat = run_timed_path(lazyev_lib, cfg, _sample(cfg, n_units, 100 + cfg.seed),
                          log=_logger(capsys, name + "/all-layers", 1024))
    _report(capsys, name + "/timed-path/all-layers", stat)
    assert stat["evictions"] == extra_windows + 1
    assert stat["near_threshold"] <= max(4, stat["decisions"] // 20000)
    assert stat["gpu_stats"]["n_evict_events"] == [extra_windows + 1] * cfg.n_layers


@pytest.mark.parametrize("name,n_units,n_events", [("cfg3", 2, 228), ("cfg4", 3, 122), ("cfg5", 1, 456)])
def test_full_length_on_sampled_units(lazyev_lib, capsys, name, n_units, n_events):
    """All 16384 / 32768 steps of the workload from its own prompt with its own schedule, two
    layers, sampled units: the growth phase, the first eviction from a mixed prompt / generated
    state and every later one; the number of evictions is the closed form of the schedule."""
    from lockstep import run_timed_path
    cfg = CONFIGS[name].scaled(n_layers=2)
    stat = run_timed_path(lazyev_lib, cfg, _sample(cfg, n_units, 200 + cfg.seed), check_rows_every=8,
                          log=_logger(capsys, name + "/full", 4096))
    _report(capsys, name + "/timed-path/full-length", stat)
    assert stat["steps"] == cfg.steps and stat["evictions"] == n_events
    assert stat["gpu_stats"]["n_evict_events"] == [n_events, n_events]
    assert stat["near_threshold"] <= max(4, stat["decisions"] // 20000)
    for u in stat["oracle_units"].values():
        assert len(u) == cfg.budget + cfg.steps % cfg.window
