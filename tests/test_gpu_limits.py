"""The sizes at the edge of what the library takes: an eviction with exactly
LAZYEV_MAX_CANDIDATES candidates (and the error one candidate beyond), and a full-cache decode
over 16.5 k entries with the largest block split, against the oracle through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2506_15969_amd.workload import CONFIGS, Workload

pytestmark = pytest.mark.gpu

MAX_CANDIDATES = 8192


def _report(name, stat):
    print("\n[%s] steps=%d decisions=%d near-threshold disagreements=%d evictions=%d "
          "max out err=%.3g max p err=%.3g" % (name, stat["steps"], stat["decisions"],
                                               stat["near_threshold"], stat["evictions"],
                                               stat["max_out_err"], stat["max_p_err"]), flush=True)


def test_eviction_with_the_largest_candidate_count(lazyev_lib):
    """Prompt 8192 > budget 8000, W = 64: the first eviction (step 64) ranks 8256 - 64 = 8192
    candidates, the most the selection kernel holds, keeps 7936 of them and the last 64."""
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg2"].scaled(batch=1, prompt_len=MAX_CANDIDATES, steps=70, budget=8000, window=64,
                                 interval_lo=10, interval_hi=60)
    units = [(0, 0, 1), (0, 0, 3)]
    stat = run_lockstep(lazyev_lib, cfg, units, mode="e2e")
    _report("max-candidates", stat)
    assert stat["evictions"] == 1 and stat["near_threshold"] <= 2
    for u in stat["oracle_units"].values():
        assert len(u) == 8000 + 6


def test_one_candidate_too_many_is_refused(lazyev_lib):
    cfg = CONFIGS["cfg2"].scaled(batch=1, prompt_len=MAX_CANDIDATES + 1, steps=64, budget=8000, window=64)
    wl = Workload(cfg)
    from lockstep import make_engine
    eng = make_engine(lazyev_lib, cfg, wl)
    q, kn, vn = wl.step_inputs(0, 1, 65, device="cuda")
    out = torch.empty((1, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
    for t in range(1, 65):
        eng.decode_step(0, t, q[t - 1], kn[t - 1], vn[t - 1], out)
        if t < 64:
            assert eng.evict(0, t) == 0
    with pytest.raises(lazyev_lib.LazyevError) as e:
        eng.evict(0, 64)
    assert e.value.code == lazyev_lib.ECAPACITY
    st = eng.stats()                                      # the context is still usable
    assert st["len"] == [MAX_CANDIDATES + 1 + 64] and st["n_evict_events"] == [0]


def test_full_cache_of_16k_entries_with_the_largest_split(lazyev_lib):
    """No eviction (the budget covers prompt and generation): 16500..16520 entries per unit, 64
    blocks per unit (the most the single-launch kernel uses), every unit followed by the oracle."""
    from lockstep import run_lockstep
    cfg = CONFIGS["cfg2"].scaled(batch=1, prompt_len=16500, steps=20, budget=17000, window=64,
                                 interval_lo=5, interval_hi=15)
    units = [(0, 0, h) for h in range(cfg.n_kv_heads)]
    stat = run_lockstep(lazyev_lib, cfg, units, mode="e2e", variant=4, target_blocks=100000)
    _report("16k-entries/64-blocks", stat)
    assert stat["evictions"] == 0 and stat["near_threshold"] <= 2
    stat = run_lockstep(lazyev_lib, cfg, units, mode="oracle_p", variant=4, target_blocks=1)
    assert stat["near_threshold"] == 0                    # one block per unit: 258 sub-tiles per wave
