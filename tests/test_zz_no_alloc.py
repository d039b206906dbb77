"""lazyev_evict_static (the eviction with its gather list in the library's own static device
array: the entry point for callers that must not allocate) against lazyev_evict on the same
inputs: caches, TS / MRI / pos, counts and counters bit for bit, on calls in a row with shrinking
inputs (the array keeps the previous call's list), and the refusal of shapes beyond the array."""
import pytest
import torch

from paper_2506_15969_amd.workload import CONFIGS, Workload

pytestmark = pytest.mark.gpu


def _drive(binding, cfg, static):
    from lockstep import make_engine
    wl = Workload(cfg)
    eng = make_engine(binding, cfg, wl)
    out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
    ins = [wl.step_inputs(l, 1, cfg.steps + 1, device="cuda") for l in range(cfg.n_layers)]
    removed = []
    for t in range(1, cfg.steps + 1):
        for l in range(cfg.n_layers):
            q, kn, vn = ins[l]
            eng.decode_step(l, t, q[t - 1], kn[t - 1], vn[t - 1], out)
        for l in range(cfg.n_layers):
            removed.append(eng.evict_static(l, t) if static else eng.evict(l, t))
    st = eng.stats()
    n = st["len"][0]
    state = (eng.k_cache[:, :, :, :n].clone(), eng.v_cache[:, :, :, :n].clone(), eng.ts[:, :, :, :n].clone(),
             eng.mri[:, :, :, :n].clone(), eng.pos[:, :, :, :n].clone())
    eng.close()
    return removed, st, state


def test_static_scratch_eviction_equals_the_workspace_one(lazyev_lib):
    # first a prompt beyond the budget (the first eviction removes 162 entries of 332 per unit,
    # the later ones 32 of 202: the list shrinks from call to call), two layers, 16 units each;
    # then a smaller batch with a smaller budget straight after it
    big = CONFIGS["cfg2"].scaled(n_layers=2, batch=4, prompt_len=300, steps=100, budget=170, window=32,
                                 interval_lo=10, interval_hi=60)
    small = CONFIGS["cfg2"].scaled(n_layers=1, batch=1, prompt_len=20, steps=70, budget=48, window=8,
                                   interval_lo=5, interval_hi=30)
    fp32 = CONFIGS["cfg1"].scaled(steps=130)
    for cfg in (big, small, fp32):
        want = _drive(lazyev_lib, cfg, static=False)
        got = _drive(lazyev_lib, cfg, static=True)
        assert got[0] == want[0] and sum(1 for x in want[0] if x) >= 3, cfg.name
        assert got[1] == want[1] and sum(want[1]["n_rows_moved"]) > 0
        for a, b in zip(got[2], want[2]):
            assert torch.equal(a, b)


def test_static_scratch_limit(lazyev_lib):
    b = lazyev_lib
    # 512 units x 2112 entries = 1 081 344 gather-list entries > 1 048 576
    eng = b.LazyEviction(1, 64, 56, 8, 128, 2048, 64, 2048, 0.004).init()
    q = torch.zeros((64, 56, 128), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((64, 8, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    for t in range(1, 65):
        eng.decode_step(0, t, q, kv, kv, out)
    with pytest.raises(b.LazyevError) as err:
        eng.evict_static(0, 64)
    assert err.value.code == b.ESCRATCH
    assert eng.stats()["len"] == [2112]                   # nothing ran
    assert eng.evict(0, 64) == 64 and eng.stats()["len"] == [2048]
    eng.close()
    # more candidates per unit than the selection keeps in LDS
    eng = b.LazyEviction(1, 1, 7, 1, 128, 9000, 8, 16, 0.004).init()
    with pytest.raises(b.LazyevError) as err:
        eng.evict_static(0, 0)
    assert err.value.code == b.ESCRATCH
    eng.close()
