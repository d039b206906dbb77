"""Per-sequence timing (lazyev_admit / lazyev_retire): sequences with different prompt lengths,
one that starts late, one slot that is empty at first, a sequence that is retired and its slot
taken again.  Every sequence that takes a step is followed by oracle units on its own clock; the
oracle thresholds the library's exported fp32 weights, so recurrence state, eviction schedule,
survivor sets and moved rows must agree exactly.  Inputs are seeded random tensors (no
structure is needed here)."""
import numpy as np
import pytest
import torch

from oracle.lazyev_oracle import OracleUnit, mri_histogram

pytestmark = pytest.mark.gpu

L, S, HQ, HKV, D = 2, 4, 8, 2, 128
G = HQ // HKV
B, W, PMAX = 96, 16, 160
ALPHA = float(np.float32(8.0 / (B + W)))
STEPS = 140
# (global step before which the event happens, kind, slot, prompt_len, t0)
EVENTS = [(1, "admit", 0, 160, 0), (1, "admit", 1, 37, 0), (1, "admit", 2, 0, 5),
          (1, "retire", 3, None, None), (41, "admit", 3, 100, 40), (61, "retire", 1, None, None),
          (71, "admit", 1, 50, 70), (120, "admit", 2, 96, 119)]


def _rand(gen, *shape):
    return torch.randn(shape, generator=gen).to(torch.bfloat16)


def _drive(binding, with_weights, follow, variant=None, evict_together=False):
    """Runs the scenario.  follow: compare with oracle units step by step (needs with_weights)."""
    gen = torch.Generator().manual_seed(77)
    eng = binding.LazyEviction(L, S, HQ, HKV, D, B, W, PMAX, ALPHA, dtype=torch.bfloat16)
    eng.init()
    if variant is not None:
        eng.set_variant(variant)
    cap = eng.capacity
    out = torch.empty((S, HQ, D), dtype=torch.bfloat16, device="cuda")
    p_out = torch.zeros((S, HQ, cap), dtype=torch.float32, device="cuda")
    orc, slot = {}, {s: None for s in range(S)}            # slot -> (prompt_len, t0) or None
    outs = []
    removed = [0] * L                                      # per layer: sum over the events of the largest cut
    for t in range(1, STEPS + 1):
        for (when, kind, s, P, t0) in EVENTS:
            if when != t:
                continue
            if kind == "retire":
                eng.retire(s)
                slot[s] = None
                for key in [k for k in orc if k[1] == s]:
                    del orc[key]
                continue
            k, v = _rand(gen, L, HKV, P, D), _rand(gen, L, HKV, P, D)
            eng.admit(s, P, t0, k.cuda(), v.cuda())
            slot[s] = (P, t0)
            for l in range(L):
                for h in range(HKV):
                    orc[(l, s, h)] = OracleUnit(k[l, h].double().numpy(), v[l, h].double().numpy(),
                                                G, B, W, ALPHA)
        active = [s for s in range(S) if slot[s] is not None and t - slot[s][1] >= 1]
        for l in range(L):
            q, kn, vn = _rand(gen, S, HQ, D), _rand(gen, S, HKV, D), _rand(gen, S, HKV, D)
            out.fill_(-7.0)
            eng.decode_step(l, t, q.cuda(), kn.cuda(), vn.cuda(), out, p_out=p_out if with_weights else None)
            outs.append(out.clone())
            o_gpu = out.float().cpu().numpy()
            for s in range(S):
                if s not in active:
                    assert np.all(o_gpu[s] == -7.0), ("row of an idle slot was written", t, l, s)
            if follow:
                p_gpu = p_out.cpu().numpy()
                for s in active:
                    tau = t - slot[s][1]
                    for h in range(HKV):
                        u = orc[(l, s, h)]
                        n1 = len(u) + 1
                        rows = slice(h * G, (h + 1) * G)
                        pg = np.ascontiguousarray(p_gpu[s, rows, :n1])
                        o, p, _ = u.decode_step(tau, q[s, rows].double().numpy(), kn[s, h].double().numpy(),
                                                vn[s, h].double().numpy(), p_override=pg)
                        err = np.linalg.norm(o_gpu[s, rows] - o, axis=-1) / np.linalg.norm(o, axis=-1)
                        assert err.max() <= 2e-2, ("output", t, l, s, h, err)
                        assert np.all(np.abs(pg - p) <= 2e-2 * np.maximum(p, 1e-6) + 1e-9)
                ts_g, mri_g = eng.ts[l].cpu().numpy(), eng.mri[l].cpu().numpy()
                for s in active:
                    for h in range(HKV):
                        u = orc[(l, s, h)]
                        assert np.array_equal(ts_g[s, h, :len(u)], u.TS), ("TS", t, l, s, h)
                        assert np.array_equal(mri_g[s, h, :len(u)], u.MRI), ("MRI", t, l, s, h)
            if evict_together:                               # after the last layer, all layers in one call
                if l == L - 1:
                    eng.evict_all(t)
                continue
            n_ev = eng.evict(l, t)
            if follow:
                gone = {(s, h): orc[(l, s, h)].evict(t - slot[s][1]) for s in active for h in range(HKV)}
                assert n_ev == max([len(g) for g in gone.values()] + [0]), ("evicted", t, l, n_ev)
                removed[l] += n_ev
                if n_ev:
                    eng.stats()
                    pos_g, ts_g, mri_g = (x[l].cpu().numpy() for x in (eng.pos, eng.ts, eng.mri))
                    for (s, h), g in gone.items():
                        u = orc[(l, s, h)]
                        n = len(u)
                        assert np.array_equal(pos_g[s, h, :n], u.pos), ("survivors", t, l, s, h)
                        assert np.array_equal(ts_g[s, h, :n], u.TS) and np.array_equal(mri_g[s, h, :n], u.MRI)
                        if g:
                            assert np.array_equal(eng.k_cache[l, s, h, :n].double().cpu().numpy(), u.K)
                            assert np.array_equal(eng.v_cache[l, s, h, :n].double().cpu().numpy(), u.V)
    st = eng.stats()
    if follow:
        # with per-sequence timing n_evicted counts, per event, the largest cut among the due units
        assert st["n_evicted"] == removed
    state = (torch.stack(outs), eng.k_cache.clone(), eng.v_cache.clone(), eng.ts.clone(),
             eng.mri.clone(), eng.pos.clone())
    return eng, orc, slot, st, state


def test_sequences_on_their_own_clocks(lazyev_lib):
    eng, orc, slot, st, state = _drive(lazyev_lib, with_weights=True, follow=True)
    lens = {l: max(len(u) for (l2, s, h), u in orc.items() if l2 == l) for l in range(L)}
    assert st["len"] == [lens[0], lens[1]] and st["last_step"] == [STEPS, STEPS]
    # the schedule ran on local clocks: slot 0 (prompt 160 > budget) evicts from local step 16 on,
    # slot 2's second occupant (prompt = budget) from its local step 16 = global step 135
    assert orc[(0, 0, 0)].n_evict_events == STEPS // W
    assert orc[(0, 2, 0)].n_evict_events == 1 and len(orc[(0, 2, 0)]) == B + (STEPS - 119 - 16)
    for l in range(L):
        want = mri_histogram(np.concatenate([u.MRI for (l2, s, h), u in orc.items() if l2 == l]), 40)
        assert eng.mri_histogram(l, 40) == want.tolist()
    # the same scenario without asking for weights (tracking rides with the next launch), with
    # every logit kept for it and with candidate lists, and with the evictions of a step asked for
    # in one call for all layers
    for variant, together in ((5, False), (6, False), (6, True)):
        _, _, _, st2, state2 = _drive(lazyev_lib, with_weights=False, follow=False, variant=variant,
                                      evict_together=together)
        assert st2 == st
        for x, y in zip(state, state2):
            assert torch.equal(x, y)


def test_slot_calls_reject_what_they_cannot_do(lazyev_lib):
    b = lazyev_lib
    eng = b.LazyEviction(1, 2, HQ, HKV, D, B, W, PMAX, ALPHA, dtype=torch.bfloat16).init()
    for bad in ((2, 10, 0), (-1, 10, 0), (0, PMAX + 1, 0), (0, -2, 0)):
        with pytest.raises(b.LazyevError):
            eng.admit(*bad)
    with pytest.raises(b.LazyevError):
        eng.retire(5)
    q = torch.zeros((2, HQ, D), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((2, HKV, D), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    eng.decode_step(0, 1, q, kv, kv, out)
    with pytest.raises(b.LazyevError):                    # its first step would lie in the past
        eng.admit(0, 10, 0)
    eng.admit(0, 10, 1)
    eng.set_variant(0)                                    # the other kernel knows no slots
    with pytest.raises(b.LazyevError):
        eng.decode_step(0, 2, q, kv, kv, out)
    fp32 = b.LazyEviction(1, 2, 4, 4, 64, 32, 4, 8, 0.1, dtype=torch.float32).init()
    with pytest.raises(b.LazyevError):
        fp32.admit(0, 4, 0)


def test_admitted_batch_on_one_clock_equals_the_uniform_batch(lazyev_lib):
    """Ten sequences admitted with the same prompt length and start step behave as the uniform
    batch: all ten are due at the same steps (more than an eviction launch lists one by one, so it
    covers every unit), outputs and state bit for bit; then with two start steps (five sequences
    due at a time: the launch covers only those) against each sequence's own uniform run."""
    from lockstep import make_engine
    from paper_2506_15969_amd.workload import CONFIGS, Workload
    cfg = CONFIGS["cfg2"].scaled(batch=10, prompt_len=100, steps=75, budget=120, window=16)
    wl = Workload(cfg)
    S, steps = cfg.batch, cfg.steps
    ins = wl.step_inputs(0, 1, steps + 1, device="cuda")

    def run(offsets):
        """offsets[s]: the global step before sequence s's first one (None: no admit calls)."""
        eng = make_engine(lazyev_lib, cfg, wl, target_blocks=2 * S * cfg.n_kv_heads)   # two blocks per unit throughout
        if offsets is not None:
            for s in range(S):
                eng.admit(s, cfg.prompt_len, offsets[s])
        out = torch.empty((S, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
        outs = []
        q, kn, vn = ins
        last = steps + (max(offsets) if offsets else 0)
        for t in range(1, last + 1):
            # sequence s is fed the inputs of ITS local step
            loc = [min(max(t - (offsets[s] if offsets else 0), 1), steps) for s in range(S)]
            idx = torch.tensor(loc, device="cuda") - 1
            ar = torch.arange(S, device="cuda")
            eng.decode_step(0, t, q[idx, ar].contiguous(), kn[idx, ar].contiguous(), vn[idx, ar].contiguous(), out)
            outs.append(out.clone())
            eng.evict_all(t)
        eng.stats()
        state = (eng.k_cache.clone(), eng.v_cache.clone(), eng.ts.clone(), eng.mri.clone(), eng.pos.clone())
        eng.close()
        return outs, state

    base_outs, base_state = run(None)
    same_outs, same_state = run([0] * S)
    n = cfg.budget + (steps % cfg.window)
    for a, b in zip(base_outs, same_outs):
        assert torch.equal(a, b)
    for a, b in zip(base_state, same_state):
        assert torch.equal(a[:, :, :, :n], b[:, :, :, :n])
    offs = [0 if s % 2 == 0 else 5 for s in range(S)]
    two_outs, two_state = run(offs)
    for s in range(S):
        for tau in range(1, steps + 1):                        # local step tau of sequence s
            assert torch.equal(two_outs[tau + offs[s] - 1][s], base_outs[tau - 1][s]), (s, tau)
