"""Lock-step driver: the HIP library and the CPU oracle consume the same seeded inputs step by
step and are compared after every step.  Helper for the GPU parity tests (not collected)."""
from __future__ import annotations

import numpy as np
import torch

from oracle.lazyev_oracle import OracleUnit
from paper_2506_15969_amd.workload import Workload, WorkloadConfig

TOL = {"fp32": 1e-5, "bf16": 2e-2}


def make_engine(binding, cfg: WorkloadConfig, wl: Workload, layers=None, score_flags=3,
                chunk=None, variant=None, target_blocks=None):
    eng = binding.LazyEviction(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads,
                               cfg.head_dim, cfg.budget, cfg.window, cfg.prompt_len, cfg.alpha,
                               dtype=cfg.torch_dtype, score_flags=score_flags)
    for layer in (range(cfg.n_layers) if layers is None else layers):
        if cfg.prompt_len:
            k, v = wl.prompt_kv(layer, device="cuda")
            eng.load_prompt(layer, k, v)
    eng.init()
    if chunk:
        eng.set_chunk(chunk)
    if variant is not None:
        eng.set_variant(variant)
    if target_blocks:
        eng.set_target_blocks(target_blocks)
    return eng


def run_lockstep(binding, cfg: WorkloadConfig, units, steps=None, mode="e2e", score_flags=3,
                 chunk=None, variant=None, target_blocks=None, gen_block=32,
                 check_rows_every=1, log=None, watch=()):
    """Runs `steps` decode steps (default: all) of the layers that `units` touch, full batch on
    the GPU, the listed (layer, seq, kv_head) units in the oracle.

    mode "e2e":       both compute their own weights; decisions may differ only within tol*alpha
                      of the threshold (counted; the oracle then takes the library's decision).
    mode "oracle_p":  the oracle's weights, rounded to fp32, are thresholded by both.
    mode "synthetic": seeded random weights are thresholded by both.
    mode "gpu_p":     the library's exported weights are thresholded (and ranked) by the oracle.
    watch: token positions whose eviction is recorded in stat["evicted_watch"][unit] as
    (pos, step, TS, MRI at that eviction).
    Returns a dict of counters.  Raises AssertionError on any mismatch.
    """
    wl = Workload(cfg)
    tol = TOL[cfg.dtype]
    G, d, C = cfg.group, cfg.head_dim, cfg.capacity
    steps = cfg.steps if steps is None else steps
    layers = sorted({u[0] for u in units})
    eng = make_engine(binding, cfg, wl, layers, score_flags, chunk, variant, target_blocks)
    dev = eng.device
    orc = {}
    for (l, s, h) in units:
        k, v = wl.prompt_kv(l, seq=[s], kv_head=[h])
        orc[(l, s, h)] = OracleUnit(k[0, 0].double().numpy(), v[0, 0].double().numpy(), G,
                                    cfg.budget, cfg.window, cfg.alpha, score_flags=score_flags)
    out = torch.empty((cfg.batch, cfg.n_q_heads, d), dtype=cfg.torch_dtype, device=dev)
    p_out = torch.zeros((cfg.batch, cfg.n_q_heads, C), dtype=torch.float32, device=dev)
    p_in = torch.zeros((cfg.batch, cfg.n_q_heads, C), dtype=torch.float32, device=dev)
    stat = dict(steps=0, decisions=0, near_threshold=0, evictions=0, max_out_err=0.0,
                max_p_err=0.0, activations=0, rows_moved=0, evicted_watch={u: [] for u in units})
    watch = set(int(x) for x in watch)
    rng = np.random.default_rng(cfg.seed + 12345)
    alpha32 = np.float32(cfg.alpha)

    for t0 in range(1, steps + 1, gen_block):
        t1 = min(steps + 1, t0 + gen_block)
        gpu_in = {l: wl.step_inputs(l, t0, t1, device="cuda") for l in layers}
        cpu_in = {u: wl.step_inputs(u[0], t0, t1, seq=[u[1]], kv_head=[u[2]]) for u in units}
        for t in range(t0, t1):
            i = t - t0
            for l in layers:
                q, kn, vn = (x[i] for x in gpu_in[l])
                mine = [u for u in units if u[0] == l]
                n1 = len(orc[mine[0]]) + 1
                if mode == "gpu_p":
                    # the oracle thresholds (and, where the score is the step's own weight,
                    # ranks by) the library's exported fp32 weights: everything must be exact
                    eng.decode_step(l, t, q, kn, vn, out, p_out=p_out)
                    o_gpu = out.float().cpu().numpy().astype(np.float64)
                    p_gpu = p_out.cpu().numpy()
                    for u in mine:
                        _, s, h = u
                        rows = slice(h * G, (h + 1) * G)
                        pg = np.ascontiguousarray(p_gpu[s, rows, :n1])
                        cq, ck, cv = (x[i, 0] for x in cpu_in[u])
                        o, p, act = orc[u].decode_step(t, cq.double().numpy(), ck[0].double().numpy(),
                                                       cv[0].double().numpy(), p_override=pg)
                        _compare_out(o_gpu[s, rows], o, tol, stat, (u, t))
                        assert np.all(np.abs(pg - p) <= tol * np.maximum(p, 1e-6) + 1e-9), (u, t)
                        stat["decisions"] += n1
                elif mode == "e2e":
                    eng.decode_step(l, t, q, kn, vn, out, p_out=p_out)
                    o_gpu = out.float().cpu().numpy().astype(np.float64)
                    p_gpu = p_out.cpu().numpy()
                    for u in mine:
                        _, s, h = u
                        rows = slice(h * G, (h + 1) * G)
                        pg = p_gpu[s, rows, :n1]
                        act_gpu = (pg >= alpha32).any(axis=0)

                        def adopt(p, act, pg=pg, act_gpu=act_gpu):
                            diff = np.nonzero(act != act_gpu)[0]
                            for j in diff:
                                near = np.abs(p[:, j] - cfg.alpha) <= tol * cfg.alpha
                                assert near.any(), ("decision differs away from the threshold",
                                                    u, t, j, p[:, j], pg[:, j], cfg.alpha)
                            stat["near_threshold"] += len(diff)
                            return act_gpu
                        cq, ck, cv = (x[i, 0] for x in cpu_in[u])
                        o, p, act = orc[u].decode_step(t, cq.double().numpy(),
                                                       ck[0].double().numpy(),
                                                       cv[0].double().numpy(), act_override=adopt)
                        _compare_out(o_gpu[s, rows], o, tol, stat, (u, t))
                        perr = np.abs(pg - p).max() / max(p.max(), 1e-30)
                        stat["max_p_err"] = max(stat["max_p_err"], float(perr))
                        assert np.all(np.abs(pg - p) <= tol * np.maximum(p, 1e-6) + 1e-9), (u, t)
                        stat["decisions"] += n1
                else:
                    if mode == "synthetic":
                        pw = (rng.random((cfg.batch, cfg.n_q_heads, n1), dtype=np.float32) ** 6
                              * np.float32(12.0 * cfg.alpha))
                        # a few values exactly at the threshold: the test is inclusive
                        pw[:, :, rng.integers(0, n1, 3)] = alpha32
                    else:
                        pw = np.zeros((cfg.batch, cfg.n_q_heads, n1), dtype=np.float32)
                    res = {}
                    if mode == "oracle_p":
                        for u in mine:
                            _, s, h = u
                            cq, ck, cv = (x[i, 0] for x in cpu_in[u])
                            # decide in fp32 on the oracle's own rounded weights
                            def from_own(p, act):
                                return (p.astype(np.float32) >= alpha32).any(axis=0)
                            o, p, act = orc[u].decode_step(t, cq.double().numpy(),
                                                           ck[0].double().numpy(),
                                                           cv[0].double().numpy(),
                                                           act_override=from_own)
                            pw[s, h * G:(h + 1) * G] = p.astype(np.float32)
                            res[u] = o
                    p_in[:, :, :n1].copy_(torch.from_numpy(pw))
                    eng.decode_step(l, t, q, kn, vn, out, p_override=p_in)
                    o_gpu = out.float().cpu().numpy().astype(np.float64)
                    for u in mine:
                        _, s, h = u
                        rows = slice(h * G, (h + 1) * G)
                        if mode == "synthetic":
                            cq, ck, cv = (x[i, 0] for x in cpu_in[u])
                            o, p, act = orc[u].decode_step(t, cq.double().numpy(),
                                                           ck[0].double().numpy(),
                                                           cv[0].double().numpy(),
                                                           p_override=pw[s, rows])
                        else:
                            o = res[u]
                        _compare_out(o_gpu[s, rows], o, tol, stat, (u, t))
                        stat["decisions"] += n1
                # recurrence state after the step: exact
                ts_g = eng.ts[l].cpu().numpy()
                mri_g = eng.mri[l].cpu().numpy()
                for u in mine:
                    _, s, h = u
                    assert np.array_equal(ts_g[s, h, :n1], orc[u].TS), ("TS", u, t)
                    assert np.array_equal(mri_g[s, h, :n1], orc[u].MRI), ("MRI", u, t)
                # lagged eviction
                n_ev = eng.evict(l, t)
                before = {u: orc[u].pos.copy() for u in mine}
                held = {u: {int(p): (int(a), int(b)) for p, a, b in zip(orc[u].pos, orc[u].TS, orc[u].MRI)
                            if int(p) in watch} for u in mine} if watch else {}
                gone = {u: orc[u].evict(t) for u in mine}
                for u in (mine if watch else ()):
                    stat["evicted_watch"][u] += [(int(p), t) + held[u][int(p)] for p in gone[u] if int(p) in watch]
                for u in mine:                       # survivors that changed slot (order is kept)
                    stat["rows_moved"] += int((orc[u].pos != before[u][:len(orc[u])]).sum()) if gone[u] else 0
                for u in mine:
                    assert len(gone[u]) == n_ev, ("eviction count", u, t, n_ev, len(gone[u]))
                if n_ev:
                    stat["evictions"] += 1
                    _compare_state(eng, l, mine, orc, t, rows=(stat["evictions"] % check_rows_every == 0))
            stat["steps"] += 1
        if log:
            log("t=%d %s" % (t1 - 1, stat))
    st = eng.stats()
    for l in layers:
        assert st["last_step"][l] == steps and st["len"][l] == len(orc[[u for u in units if u[0] == l][0]])
    # final full comparison, rows included
    for l in layers:
        _compare_state(eng, l, [u for u in units if u[0] == l], orc, steps, rows=True)
    # distribution of MRI over everything cached (all units of all layers on the library's side)
    from oracle.lazyev_oracle import mri_histogram
    stat["gpu_mri_hist"] = eng.mri_histogram(-1, 48)
    stat["gpu_mri_hist_layer"] = {l: eng.mri_histogram(l, 48) for l in layers}
    stat["oracle_mri_hist_layer"] = {
        l: mri_histogram(np.concatenate([orc[u].MRI for u in units if u[0] == l]), 48).tolist()
        for l in layers}
    stat["gpu_stats"] = st
    stat["oracle_units"] = orc
    stat["engine"] = eng
    return stat


def _compare_out(o_gpu, o, tol, stat, where):
    err = np.linalg.norm(o_gpu - o, axis=-1) / np.maximum(np.linalg.norm(o, axis=-1), 1e-30)
    stat["max_out_err"] = max(stat["max_out_err"], float(err.max()))
    assert err.max() <= tol, ("attention output", where, err)


def _compare_state(eng, l, mine, orc, t, rows):
    pos_g = eng.pos[l].cpu().numpy()
    ts_g = eng.ts[l].cpu().numpy()
    mri_g = eng.mri[l].cpu().numpy()
    for u in mine:
        _, s, h = u
        n = len(orc[u])
        assert np.array_equal(pos_g[s, h, :n], orc[u].pos), ("survivor set", u, t)
        assert np.array_equal(ts_g[s, h, :n], orc[u].TS), ("TS after eviction", u, t)
        assert np.array_equal(mri_g[s, h, :n], orc[u].MRI), ("MRI after eviction", u, t)
        if rows:
            kg = eng.k_cache[l, s, h, :n].double().cpu().numpy()
            vg = eng.v_cache[l, s, h, :n].double().cpu().numpy()
            assert np.array_equal(kg, orc[u].K), ("K rows", u, t)
            assert np.array_equal(vg, orc[u].V), ("V rows", u, t)


def run_timed_path(binding, cfg: WorkloadConfig, units, steps=None, gen_block=32,
                   check_rows_every=1, variant=None, log=None):
    """The path the benchmark times, next to the oracle: lazyev_decode_step WITHOUT p_out /
    p_override for every layer of every step (so the tracking of a call is applied by the
    tracking blocks that ride with the next launch, from all logits or, over a long cache, from
    the candidate lists) and lazyev_evict_all after every step at which an eviction is due.

    The oracle follows the listed (layer, seq, kv_head) units on its own fp64 weights.  What the
    library decided at a call is read after the NEXT call has been enqueued: from the activation
    log, in which that launch leaves one bit per entry (lazyev_log_peek looks at it and applies
    nothing), or, for a configuration without a log, from TS (an entry older than the call's
    appended one has TS == t exactly if the call activated it).  Before a due eviction
    lazyev_stats applies everything outstanding, which is what lazyev_evict_all would do first
    anyway.  A differing decision is accepted only within tol * alpha of the threshold (counted,
    adopted); TS / MRI are compared whenever the library has applied its tracking (after every
    call without a log; with one, before every eviction and at the end), survivor sets, TS, MRI,
    pos (and rows) after every eviction, outputs at every call.
    """
    wl = Workload(cfg)
    tol = TOL[cfg.dtype]
    G, d = cfg.group, cfg.head_dim
    L = cfg.n_layers
    steps = cfg.steps if steps is None else steps
    eng = make_engine(binding, cfg, wl, None, 3, None, variant, None)
    dev = eng.device
    by_layer = {l: [u for u in units if u[0] == l] for l in range(L)}
    orc = {}
    for (l, s, h) in units:
        k, v = wl.prompt_kv(l, seq=[s], kv_head=[h])
        orc[(l, s, h)] = OracleUnit(k[0, 0].double().numpy(), v[0, 0].double().numpy(), G,
                                    cfg.budget, cfg.window, cfg.alpha)
    out = torch.empty((2, L, cfg.batch, cfg.n_q_heads, d), dtype=cfg.torch_dtype, device=dev)
    stat = dict(steps=0, calls_checked=0, decisions=0, near_threshold=0, evictions=0,
                max_out_err=0.0, compact_calls=0)
    n_len = cfg.prompt_len                      # entries per unit before the next append

    def resolve(call, applied=False):
        """Oracle step for a finished call whose tracking the library has logged or (applied)
        written to TS / MRI."""
        l, t, n1, cpu_rows = call
        mine = by_layer[l]
        if not mine:
            return
        ss = torch.tensor([u[1] for u in mine], device=dev)
        hh = torch.tensor([u[2] for u in mine], device=dev)
        logged = None if applied else eng.log_peek(l, [(u[1], u[2]) for u in mine])
        if logged is not None:
            assert logged[0] == t, ("the layer's latest logged call", l, t, logged[0])
            stat["logged_calls"] = stat.get("logged_calls", 0) + 1
            act_log = logged[1]
        ts_g = eng.ts[l][ss, hh, :n1].cpu().numpy()
        mri_g = eng.mri[l][ss, hh, :n1].cpu().numpy()
        o_gpu = out[t % 2, l].float().cpu().numpy().astype(np.float64)
        for k_u, u in enumerate(mine):
            _, s, h = u
            rows = slice(h * G, (h + 1) * G)

            def adopt(p, act, k_u=k_u):
                act_gpu = act.copy()                            # (the appended entry's own flag is not visible)
                act_gpu[:n1 - 1] = act_log[k_u, :n1 - 1] if logged is not None else ts_g[k_u, :n1 - 1] == t
                diff = np.nonzero(act != act_gpu)[0]
                for j in diff:
                    near = np.abs(p[:, j] - cfg.alpha) <= tol * cfg.alpha
                    assert near.any(), ("decision differs away from the threshold", u, t, j,
                                        p[:, j], cfg.alpha)
                stat["near_threshold"] += len(diff)
                return act_gpu
            cq, ck, cv = cpu_rows[u]
            o, p, act = orc[u].decode_step(t, cq, ck, cv, act_override=adopt)
            _compare_out(o_gpu[s, rows], o, tol, stat, (u, t))
            if logged is None:                                  # (TS / MRI hold this call's tracking)
                assert np.array_equal(ts_g[k_u], orc[u].TS), ("TS", u, t)
                assert np.array_equal(mri_g[k_u], orc[u].MRI), ("MRI", u, t)
            else:
                assert not act_log[k_u, n1 - 1:].any(), ("bits beyond the call's entries", u, t)
            stat["decisions"] += n1
        stat["calls_checked"] += 1

    pending = None
    for t0 in range(1, steps + 1, gen_block):
        t1 = min(steps + 1, t0 + gen_block)
        gpu_in = [wl.step_inputs(l, t0, t1, device="cuda") for l in range(L)]
        cpu_in = {u: wl.step_inputs(u[0], t0, t1, seq=[u[1]], kv_head=[u[2]]) for u in units}
        cpu_in = {u: tuple(x.double().numpy() for x in v) for u, v in cpu_in.items()}
        for t in range(t0, t1):
            i = t - t0
            n1 = n_len + 1
            for l in range(L):
                q, kn, vn = (x[i] for x in gpu_in[l])
                eng.decode_step(l, t, q, kn, vn, out[t % 2, l])
                if G < 8:                          # (candidate lists whenever nobody reads the logits)
                    stat["compact_calls"] += 1
                if pending is not None:
                    resolve(pending)
                pending = (l, t, n1, {u: (cpu_in[u][0][i, 0], cpu_in[u][1][i, 0, 0], cpu_in[u][2][i, 0, 0])
                                      for u in by_layer[l]})
            n_len = n1
            if t % cfg.window == 0 and n_len > cfg.budget:
                eng.stats()                          # all outstanding tracking, as lazyev_evict_all applies it
                resolve(pending, applied=True)
                pending = None
                n_ev = eng.evict_all(t)
                assert n_ev == n_len - cfg.budget, (t, n_ev)
                for u in units:
                    assert len(orc[u].evict(t)) == n_ev, ("eviction count", u, t)
                stat["evictions"] += 1
                for l in range(L):
                    if by_layer[l]:
                        _compare_state(eng, l, by_layer[l], orc, t,
                                       rows=(stat["evictions"] % check_rows_every == 0))
                n_len = cfg.budget
            stat["steps"] += 1
        if log:
            log("t=%d %s" % (t1 - 1, stat))
    st = eng.stats()
    if pending is not None:
        resolve(pending, applied=True)
    for l in range(L):
        assert st["last_step"][l] == steps and st["len"][l] == n_len
        if by_layer[l]:
            _compare_state(eng, l, by_layer[l], orc, steps, rows=True)
    stat["gpu_stats"] = st
    stat["oracle_units"] = orc
    eng.close()
    return stat
