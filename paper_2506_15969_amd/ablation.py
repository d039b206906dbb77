"""Score-variant comparison on a synthetic workload (Table 4's ablation, and the two readings
of the H2 term of Sec. 4), run through the HIP library.

For every variant the same seeded inputs are decoded twice, once with a budget that covers the
whole generation (full cache) and once with eviction, and three things are reported:

  out_err   mean over steps, sequences and query heads of ||A_t - A'_t||_2 / ||A_t||_2, the
            quantity the eviction problem of App. A (Eq. 5) minimises, A_t from the full cache;
  err@fire  the same error over the (step, query head) pairs at which a planted key fires, i.e.
            where one cached entry carries nearly all of the attention;
  recall    fraction of the planted keys' firing events (a query that re-attends key j at step
            t) that still find their key in the cache, per (sequence, KV head);
  survive   fraction of the planted keys older than the last window that are cached at the end.

Usage: python -m paper_2506_15969_amd.ablation [--config cfg2] [--steps N] [--layer 0]
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding
from .workload import CONFIGS, Workload

VARIANTS = [
    ("H1+H2 (as printed)", binding.SCORE_H1 | binding.SCORE_H2),
    ("H1+H2 (H2 reflected)", binding.SCORE_H1 | binding.SCORE_H2 | binding.SCORE_H2_DECREASING),
    ("w/o H2", binding.SCORE_H1),
    ("w/o H1", binding.SCORE_H2),
    ("w/o H1 (H2 reflected)", binding.SCORE_H2 | binding.SCORE_H2_DECREASING),
    ("neither (sliding window)", 0),
    # the rule of the current-attention baselines (Sec. 2 (2); App. C): rank by the weights of the
    # eviction's own step; per step (window 1: greedy) and behind the workload's window
    ("current attention, every step", binding.SCORE_CURRENT_ATTENTION, 1),
    ("current attention, every W steps", binding.SCORE_CURRENT_ATTENTION),
]


def _engine(cfg, wl, layer, budget, flags, window=None):
    eng = binding.LazyEviction(1, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, budget,
                               window or cfg.window, cfg.prompt_len, cfg.alpha, dtype=cfg.torch_dtype,
                               score_flags=flags)
    if cfg.prompt_len:
        k, v = wl.prompt_kv(layer, device="cuda")
        eng.load_prompt(0, k, v)
    return eng.init()


def run(cfg, layer=0, steps=None, gen_block=128, variants=VARIANTS):
    wl = Workload(cfg)
    steps = cfg.steps if steps is None else steps
    S, Hq, Hkv, d, P, W = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.prompt_len, cfg.window
    dev = torch.device("cuda:0")
    # full-cache outputs of every step, kept on the device
    full = _engine(cfg, wl, layer, P + steps, binding.SCORE_H1 | binding.SCORE_H2)
    ref = torch.empty((steps, S, Hq, d), dtype=cfg.torch_dtype, device=dev)
    for t0 in range(1, steps + 1, gen_block):
        t1 = min(steps + 1, t0 + gen_block)
        q, kn, vn = wl.step_inputs(layer, t0, t1, device="cuda")
        for t in range(t0, t1):
            full.decode_step(0, t, q[t - t0], kn[t - t0], vn[t - t0], ref[t - 1])
    full.stats()
    full.close()
    ref_norm = ref.float().norm(dim=-1).clamp_min(1e-30)

    rows = []
    for name, flags, *rest in variants:
        W = rest[0] if rest else cfg.window
        if (flags & binding.SCORE_CURRENT_ATTENTION) and (cfg.dtype != "bf16" or d != 128):
            continue                                 # that ranking exists for the bf16 shape only
        eng = _engine(cfg, wl, layer, cfg.budget, flags, W)
        out = torch.empty((S, Hq, d), dtype=cfg.torch_dtype, device=dev)
        err_sum = torch.zeros((), dtype=torch.float64, device=dev)
        present = torch.ones((S, Hkv, P + steps), dtype=torch.bool, device=dev)
        hits = torch.zeros((), dtype=torch.int64, device=dev)
        fire_err = torch.zeros((), dtype=torch.float64, device=dev)
        kv_heads = torch.arange(Hkv, device=dev) * cfg.group
        n_events = 0
        for t0 in range(1, steps + 1, gen_block):
            t1 = min(steps + 1, t0 + gen_block)
            q, kn, vn = wl.step_inputs(layer, t0, t1, device="cuda")
            for t in range(t0, t1):
                ev_t, ev_j = wl.firings(t, t + 1)
                if len(ev_j):
                    hits += present[:, :, torch.as_tensor(ev_j, device=dev)].sum()
                    n_events += len(ev_j) * S * Hkv
                eng.decode_step(0, t, q[t - t0], kn[t - t0], vn[t - t0], out)
                rel = ((out.float() - ref[t - 1].float()).norm(dim=-1) / ref_norm[t - 1]).double()
                err_sum += rel.sum()
                for j in ev_j:                       # key j fires in query head j mod G of every group
                    fire_err += rel[:, kv_heads + int(j) % cfg.group].sum()
                if t % W == 0 and eng.evict(0, t) > 0:
                    n = eng.stats()["len"][0]
                    present[:, :, :P + t] = False
                    present.scatter_(2, eng.pos[0, :, :, :n].long(), True)
        st = eng.stats()
        old = wl.planted[wl.planted < P + steps - cfg.window]
        survive = (float(present[:, :, torch.as_tensor(old, device=dev)].float().mean())
                   if len(old) else float("nan"))
        rows.append(dict(variant=name, score_flags=flags,
                         out_err=float(err_sum) / (steps * S * Hq),
                         err_at_fire=float(fire_err) / max(n_events, 1),
                         recall=int(hits) / max(n_events, 1), survive=survive,
                         evictions=st["n_evict_events"][0], activations=st["n_activations"][0]))
        eng.close()
    return rows


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", default="cfg2", choices=sorted(CONFIGS))
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args()
    cfg = CONFIGS[a.config]
    rows = run(cfg, a.layer, a.steps)
    if a.json:
        print(json.dumps(dict(config=a.config, steps=a.steps or cfg.steps, rows=rows)))
        return
    print(f"{a.config}: layer {a.layer}, {a.steps or cfg.steps} steps, budget {cfg.budget}, window {cfg.window}")
    print(f"{'variant':34s} {'out_err':>9s} {'err@fire':>9s} {'recall':>8s} {'survive':>8s} {'evictions':>9s}")
    for r in rows:
        print(f"{r['variant']:34s} {r['out_err']:9.5f} {r['err_at_fire']:9.5f} {r['recall']:8.4f} {r['survive']:8.4f} {r['evictions']:9d}")


if __name__ == "__main__":
    main()
