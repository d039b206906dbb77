"""Offline choice of the observation window W (Sec. 4, "Observation Window"; Sec. 3, Fig. 2(c)):
decode a synthetic workload with a budget that covers the whole generation, so that no token is
evicted, collect the distribution of the Maximum Recurrence Interval over all cached tokens and
report the MRI value that a given share (the paper: 80 %) of the recurring tokens stay below.

Usage: python -m paper_2506_15969_amd.mri_stats [--config cfg2] [--steps N] [--layers 1]
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding
from .workload import CONFIGS, Workload


def collect(cfg, steps=None, n_layers=1, n_bins=binding.MAX_HIST_BINS, gen_block=128):
    """Histogram (list of n_bins ints) of MRI after `steps` full-cache decode steps of the first
    `n_layers` layers of the workload."""
    wl = Workload(cfg)
    steps = cfg.steps if steps is None else steps
    eng = binding.LazyEviction(n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                               cfg.prompt_len + steps, cfg.window, cfg.prompt_len, cfg.alpha,
                               dtype=cfg.torch_dtype)
    for l in range(n_layers):
        if cfg.prompt_len:
            eng.load_prompt(l, *wl.prompt_kv(l, device="cuda"))
    eng.init()
    out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=cfg.torch_dtype, device="cuda")
    for t0 in range(1, steps + 1, gen_block):
        t1 = min(steps + 1, t0 + gen_block)
        inputs = [wl.step_inputs(l, t0, t1, device="cuda") for l in range(n_layers)]
        for t in range(t0, t1):
            for l in range(n_layers):
                q, kn, vn = inputs[l]
                eng.decode_step(l, t, q[t - t0], kn[t - t0], vn[t - t0], out)
    hist = eng.mri_histogram(-1, n_bins)
    eng.close()
    return hist


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", default="cfg2", choices=sorted(CONFIGS))
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--layers", type=int, default=1)
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args()
    cfg = CONFIGS[a.config]
    hist = collect(cfg, a.steps, a.layers)
    total, rec = sum(hist), sum(hist[1:])
    qs = {q: binding.window_from_histogram(hist, q) for q in (0.5, 0.8, 0.9, 0.95)}
    if a.json:
        print(json.dumps(dict(config=a.config, entries=total, recurring=rec, quantiles=qs)))
        return
    print(f"{a.config}: {total} cached entries, {rec} re-activated at least once "
          f"({100.0 * rec / max(total, 1):.1f} %)")
    for q, w in qs.items():
        print(f"  {100 * q:4.0f} % of the recurring tokens have MRI <= {w}")
    print(f"  window by the 80 % rule: W = {qs[0.8]}"
          + ("  (overflow bin: raise n_bins)" if qs[0.8] == len(hist) - 1 else ""))


if __name__ == "__main__":
    main()
