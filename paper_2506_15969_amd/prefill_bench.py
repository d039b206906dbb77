"""Times lazyev_prefill_track (the tracking loop of Alg. 1 and Eq. 1 run over the prompt's own
causal attention) on a synthetic prompt of one of the benchmark workloads and prints one JSON
line: milliseconds per layer, prompt tokens per second, and the rate of the two causal Q K^T
passes against the dense bf16 MFMA peak.

Usage: python -m paper_2506_15969_amd.prefill_bench [--config cfg3] [--prompt-len 2048] [--reps 5]
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding
from .workload import CONFIGS, Workload

MFMA_BF16_PEAK_TFLOPS = 2500.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--prompt-len", type=int, default=2048)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    P = args.prompt_len
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
    for _ in range(args.reps):
        eng.prefill_track(0, q)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.reps
    units = cfg.batch * cfg.n_kv_heads
    # 2 flops per multiply-add, causal triangle incl. the diagonal, G heads, two passes
    flops = 2.0 * 2.0 * units * cfg.group * (P * (P + 1) / 2.0) * cfg.head_dim
    st = eng.stats()
    print(json.dumps({
        "metric": "prompt_tracking_ms_per_layer", "value": ms, "unit": "ms", "higher_is_better": False,
        "config": {"workload": "%s-prompt%d" % (cfg.name, P), "batch": cfg.batch, "prompt_len": P,
                   "n_q_heads": cfg.n_q_heads, "n_kv_heads": cfg.n_kv_heads, "alpha": cfg.alpha},
        "prompt_tokens_per_s": cfg.batch * P / (ms * 1e-3), "dtype": "bf16", "data": "synthetic",
        "activations_per_call": st["n_activations"][0] // (args.reps + 1),
        "roofline": {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "flops_per_call": flops}}))
    eng.close()


if __name__ == "__main__":
    main()
