"""Seeded synthetic decode workloads (inputs only; none of the method's arithmetic lives here).

The paper evaluates on reasoning benchmarks with trained models (Sec. 5, Appendix C); neither
is available to this repository, so these generators stand in for them.  They take from the
paper only the shapes (7B/14B-class GQA, 4k-32k generated tokens) and the qualitative attention
structure it reports in Sec. 3: most tokens are re-attended after a gap (Token Importance
Recurrence), a few initial tokens are attended all the time.

Everything is a pure function of (seed, stream, layer, index, sequence, head, lane), so any
slice of the inputs -- one unit on the CPU, a whole batch on the GPU -- can be produced on its
own and is bit-identical wherever it is produced:

  * a 64-bit integer mix of the counter gives two words = eight 16-bit fields; their centred
    sum is an integer in [-262140, 262140] with a near-normal (Irwin-Hall, n = 8) law;
  * planted recurring keys: when key j "fires" at step t, query head (j mod G) of every group
    gets q += 4*K_j (integer arithmetic, so accumulation order cannot matter);
  * attention-sink keys (positions 0..n_sink-1): every query gets + (gain/32) * sum K_sink;
  * one int -> float32 conversion, one float32 multiply by the unit-variance scale, then a
    round-to-nearest-even cast if the workload dtype is bf16.

Only integer tensor ops and those two float ops are used, all of which are exact or correctly
rounded on both the CPU and the GPU back ends of torch.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MIX1 = 0xBF58476D1CE4E5B9
_MIX2 = 0x94D049BB133111EB
_SECOND = 0xD6E8FEB86659FD93

STREAM_K, STREAM_V, STREAM_Q, STREAM_QP = 1, 2, 3, 4

# float32 factor that turns the centred eight-field sum into a unit-variance value
_UNIT_SCALE = float(np.float32(1.0 / math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0)))


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 stores for it."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(z: torch.Tensor, n: int) -> torch.Tensor:
    """Logical right shift of int64 bit patterns."""
    return (z >> n) & ((1 << (64 - n)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_MIX1)
    z = (z ^ _lsr(z, 27)) * _s64(_MIX2)
    return z ^ _lsr(z, 31)


def _mix_py(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _MIX1) & _M64
    z = ((z ^ (z >> 27)) * _MIX2) & _M64
    return z ^ (z >> 31)


def _field_sum(z: torch.Tensor) -> torch.Tensor:
    return (z & 0xFFFF) + (_lsr(z, 16) & 0xFFFF) + (_lsr(z, 32) & 0xFFFF) + _lsr(z, 48)


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                      # "fp32" | "bf16"
    prompt_len: int
    steps: int
    budget: int
    window: int
    seed: int
    planted_frac: float = 0.0       # fraction of token positions that are recurring keys
    planted_count_in_prompt: int = 0   # >0: exactly this many planted keys, all in the prompt
    schedule: str = "uniform"       # "uniform" | "loguniform" | "bursty"
    interval_lo: int = 32
    interval_hi: int = 512
    n_sink: int = 0
    alpha_numer: float = 8.0        # alpha = alpha_numer / (budget + window)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def alpha(self) -> float:
        return float(np.float32(self.alpha_numer / (self.budget + self.window)))

    @property
    def capacity(self) -> int:
        return max(self.prompt_len, self.budget) + self.window

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def scaled(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


# The five benchmark workloads, "cfg1".."cfg5": shapes of 7B- and 14B-class GQA models, 512 to 32768 generated tokens.
CONFIGS = {
    "cfg1": WorkloadConfig("cfg1", 1, 1, 4, 4, 64, "fp32", 64, 512, 128, 16, seed=1,
                           planted_count_in_prompt=8, schedule="uniform",
                           interval_lo=40, interval_hi=90),
    "cfg2": WorkloadConfig("cfg2", 1, 8, 28, 4, 128, "bf16", 512, 4096, 1024, 32, seed=2,
                           planted_frac=0.05, schedule="uniform", interval_lo=32, interval_hi=512),
    "cfg3": WorkloadConfig("cfg3", 28, 32, 28, 4, 128, "bf16", 256, 16384, 2048, 64, seed=3,
                           planted_frac=0.10, schedule="loguniform", interval_lo=16,
                           interval_hi=4096, n_sink=4),
    "cfg4": WorkloadConfig("cfg4", 28, 32, 28, 4, 128, "bf16", 256, 16384, 1024, 128, seed=4,
                           planted_frac=0.20, schedule="bursty", interval_lo=1000,
                           interval_hi=8000),
    "cfg5": WorkloadConfig("cfg5", 36, 16, 40, 8, 128, "bf16", 512, 32768, 4096, 64, seed=5,
                           planted_frac=0.15, schedule="loguniform", interval_lo=16,
                           interval_hi=16384),
}


class Workload:
    """Stateless generator of prompt K/V and per-step (q, k_new, v_new) for one config."""

    def __init__(self, cfg: WorkloadConfig):
        self.cfg = cfg
        self._base = {s: _mix_py(cfg.seed * _GOLDEN + s * _SECOND) for s in (1, 2, 3, 4)}
        self._events_t, self._events_j = self._firing_schedule()

    # ---- planted recurring keys: host-side schedule (plain numpy, seeded) ---------------
    def _firing_schedule(self):
        c = self.cfg
        rng = np.random.default_rng(1000003 * c.seed + 17)
        n_pos = c.prompt_len + c.steps
        if c.planted_count_in_prompt > 0:
            planted = np.sort(rng.choice(c.prompt_len, size=c.planted_count_in_prompt,
                                         replace=False))
        else:
            planted = np.nonzero(rng.random(n_pos) < c.planted_frac)[0]
            planted = planted[planted >= c.n_sink]
        self.planted = planted.astype(np.int64)
        self.period = np.zeros(len(planted), dtype=np.int64)
        ev_t, ev_j = [], []
        for idx, j in enumerate(planted):
            born = max(0, int(j) - c.prompt_len + 1)        # decode step that appends j (0: prompt)
            if c.schedule == "bursty":
                t = born + int(rng.integers(1, c.window + 1))
                while t <= c.steps:
                    for _ in range(int(rng.integers(3, 6))):
                        if t <= c.steps:
                            ev_t.append(t)
                            ev_j.append(int(j))
                        t += int(rng.integers(1, 9))
                    t += int(rng.integers(c.interval_lo, c.interval_hi + 1))
                continue
            if c.schedule == "loguniform":
                tau = int(round(math.exp(rng.uniform(math.log(c.interval_lo),
                                                     math.log(c.interval_hi)))))
            else:
                tau = int(rng.integers(c.interval_lo, c.interval_hi + 1))
            self.period[idx] = tau
            first = born + int(rng.integers(1, min(tau, 64) + 1))
            ts = np.arange(first, c.steps + 1, tau, dtype=np.int64)
            ev_t.extend(ts.tolist())
            ev_j.extend([int(j)] * len(ts))
        ev_t = np.asarray(ev_t, dtype=np.int64)
        ev_j = np.asarray(ev_j, dtype=np.int64)
        order = np.lexsort((ev_j, ev_t))
        return ev_t[order], ev_j[order]

    def firings(self, t0: int, t1: int):
        """(t, j) arrays of the firing events with t0 <= t < t1."""
        lo, hi = np.searchsorted(self._events_t, [t0, t1])
        return self._events_t[lo:hi], self._events_j[lo:hi]

    # ---- integer noise -----------------------------------------------------------------
    def _noise(self, stream: int, layer: int, idx, seq, head, n_heads_total: int, device):
        """Centred field sums, int64 [len(idx), len(seq), len(head), d]."""
        c = self.cfg
        dev = torch.device(device)
        idx = torch.as_tensor(idx, dtype=torch.int64, device=dev).view(-1, 1, 1, 1)
        seq = torch.as_tensor(seq, dtype=torch.int64, device=dev).view(1, -1, 1, 1)
        head = torch.as_tensor(head, dtype=torch.int64, device=dev).view(1, 1, -1, 1)
        lane = torch.arange(c.head_dim, dtype=torch.int64, device=dev).view(1, 1, 1, -1)
        e = ((idx * c.batch + seq) * n_heads_total + head) * c.head_dim + lane
        key = _s64(_mix_py(self._base[stream] + layer * _GOLDEN))
        z1 = _mix(e * _s64(_GOLDEN) + key)
        z2 = _mix(z1 ^ _s64(_SECOND))
        return _field_sum(z1) + _field_sum(z2) - 262140

    def _finish(self, ints: torch.Tensor) -> torch.Tensor:
        x = ints.to(torch.float32) * _UNIT_SCALE
        return x if self.cfg.dtype == "fp32" else x.to(torch.bfloat16)

    # ---- K/V rows by token position ------------------------------------------------------
    def _k_int(self, layer, positions, seq, kv_head, device):
        return self._noise(STREAM_K, layer, positions, seq, kv_head, self.cfg.n_kv_heads, device)

    def kv_rows(self, layer: int, positions, device="cpu", seq=None, kv_head=None):
        """K, V rows of the tokens at `positions`: [len(seq), len(kv_head), len(positions), d]."""
        c = self.cfg
        seq = range(c.batch) if seq is None else seq
        kv_head = range(c.n_kv_heads) if kv_head is None else kv_head
        k = self._k_int(layer, positions, list(seq), list(kv_head), device)
        v = self._noise(STREAM_V, layer, positions, list(seq), list(kv_head), c.n_kv_heads, device)
        return (self._finish(k).permute(1, 2, 0, 3).contiguous(),
                self._finish(v).permute(1, 2, 0, 3).contiguous())

    def prompt_kv(self, layer: int, device="cpu", seq=None, kv_head=None):
        return self.kv_rows(layer, range(self.cfg.prompt_len), device, seq, kv_head)

    def prompt_queries(self, layer: int, device="cpu", seq=None, kv_head=None):
        """Queries of the prompt positions, [len(seq), P, len(kv_head)*G, d] (for the tracking over
        the prompt).  Noise, plus for position i >= 32 four times the key of position
        (5 i) mod 32 on query head i mod G (each of the first 32 keys is read again every 32
        positions), plus the sink term of the decode queries."""
        c = self.cfg
        G, P = c.group, c.prompt_len
        seq = list(range(c.batch) if seq is None else seq)
        kv_head = list(range(c.n_kv_heads) if kv_head is None else kv_head)
        q_heads = [h * G + g for h in kv_head for g in range(G)]
        q = self._noise(STREAM_QP, layer, range(P), seq, q_heads, c.n_q_heads, device)   # [P,s,hq,d]
        q = q.view(P, len(seq), len(kv_head), G, c.head_dim)
        if P > 32:
            k_hot = self._k_int(layer, range(32), seq, kv_head, device)                # [32,s,h,d]
            i = torch.arange(32, P, device=q.device)
            flat = q.permute(0, 3, 1, 2, 4).contiguous().view(P * G, len(seq), len(kv_head), c.head_dim)
            flat.index_add_(0, i * G + i % G, 4 * k_hot[(5 * i) % 32])
            q = flat.view(P, G, len(seq), len(kv_head), c.head_dim).permute(0, 2, 3, 1, 4)
        if c.n_sink:
            gain = int(round(32.0 * 6.0 / math.sqrt(c.head_dim)))
            k_sink = self._k_int(layer, range(c.n_sink), seq, kv_head, device).sum(dim=0)
            q = q + ((k_sink * gain) >> 5).view(1, len(seq), len(kv_head), 1, c.head_dim)
        q = self._finish(q.reshape(P, len(seq), len(kv_head) * G, c.head_dim).contiguous())
        return q.permute(1, 0, 2, 3).contiguous()

    # ---- per-step inputs -----------------------------------------------------------------
    def step_inputs(self, layer: int, t0: int, t1: int, device="cpu", seq=None, kv_head=None):
        """Inputs of decode steps t0..t1-1 (1-based steps).

        Returns q [n, len(seq), len(kv_head)*G, d], k_new and v_new [n, len(seq), len(kv_head), d].
        With kv_head given, q holds only the query heads of those groups, in order.
        """
        c = self.cfg
        G = c.group
        seq = list(range(c.batch) if seq is None else seq)
        kv_head = list(range(c.n_kv_heads) if kv_head is None else kv_head)
        steps = list(range(t0, t1))
        pos = [c.prompt_len + t - 1 for t in steps]
        k_new, v_new = self.kv_rows(layer, pos, device, seq, kv_head)      # [s,h,n,d]
        k_new = k_new.permute(2, 0, 1, 3).contiguous()
        v_new = v_new.permute(2, 0, 1, 3).contiguous()

        q_heads = [h * G + g for h in kv_head for g in range(G)]
        q = self._noise(STREAM_Q, layer, steps, seq, q_heads, c.n_q_heads, device)  # [n,s,hq,d]
        n, ns = len(steps), len(seq)
        q = q.view(n, ns, len(kv_head), G, c.head_dim)

        ev_t, ev_j = self.firings(t0, t1)
        if len(ev_t):
            uniq = np.unique(ev_j)
            k_fire = self._k_int(layer, uniq.tolist(), seq, kv_head, device)  # [u,s,h,d]
            row = torch.as_tensor(np.searchsorted(uniq, ev_j), device=k_fire.device)
            ti = torch.as_tensor(ev_t - t0, device=k_fire.device)
            gi = torch.as_tensor(ev_j % G, device=k_fire.device)
            flat = q.permute(0, 3, 1, 2, 4).contiguous().view(n * G, ns, len(kv_head), c.head_dim)
            flat.index_add_(0, ti * G + gi, 4 * k_fire[row])
            q = flat.view(n, G, ns, len(kv_head), c.head_dim).permute(0, 2, 3, 1, 4)
        if c.n_sink:
            gain = int(round(32.0 * 6.0 / math.sqrt(c.head_dim)))
            k_sink = self._k_int(layer, range(c.n_sink), seq, kv_head, device).sum(dim=0)  # [s,h,d]
            q = q + ((k_sink * gain) >> 5).view(1, ns, len(kv_head), 1, c.head_dim)
        q = self._finish(q.reshape(n, ns, len(kv_head) * G, c.head_dim).contiguous())
        return q, k_new, v_new
