"""CPU oracle for the LazyEviction decode-time path.  TEST INFRASTRUCTURE ONLY.

This file is a plain, slow, fp64 statement of what the method computes, written from the
paper (arXiv 2506.15969).  It shares no code with the HIP library and must never be imported
by it: only the tests, the smoke check and the CPU-baseline leg of the benchmark may use it.

What follows the paper, and where:
  * decode attention over the retained cache ............ Appendix A, Eq. 4
  * timestamp vector TS (last step with attention >= alpha) Sec. 4 "Recurrence Interval
    Tracking"; Algorithm 1, first loop
  * Maximum Recurrence Interval MRI ..................... Eq. 1
  * H1 / H2 scores and the MRI-centric importance I ..... Sec. 4 "MRI-Centric Eviction", Eq. 3
  * lagged eviction Top_{B-W}(I) united with the last W . Eq. 6, Algorithm 1
  * MRI distribution and the window chosen from it ...... Sec. 3 (Fig. 2(c)); Sec. 4
    "Observation Window"
  * current-attention ranking as an alternative score ... Sec. 2 (2); Appendix C "Baselines"
  * greedy current-attention comparator ................. Appendix C "Baselines" (TOVA sentence)
  * the same tracking run over the prompt (`prefill_tracking`) Algorithm 1, first loop, and Eq. 1
    applied to the prompt's own causal attention (the paper starts its clock at the first
    generated token and says nothing of the prompt: reading R18)

Readings taken where the paper is silent or inconsistent (each is also listed in the design
notes of the repository):
  R1  activation test is `>=` (Algorithm 1), not the prose's "exceeding".
  R2  eviction fires iff t is a multiple of W and the cache holds MORE than B entries (the
      prose of Sec. 4; the comparison printed in Algorithm 1 is the other way round).
  R3  t counts decode steps from 1.  Prompt entries start with TS = 0, MRI = 0; the entry
      generated at step t starts with TS = t, MRI = 0 (Sec. 4: "initialized to 0").
  R4  the new token's K/V is appended before attention and attends to itself (Eq. 4 uses
      K_1..K_{N_t}).
  R5  one recurrence state and one survivor set per (layer, sequence, KV head); the G query
      heads sharing a KV head are reduced by OR: active iff any head's probability >= alpha.
  R6  the thresholded quantity is the post-softmax probability over the retained cache.
  R7  tracking for step t is applied first, then scores use TS_t and MRI_t (Algorithm 1 order).
  R8  H2 is used exactly as printed, 2*sigmoid(-1/(MRI-1)), with H2 = 0 for MRI <= 1 (MRI = 1
      is the IEEE limit of the printed formula, MRI = 0 is stated by the paper).  H1 with
      MRI = 0 is the IEEE limit: 1 when t == TS, else 0.  The printed H2 grows with MRI although
      the sentence introducing it and App. D describe a decreasing term; the flag H2_DECREASING
      selects the reflected term 1 - H2 (1 at MRI = 1, 0 at MRI = 0) as the second reading.
  R9  ties in the top-k go to the more recent entry (larger slot index).
  R10 scores are binary64 and produced by ONE fixed sequence of IEEE operations (see
      `two_sigmoid_neg`), so that another implementation running the same sequence ranks
      identically; `two_sigmoid_neg_libm` is the same function through the C library and is
      what the fixed sequence is pinned against.

  R18 optional start state from the prompt: prompt token i (0-based, P tokens) is the query of
      step i + 1 - P <= 0 over the keys 0..i, tracked exactly like a decode step (R1, R4-R6);
      decoding then continues at step 1.  Without it prompt entries start as in R3.

Pins (tests/test_oracle_*.py, CPU only): closed forms of Eq. 3 via 50-digit decimals, a hand
trace of Eq. 1, full attention when B >= P+T against a library attention routine, the
sliding-window degenerate cases (alpha > 1 and alpha = 0), the closed-form eviction schedule and
saw-tooth cache length, window protection / stability / row-tag invariants, brute-force top-k on
tiny inputs, and planted recurring keys surviving where the greedy comparator drops them.
Accuracy on the paper's task benchmarks: parity unpinned (needs datasets and model weights).
"""
from __future__ import annotations

import math

import numpy as np

# --------------------------------------------------------------------------------------
# Eq. 3 building block: f(x) = 2*sigmoid(-x) = 2 / (1 + e^x) for x >= 0, in binary64.
# --------------------------------------------------------------------------------------

_LOG2E = float.fromhex("0x1.71547652b82fep+0")     # 1/ln 2, nearest double
_LN2_HI = float.fromhex("0x1.62e42fee00000p-1")    # ln 2 cut to 32 significant bits
_LN2_LO = float.fromhex("0x1.a39ef35793c76p-33")   # ln 2 - _LN2_HI, nearest double
_X_CUTOFF = 700.0                                  # e^x beyond this: f(x) := 0


def _inverse_factorials(n_terms: int) -> list[float]:
    out, fact = [], 1
    for n in range(n_terms):
        if n > 0:
            fact *= n
        out.append(1.0 / float(fact))              # one correctly rounded division each
    return out


_EXP_COEF = _inverse_factorials(14)                # c_0 .. c_13 = fl(1/n!)


def two_sigmoid_neg(x) -> np.ndarray:
    """f(x) = 2*sigmoid(-x) for x >= 0 (x may be +inf), by a fixed IEEE binary64 sequence.

    Sequence (every * and + and / is one round-to-nearest operation, nothing fused):
      x >= 700 or x = inf  ->  0
      k = floor(x*LOG2E + 0.5);  r = (x - k*LN2_HI) - k*LN2_LO
      p = c13; for n = 12..0: p = p*r + c_n        (two roundings per step)
      e = p * 2^k (exact scaling);  f = 2 / (1 + e)
    """
    x = np.asarray(x, dtype=np.float64)
    big = ~(x < _X_CUTOFF)                          # also catches inf
    xs = np.where(big, 0.0, x)
    k = np.floor(xs * _LOG2E + 0.5)
    r = (xs - k * _LN2_HI) - k * _LN2_LO
    p = np.full_like(xs, _EXP_COEF[13])
    for n in range(12, -1, -1):
        p = p * r
        p = p + _EXP_COEF[n]
    e = np.ldexp(p, k.astype(np.int64))
    f = 2.0 / (1.0 + e)
    return np.where(big, 0.0, f)


def two_sigmoid_neg_libm(x) -> np.ndarray:
    """The same function straight from its definition with the C library's exp."""
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(over="ignore"):
        return 2.0 / (1.0 + np.exp(x))


USE_H1 = 1
USE_H2 = 2
USE_CURRENT_ATTENTION = 32   # score = the step's own attention weight (the greedy baselines' rule)
H2_DECREASING = 16      # H2 reflected: 1 - f(1/(MRI-1)), the reading under which Sec. 4 item 2's prose holds


def mri_centric_score(t: int, ts, mri, score_flags: int = USE_H1 | USE_H2,
                      f=two_sigmoid_neg) -> np.ndarray:
    """Eq. 3: I = H1 + H2 (H2 only where MRI != 0), per cached entry, binary64.

    H1 = f((t - TS)/MRI)         Sec. 4 item 1;   MRI = 0: 1 if t == TS else 0 (R8)
    H2 = f(1/(MRI - 1))          Sec. 4 item 2;   0 for MRI <= 1 (R8)
    `score_flags` switches the two terms for the ablation of Table 4.  With H2_DECREASING the
    second term is 1 - f(1/(MRI - 1)) for MRI >= 1 (1 at MRI = 1, falling towards 0) and 0 for
    MRI = 0: the printed H2 grows with MRI, while the sentence that introduces it and App. D
    ask for a term that falls with MRI (R8); the reflection keeps the printed building block.
    """
    ts = np.asarray(ts, dtype=np.int64)
    mri = np.asarray(mri, dtype=np.int64)
    dt = (t - ts).astype(np.float64)
    m = mri.astype(np.float64)

    h1 = np.zeros(ts.shape, dtype=np.float64)
    if score_flags & USE_H1:
        has = mri > 0
        ratio = np.divide(dt, m, out=np.zeros_like(dt), where=has)
        h1 = np.where(has, f(ratio), np.where(dt == 0.0, 1.0, 0.0))

    h2 = np.zeros(ts.shape, dtype=np.float64)
    if score_flags & USE_H2:
        has = mri > 1
        inv = np.divide(1.0, m - 1.0, out=np.zeros_like(m), where=has)
        h2 = np.where(has, f(inv), 0.0)
        if score_flags & H2_DECREASING:
            h2 = np.where(mri >= 1, 1.0 - h2, 0.0)  # one more correctly rounded subtraction

    return h1 + h2


def mri_histogram(mri_values, n_bins: int) -> np.ndarray:
    """Number of cached entries per MRI value (Sec. 3, Fig. 2(c)); MRI >= n_bins - 1 share the
    last bin."""
    hist = np.zeros(n_bins, dtype=np.int64)
    for m in np.asarray(mri_values, dtype=np.int64).ravel():
        hist[min(int(m), n_bins - 1)] += 1
    return hist


def window_from_mri(mri_values, quantile: float = 0.8) -> int:
    """Sec. 4, "Observation Window": W = the MRI value that `quantile` of the recurring tokens
    (MRI >= 1) do not exceed, i.e. the ceil(quantile * n)-th smallest of their n MRI values."""
    v = np.sort(np.asarray(mri_values, dtype=np.int64).ravel())
    v = v[v >= 1]
    if len(v) == 0:
        return 0
    return int(v[max(int(math.ceil(quantile * len(v))) - 1, 0)])


def prefill_tracking(k_prompt, q_prompt, alpha: float, scale: float | None = None,
                     p_override=None):
    """TS and MRI of the P prompt entries of one unit after the first loop of Algorithm 1 and
    Eq. 1 have run over the prompt's own causal attention (R18).

    k_prompt [P,d]; q_prompt [P,G,d]: the G query heads of the unit's group at every prompt
    position.  Position i is step tau_i = i + 1 - P: its entry is born with TS = tau_i, MRI = 0,
    and its query sees the keys 0..i (Eq. 4 on the prefix).  p_override [G,P,P] (query row,
    key column; the lower triangle is read): weights to threshold instead of the computed
    ones, float32 compared in float32 as in `OracleUnit.decode_step`.
    Returns (TS [P] int64, MRI [P] int64, n_activations).
    """
    k = np.asarray(k_prompt, dtype=np.float64)
    q = np.asarray(q_prompt, dtype=np.float64)
    P, d = k.shape
    assert q.ndim == 3 and q.shape[0] == P and q.shape[2] == d
    scale = float(scale) if scale else 1.0 / np.sqrt(np.float64(d))
    TS = np.arange(P, dtype=np.int64) + 1 - P
    MRI = np.zeros(P, dtype=np.int64)
    n_act = 0
    for i in range(P):
        tau = i + 1 - P
        if p_override is not None:
            pw = np.asarray(p_override)[:, i, :i + 1]
            thr = np.float32(alpha) if pw.dtype == np.float32 else np.float64(alpha)
            act = (pw >= thr).any(axis=0)
        else:
            s = (q[i] @ k[:i + 1].T) * scale                     # [G, i+1]
            e = np.exp(s - s.max(axis=1, keepdims=True))
            p = e / e.sum(axis=1, keepdims=True)
            act = (p >= alpha).any(axis=0)
        idx = np.nonzero(act)[0]
        MRI[idx] = np.maximum(MRI[idx], tau - TS[idx])           # Eq. 1
        TS[idx] = tau                                            # Alg. 1
        n_act += len(idx)
    return TS, MRI, n_act


def select_survivors(score: np.ndarray, n_keep: int) -> np.ndarray:
    """Indices (ascending) of the `n_keep` best candidates: larger score first, and among equal
    scores the larger index (more recent) first (R9)."""
    n = score.shape[0]
    order = sorted(range(n), key=lambda i: (score[i], i), reverse=True)
    return np.array(sorted(order[:n_keep]), dtype=np.int64)


# --------------------------------------------------------------------------------------
# One (layer, sequence, KV head) unit
# --------------------------------------------------------------------------------------

class OracleUnit:
    """State of one KV head of one sequence in one layer, and Algorithm 1 on it.

    Every cached entry carries (pos, K row, V row, TS, MRI); the arrays stay in order of age
    (entry i of each array belongs to the same token).  Inputs are widened to fp64 exactly;
    nothing is rounded back except where a caller asks.
    """

    def __init__(self, k_prompt, v_prompt, n_group: int, budget: int, window: int,
                 alpha: float, scale: float | None = None,
                 score_flags: int = USE_H1 | USE_H2):
        k_prompt = np.asarray(k_prompt, dtype=np.float64)
        v_prompt = np.asarray(v_prompt, dtype=np.float64)
        assert k_prompt.ndim == 2 and k_prompt.shape == v_prompt.shape
        assert budget > window >= 1
        self.P, self.d = k_prompt.shape
        self.G, self.B, self.W = n_group, budget, window
        self.alpha = float(alpha)
        self.scale = float(scale) if scale else 1.0 / np.sqrt(np.float64(self.d))
        self.score_flags = score_flags
        self.K = k_prompt.copy()                     # [N,d]
        self.V = v_prompt.copy()
        self.pos = np.arange(self.P, dtype=np.int64)
        self.TS = np.zeros(self.P, dtype=np.int64)   # R3
        self.MRI = np.zeros(self.P, dtype=np.int64)  # R3
        self.t = 0
        self.n_activations = 0
        self.n_evict_events = 0
        self.last_weight = np.zeros(self.P)          # max over the group of the last step's weights

    def __len__(self) -> int:
        return len(self.pos)

    # -- Eq. 4 -------------------------------------------------------------------------
    def attention(self, q):
        """(out [G,d], p [G,N]) for the current cache; plain softmax attention in fp64."""
        q = np.asarray(q, dtype=np.float64).reshape(self.G, self.d)
        s = (q @ self.K.T) * self.scale              # [G,N]
        s = s - s.max(axis=1, keepdims=True)
        e = np.exp(s)
        p = e / e.sum(axis=1, keepdims=True)
        return p @ self.V, p

    # -- one decode step: append, attend, track (Algorithm 1 up to the MRI update) -------
    def decode_step(self, t: int, q, k_new, v_new, p_override=None, act_override=None):
        """Returns (out [G,d] fp64, p [G,N] fp64, act [N] bool).

        p_override [G,N]: attention weights to threshold instead of the computed ones
        (tracking only; `out` always comes from the computed weights).  float32 input is
        compared in float32 against float32(alpha), anything else in fp64.
        act_override: [N] bool array of activation decisions to take as given, or a callable
        (p, act) -> act that sees the oracle's own weights and decisions first.
        """
        assert t == self.t + 1, "decode steps are consecutive"
        self.t = t
        k_new = np.asarray(k_new, dtype=np.float64).reshape(1, self.d)
        v_new = np.asarray(v_new, dtype=np.float64).reshape(1, self.d)
        self.K = np.concatenate([self.K, k_new])                                     # R4
        self.V = np.concatenate([self.V, v_new])
        self.pos = np.append(self.pos, self.P + t - 1)
        self.TS = np.append(self.TS, t)                                              # R3
        self.MRI = np.append(self.MRI, 0)

        out, p = self.attention(q)

        if p_override is not None:
            pw = np.asarray(p_override).reshape(self.G, -1)
            self.last_weight = pw.max(axis=0).astype(np.float64)
        else:
            self.last_weight = p.max(axis=0)
        if act_override is not None and not callable(act_override):
            act = np.asarray(act_override, dtype=bool)
        elif p_override is not None:
            thr = np.float32(self.alpha) if pw.dtype == np.float32 else np.float64(self.alpha)
            act = (pw >= thr).any(axis=0)                                            # R1, R5
        else:
            act = (p >= self.alpha).any(axis=0)                                      # R1, R5, R6
        if callable(act_override):
            act = np.asarray(act_override(p, act), dtype=bool)
        assert act.shape == (len(self),)

        ts_prev = self.TS.copy()
        self.TS[act] = t                                                             # Alg. 1
        self.MRI = np.maximum(self.MRI, self.TS - ts_prev)                           # Eq. 1
        self.n_activations += int(act.sum())
        return out, p, act

    # -- lagged eviction (Eq. 6) ---------------------------------------------------------
    def eviction_due(self, t: int) -> bool:
        return t % self.W == 0 and len(self) > self.B                                # R2

    def scores(self, t: int) -> np.ndarray:
        if self.score_flags & USE_CURRENT_ATTENTION:
            # the rule of the current-attention baselines (Sec. 2; App. C, TOVA): rank by the
            # weight the entry received at this very step, largest over the query group
            assert t == self.t and len(self.last_weight) == len(self)
            return self.last_weight.copy()
        return mri_centric_score(t, self.TS, self.MRI, self.score_flags)

    def evict(self, t: int):
        """Runs the eviction check after step t.  Returns the evicted `pos` values (ascending),
        empty when nothing is due."""
        assert t == self.t
        if not self.eviction_due(t):
            return []
        n = len(self)
        n_cand = n - self.W                          # the last W entries are never candidates
        score = self.scores(t)[:n_cand]              # R7
        keep = np.zeros(n, dtype=bool)
        keep[select_survivors(score, self.B - self.W)] = True                        # Top_{B-W}
        keep[n_cand:] = True                                                         # last W
        gone = self.pos[~keep].tolist()
        for name in ("K", "V", "pos", "TS", "MRI"):                                  # order kept
            setattr(self, name, getattr(self, name)[keep])
        assert len(self) == self.B
        self.n_evict_events += 1
        return gone


class GreedyUnit:
    """Comparator: keeps the entries with the highest current attention at every step
    (Appendix C, the sentence describing TOVA).  After each step, while more than B entries are
    cached, the entry with the smallest max-over-group probability is dropped (never the newest;
    ties drop the older one).  CPU only; exists for the planted-key test."""

    def __init__(self, k_prompt, v_prompt, n_group: int, budget: int, scale=None):
        k_prompt = np.asarray(k_prompt, dtype=np.float64)
        self.P, self.d = k_prompt.shape
        self.G, self.B = n_group, budget
        self.scale = float(scale) if scale else 1.0 / np.sqrt(np.float64(self.d))
        self.K = [r.copy() for r in k_prompt]
        self.V = [r.copy() for r in np.asarray(v_prompt, dtype=np.float64)]
        self.pos = list(range(self.P))
        self.t = 0

    def __len__(self):
        return len(self.pos)

    def decode_step(self, t, q, k_new, v_new):
        self.t = t
        self.K.append(np.asarray(k_new, dtype=np.float64).copy())
        self.V.append(np.asarray(v_new, dtype=np.float64).copy())
        self.pos.append(self.P + t - 1)
        q = np.asarray(q, dtype=np.float64).reshape(self.G, self.d)
        s = (q @ np.stack(self.K).T) * self.scale
        s = s - s.max(axis=1, keepdims=True)
        e = np.exp(s)
        p = e / e.sum(axis=1, keepdims=True)
        out = p @ np.stack(self.V)
        cur = p.max(axis=0).tolist()
        while len(self.pos) > self.B:
            n = len(self.pos)
            victim = min(range(n - 1), key=lambda i: (cur[i], i))
            for lst in (self.K, self.V, self.pos, cur):
                del lst[victim]
        return out


# --------------------------------------------------------------------------------------
# All units of a model: [layer][sequence][KV head]
# --------------------------------------------------------------------------------------

class LazyEvictionOracle:
    """Independent units arranged as the library's caches are: no unit reads another's state."""

    def __init__(self, k_prompt, v_prompt, n_q_heads: int, budget: int, window: int,
                 alpha: float, scale=None, score_flags: int = USE_H1 | USE_H2):
        k_prompt = np.asarray(k_prompt)
        v_prompt = np.asarray(v_prompt)
        L, S, Hkv, P, d = k_prompt.shape
        assert n_q_heads % Hkv == 0
        self.L, self.S, self.Hkv, self.P, self.d = L, S, Hkv, P, d
        self.Hq, self.G = n_q_heads, n_q_heads // Hkv
        self.units = [[[OracleUnit(k_prompt[l, s, h], v_prompt[l, s, h], self.G, budget, window,
                                   alpha, scale, score_flags)
                        for h in range(Hkv)] for s in range(S)] for l in range(L)]

    def decode_step(self, layer: int, t: int, q, k_new, v_new, p_override=None):
        """q [S,Hq,d]; k_new, v_new [S,Hkv,d]; p_override [S,Hq,>=N] or None.
        Returns out [S,Hq,d] fp64 and p [S,Hq,N] fp64."""
        q = np.asarray(q)
        out = np.zeros((self.S, self.Hq, self.d))
        p_all = None
        for s in range(self.S):
            for h in range(self.Hkv):
                u = self.units[layer][s][h]
                g0, g1 = h * self.G, (h + 1) * self.G
                po = None
                if p_override is not None:
                    po = np.asarray(p_override)[s, g0:g1, :len(u) + 1]
                o, p, _ = u.decode_step(t, q[s, g0:g1], k_new[s, h], v_new[s, h], p_override=po)
                if p_all is None:
                    p_all = np.zeros((self.S, self.Hq, p.shape[1]))
                out[s, g0:g1] = o
                p_all[s, g0:g1] = p
        return out, p_all

    def evict(self, layer: int, t: int):
        return [[self.units[layer][s][h].evict(t) for h in range(self.Hkv)]
                for s in range(self.S)]

    def state(self, layer: int, name: str) -> np.ndarray:
        """[S,Hkv,N] int64 copy of 'pos', 'TS' or 'MRI'."""
        return np.array([[getattr(self.units[layer][s][h], name) for h in range(self.Hkv)]
                         for s in range(self.S)], dtype=np.int64)
