"""Pins for the CPU oracle: each test checks it against something fixed by the paper or by
mathematics, not against itself.  CPU only."""
import math
from decimal import Decimal, getcontext

import numpy as np
import pytest
import torch

from oracle.lazyev_oracle import (prefill_tracking, H2_DECREASING, USE_CURRENT_ATTENTION, USE_H1, USE_H2, GreedyUnit, LazyEvictionOracle, OracleUnit,
                                  mri_histogram, window_from_mri,
                                  mri_centric_score, select_survivors, two_sigmoid_neg,
                                  two_sigmoid_neg_libm)
from paper_2506_15969_amd.workload import CONFIGS, Workload

getcontext().prec = 50


def _f_exact(x: Decimal) -> Decimal:
    """2*sigmoid(-x) = 2/(1+e^x) in 50-digit decimal arithmetic (Sec. 4, H1/H2 definitions)."""
    return Decimal(2) / (Decimal(1) + x.exp())


def _ulps(a: float, b: float) -> float:
    if a == b:
        return 0.0
    return abs(a - b) / math.ulp(max(abs(a), abs(b)))


# ---------------------------------------------------------------- Eq. 3 closed forms
@pytest.mark.parametrize("dt,mri", [(0, 1), (1, 1), (5, 5), (10, 5), (50, 100), (300, 100),
                                    (7, 2), (90, 90), (1, 2), (4000, 3), (16384, 1), (3, 16000)])
def test_score_matches_printed_formula(dt, mri):
    """I = 2s(-(t-TS)/MRI) + 2s(-1/(MRI-1)) evaluated from the printed formulas in decimals."""
    t = 20000
    h1 = _f_exact(Decimal(dt) / Decimal(mri))
    h2 = _f_exact(Decimal(1) / Decimal(mri - 1)) if mri > 1 else Decimal(0)
    got = float(mri_centric_score(t, [t - dt], [mri])[0])
    assert abs(Decimal(got) - (h1 + h2)) <= Decimal(4) * Decimal(math.ulp(got))


def test_score_matches_golden_file():
    """tests/golden/eq3_values.txt: Eq. 3 from the printed formulas in decimal arithmetic."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "eq3_values.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 10
    t = 40000
    for dt, mri, want in rows:
        got = float(mri_centric_score(t, [t - int(dt)], [int(mri)])[0])
        assert abs(got - float(want)) <= 1e-12, (dt, mri, got, want)


def test_score_known_constants():
    """Values that follow by hand: f(0)=1, f(1)=2/(1+e); MRI=1 has no H2; MRI=0 rules."""
    t = 100
    f1 = 2.0 / (1.0 + math.e)
    s = mri_centric_score(t, [100, 99, 95, 100, 40], [1, 1, 5, 0, 0])
    assert s[0] == 1.0                                    # dt=0, MRI=1: H1=1, H2=0
    assert _ulps(s[1], f1) <= 2                           # dt=1, MRI=1
    assert _ulps(s[2], f1 + 2.0 / (1.0 + math.exp(0.25))) <= 2   # dt=MRI=5: f(1)+f(1/4)
    assert s[3] == 1.0                                    # MRI=0, dt=0
    assert s[4] == 0.0                                    # MRI=0, never re-activated
    # ablation switches (Table 4)
    assert mri_centric_score(t, [95], [5], USE_H1)[0] == two_sigmoid_neg(1.0)
    assert mri_centric_score(t, [95], [5], USE_H2)[0] == two_sigmoid_neg(0.25)
    assert mri_centric_score(t, [95], [5], 0)[0] == 0.0


def test_score_ranges_and_monotonicity():
    t = 5000
    ts = np.arange(0, t + 1)
    for mri in (1, 2, 3, 17, 175, 4096):
        s1 = mri_centric_score(t, ts, np.full_like(ts, mri), USE_H1)
        assert np.all((s1 >= 0) & (s1 <= 1))
        assert np.all(np.diff(s1) >= 0)                   # larger TS = smaller dt = larger H1
    m = np.arange(0, 5000)
    s2 = mri_centric_score(t, np.zeros_like(m), m, USE_H2)
    assert np.all((s2 >= 0) & (s2 < 1)) and s2[0] == 0 and s2[1] == 0
    assert np.all(np.diff(s2[2:]) > 0)                    # the printed H2 increases with MRI
    assert 0.5378 < s2[2] < 0.5379


def test_reflected_h2_is_tanh_and_decreases():
    """1 - 2/(1+e^x) = tanh(x/2): the reflected second term against the C library's tanh and
    decimals; it falls with MRI (what Sec. 4 item 2's prose and App. D ask of H2), is 1 at
    MRI = 1 and 0 for a never re-activated entry, and leaves H1 alone."""
    t = 9000
    m = np.arange(0, 6000)
    flags = USE_H2 | H2_DECREASING
    s = mri_centric_score(t, np.zeros_like(m), m, flags)
    assert s[0] == 0.0 and s[1] == 1.0
    want = np.tanh(0.5 / (m[2:] - 1.0))
    assert np.max(np.abs(s[2:] - want)) <= 5e-16            # 4 ulp of f near 1, then the subtraction
    assert np.all(np.diff(s[1:]) < 0) and np.all((s >= 0) & (s <= 1))
    for mri in (2, 3, 10, 175, 4096):
        exact = 1 - _f_exact(Decimal(1) / Decimal(mri - 1))
        assert abs(Decimal(float(s[mri])) - exact) <= Decimal(2) ** -51
    # printed + reflected = 1 for MRI > 1; the bit alone (without H2) changes nothing
    printed = mri_centric_score(t, np.zeros_like(m), m, USE_H2)
    assert np.max(np.abs(printed[2:] + s[2:] - 1.0)) <= 2.3e-16     # one rounding
    both = mri_centric_score(t, t - m, np.maximum(m, 1), USE_H1 | flags)
    h1 = mri_centric_score(t, t - m, np.maximum(m, 1), USE_H1)
    assert np.array_equal(both, h1 + mri_centric_score(t, t - m, np.maximum(m, 1), flags))
    assert np.array_equal(mri_centric_score(t, t - m, m, USE_H1 | H2_DECREASING),
                          mri_centric_score(t, t - m, m, USE_H1))


def test_fixed_sequence_exp_against_libm_and_decimal():
    rng = np.random.default_rng(7)
    x = np.concatenate([rng.uniform(0, 700, 200000), rng.uniform(0, 2, 50000),
                        1.0 / np.arange(1, 20000), np.arange(0, 700, 0.5)])
    a, b = two_sigmoid_neg(x), two_sigmoid_neg_libm(x)
    norm = a > 1e-300                                     # skip subnormal results
    ulp = np.abs(a[norm] - b[norm]) / np.spacing(np.maximum(a[norm], b[norm]))
    assert ulp.max() <= 4
    for xv in (0.0, 1e-9, 0.3, 1.0, 2.5, 17.0, 333.25, 699.99):
        assert _ulps(float(two_sigmoid_neg(xv)), float(_f_exact(Decimal(xv)))) <= 3
    assert two_sigmoid_neg(700.0) == 0 and two_sigmoid_neg(np.inf) == 0 and two_sigmoid_neg(0.0) == 1


def test_ln2_split_constants():
    from oracle import lazyev_oracle as o
    ln2 = Decimal(2).ln()
    assert Decimal(o._LN2_HI) <= ln2 and ln2 - Decimal(o._LN2_HI) < Decimal(2) ** -32
    assert int(Decimal(o._LN2_HI) * 2 ** 32) == Decimal(o._LN2_HI) * 2 ** 32   # 32 significant bits
    assert abs(Decimal(o._LN2_HI) + Decimal(o._LN2_LO) - ln2) < Decimal(2) ** -85
    assert abs(Decimal(o._LOG2E) - 1 / ln2) < Decimal(2) ** -53
    fact = 1
    for n, c in enumerate(o._EXP_COEF):
        fact *= max(n, 1)
        assert abs(Decimal(c) * fact - 1) < Decimal(2) ** -52


# ---------------------------------------------------------------- Eq. 1 hand trace
def _scripted_unit(P=1, d=4, B=1000, W=1):
    k = np.zeros((P, d))
    return OracleUnit(k, k, 1, B, W, alpha=0.5)


def test_ts_mri_hand_trace():
    """Token born at t=5, activated at 9, 10, 30: (TS,MRI) = (5,0),(9,4),(10,4),(30,20)."""
    u = _scripted_unit()
    seen = {}
    for t in range(1, 31):
        n = len(u) + 1
        act = np.zeros(n, dtype=bool)
        if t in (9, 10, 30):
            act[5] = True                                 # slot 5 = token appended at t=5 (P=1)
        u.decode_step(t, np.zeros((1, 4)), np.zeros(4), np.zeros(4), act_override=act)
        if t >= 5:
            seen[t] = (int(u.TS[5]), int(u.MRI[5]))
    assert seen[5] == (5, 0) and seen[8] == (5, 0)
    assert seen[9] == (9, 4) and seen[10] == (10, 4) and seen[29] == (10, 4) and seen[30] == (30, 20)
    # prompt token never activated keeps the initial state
    assert (u.TS[0], u.MRI[0]) == (0, 0)


def test_periodic_key_gets_its_period_as_mri():
    u = _scripted_unit()
    tau = 37
    for t in range(1, 3 * tau + 2):
        act = np.zeros(len(u) + 1, dtype=bool)
        if t % tau == 0:
            act[0] = True
        u.decode_step(t, np.zeros((1, 4)), np.zeros(4), np.zeros(4), act_override=act)
    assert u.MRI[0] == tau and u.TS[0] == 3 * tau


def test_self_activation_at_birth_leaves_mri_zero():
    u = _scripted_unit()
    act = np.array([False, True])
    u.decode_step(1, np.zeros((1, 4)), np.zeros(4), np.zeros(4), act_override=act)
    assert (u.TS[1], u.MRI[1]) == (1, 0)


def test_threshold_is_inclusive_and_grouped_by_or():
    k = np.zeros((3, 4))
    u = OracleUnit(k, k, 2, 100, 1, alpha=0.25)
    p = np.array([[0.25, 0.1, 0.1, 0.55], [0.0, 0.2499, 0.3, 0.45]], dtype=np.float32)
    _, _, act = u.decode_step(1, np.zeros((2, 4)), np.zeros(4), np.zeros(4), p_override=p)
    assert act.tolist() == [True, False, True, True]


def test_threshold_on_the_oracles_own_weights():
    """The same two rules on computed weights.  Head 0 has a zero query: its weights are exactly
    1/4 over four entries, equal to alpha; head 1 puts everything on entry 0.  Inclusive test
    and OR over the group: every entry is active (a strict test or an AND leaves only entry 0)."""
    k = np.zeros((3, 4))
    k[0, 0] = 3.0
    u = OracleUnit(k, k, 2, 100, 1, alpha=0.25)
    q = np.array([[0.0, 0, 0, 0], [40.0, 0, 0, 0]])
    _, p, act = u.decode_step(1, q, np.zeros(4), np.zeros(4))
    assert np.all(p[0] == 0.25) and p[1, 0] > 0.999 and np.all(p[1, 1:] < 1e-6)
    assert act.tolist() == [True, True, True, True]
    assert u.TS.tolist() == [1, 1, 1, 1] and u.MRI.tolist() == [1, 1, 1, 0]


# ---------------------------------------------------------------- Eq. 4 against a library routine
def test_budget_at_least_sequence_length_is_full_attention():
    rng = np.random.default_rng(3)
    P, T, d, G = 9, 40, 16, 3
    kp, vp = rng.standard_normal((P, d)), rng.standard_normal((P, d))
    u = OracleUnit(kp, vp, G, budget=P + T, window=4, alpha=0.01)
    K, V = torch.tensor(kp), torch.tensor(vp)
    for t in range(1, T + 1):
        q, kn, vn = rng.standard_normal((G, d)), rng.standard_normal(d), rng.standard_normal(d)
        out, p, _ = u.decode_step(t, q, kn, vn)
        assert u.evict(t) == []
        K = torch.cat([K, torch.tensor(kn)[None]])
        V = torch.cat([V, torch.tensor(vn)[None]])
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.tensor(q)[None], K[None], V[None])[0].numpy()
        np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-13)
    assert len(u) == P + T


def test_attention_of_identical_keys_is_the_mean_value():
    d = 8
    k = np.ones((5, d))
    v = np.arange(5 * d, dtype=float).reshape(5, d)
    u = OracleUnit(k, v, 1, 100, 1, alpha=2.0)
    out, p, _ = u.decode_step(1, np.ones((1, d)), np.ones(d), v[2])
    np.testing.assert_allclose(p, 1 / 6)
    np.testing.assert_allclose(out[0], (v.sum(0) + v[2]) / 6)


# ---------------------------------------------------------------- top-k, ties, degenerate cases
def test_select_survivors_brute_force():
    rng = np.random.default_rng(11)
    for trial in range(200):
        n = int(rng.integers(2, 24))
        k = int(rng.integers(1, n))
        score = rng.integers(0, 4, n).astype(float) if trial % 2 else rng.random(n)
        keep = set(select_survivors(score, k).tolist())
        assert len(keep) == k
        for i in keep:                                    # nothing left out beats anything kept
            for j in set(range(n)) - keep:
                assert (score[i], i) > (score[j], j)


def _run_random_unit(alpha, P=20, T=130, B=32, W=8, d=8, G=2, seed=5, flags=USE_H1 | USE_H2):
    rng = np.random.default_rng(seed)
    u = OracleUnit(rng.standard_normal((P, d)), rng.standard_normal((P, d)), G, B, W, alpha,
                   score_flags=flags)
    trace = []
    for t in range(1, T + 1):
        u.decode_step(t, rng.standard_normal((G, d)), rng.standard_normal(d), rng.standard_normal(d))
        gone = u.evict(t)
        trace.append((t, len(u), gone, u.pos.copy()))
    return u, trace


@pytest.mark.parametrize("alpha", [2.0, 0.0])
def test_degenerate_alpha_is_a_sliding_window(alpha):
    """alpha > 1: nothing activates, every score is 0.  alpha = 0: everything activates every
    step, every candidate scores 1.  All tied, and ties go to the recent: keep the newest B."""
    u, trace = _run_random_unit(alpha)
    for t, n, gone, pos in trace:
        if gone:
            newest = 20 + t - 1
            assert pos.tolist() == list(range(newest - 32 + 1, newest + 1))


def test_scores_off_is_a_sliding_window():
    u, trace = _run_random_unit(0.05, flags=0)
    for t, n, gone, pos in trace:
        if gone:
            assert pos.tolist() == list(range(20 + t - 32, 20 + t))


def test_schedule_sawtooth_and_protection():
    """Eviction at t = kW once the cache exceeds B; length climbs B+1..B+W in between and is
    exactly B after an eviction; nothing from the last W steps is evicted; order is kept."""
    P, B, W = 20, 32, 8
    u, trace = _run_random_unit(0.08)
    first = min(t for t in range(W, 1000, W) if P + t > B)
    assert first == 16
    for t, n, gone, pos in trace:
        assert n <= B + W
        if t % W == 0 and t >= first:
            assert n == B and len(gone) > 0
            assert all(g < P + t - W for g in gone)        # window protected
        else:
            assert gone == []
        assert np.all(np.diff(pos) > 0)                   # stable compaction
    assert u.n_evict_events == (130 - first) // W + 1


@pytest.mark.parametrize("name,first,events", [("cfg1", 80, 28), ("cfg2", 544, 112),
                                               ("cfg3", 1856, 228), ("cfg4", 896, 122),
                                               ("cfg5", 3648, 456)])
def test_closed_form_schedule_of_the_configs(name, first, events):
    c = CONFIGS[name]
    due = [t for t in range(c.window, c.steps + 1, c.window) if c.prompt_len + t > c.budget]
    assert due[0] == first and len(due) == events
    # the oracle's trigger agrees with it (lengths follow the saw-tooth, so test the predicate)
    u = OracleUnit(np.zeros((c.budget + c.window, 2)), np.zeros((c.budget + c.window, 2)), 1,
                   c.budget, c.window, 0.5)
    assert u.eviction_due(first) and not u.eviction_due(first + 1)
    u2 = OracleUnit(np.zeros((c.budget, 2)), np.zeros((c.budget, 2)), 1, c.budget, c.window, 0.5)
    assert not u2.eviction_due(first)                     # exactly B entries: nothing to do


def test_rows_and_statistics_travel_with_their_token():
    rng = np.random.default_rng(9)
    P, B, W, d = 12, 24, 6, 4
    tag = lambda pos: np.full(d, float(pos))
    u = OracleUnit(np.stack([tag(i) for i in range(P)]), np.stack([-tag(i) for i in range(P)]),
                   1, B, W, alpha=0.5)
    book = {i: (0, 0) for i in range(P)}
    for t in range(1, 80):
        n = len(u) + 1
        act = rng.random(n) < 0.2
        pos_now = list(u.pos) + [P + t - 1]
        u.decode_step(t, np.zeros((1, d)), tag(P + t - 1), -tag(P + t - 1), act_override=act)
        book[P + t - 1] = (t, 0)
        for i in np.nonzero(act)[0]:
            ts, mri = book[pos_now[i]]
            book[pos_now[i]] = (t, max(mri, t - ts))
        u.evict(t)
        for i, pos in enumerate(u.pos):
            assert u.K[i, 0] == pos and u.V[i, 0] == -pos
            assert (u.TS[i], u.MRI[i]) == book[pos]
            assert u.TS[i] <= t and u.MRI[i] <= t - max(0, pos - P + 1)


# ---------------------------------------------------------------- heuristic quality
def test_planted_recurring_keys_survive_where_greedy_drops_them():
    """cfg1: 8 prompt keys re-attended every 40-90 steps.  LazyEviction keeps all of them for
    the whole run; keeping the highest current attention at every step loses them."""
    w = Workload(CONFIGS["cfg1"])
    c = w.cfg
    K, V = w.prompt_kv(0)
    q, kn, vn = w.step_inputs(0, 1, c.steps + 1)
    lazy_alive, greedy_alive = [], []
    for h in range(c.n_kv_heads):
        lazy = OracleUnit(K[0, h].numpy(), V[0, h].numpy(), 1, c.budget, c.window, c.alpha)
        greedy = GreedyUnit(K[0, h].numpy(), V[0, h].numpy(), 1, c.budget)
        for t in range(1, c.steps + 1):
            lazy.decode_step(t, q[t - 1, 0, h:h + 1].numpy(), kn[t - 1, 0, h].numpy(),
                             vn[t - 1, 0, h].numpy())
            lazy.evict(t)
            greedy.decode_step(t, q[t - 1, 0, h:h + 1].numpy(), kn[t - 1, 0, h].numpy(),
                               vn[t - 1, 0, h].numpy())
            assert len(lazy) <= c.budget + c.window and len(greedy) <= c.budget
        lazy_alive.append(len(set(w.planted.tolist()) & set(lazy.pos.tolist())))
        greedy_alive.append(len(set(w.planted.tolist()) & set(greedy.pos)))
    assert lazy_alive == [8] * c.n_kv_heads
    assert max(greedy_alive) < 8 and sum(greedy_alive) <= 0.5 * sum(lazy_alive)


def test_multi_unit_wrapper_matches_single_units():
    w = Workload(CONFIGS["cfg2"].scaled(batch=2, prompt_len=24, steps=40, budget=32, window=8))
    c = w.cfg
    K, V = w.prompt_kv(0)
    q, kn, vn = w.step_inputs(0, 1, c.steps + 1)
    full = LazyEvictionOracle(K[None].float().numpy(), V[None].float().numpy(), c.n_q_heads,
                              c.budget, c.window, c.alpha)
    s, h, G = 1, 2, c.group
    one = OracleUnit(K[s, h].float().numpy(), V[s, h].float().numpy(), G, c.budget, c.window, c.alpha)
    for t in range(1, c.steps + 1):
        out, _ = full.decode_step(0, t, q[t - 1].float().numpy(), kn[t - 1].float().numpy(),
                                  vn[t - 1].float().numpy())
        o1, _, _ = one.decode_step(t, q[t - 1, s, h * G:(h + 1) * G].float().numpy(),
                                   kn[t - 1, s, h].float().numpy(), vn[t - 1, s, h].float().numpy())
        full.evict(0, t)
        one.evict(t)
        assert np.array_equal(out[s, h * G:(h + 1) * G], o1)
    assert np.array_equal(full.state(0, "pos")[s, h], one.pos)
    assert np.array_equal(full.state(0, "MRI")[s, h], one.MRI)


# ---------------------------------------------------------------- MRI statistics (Sec. 3 / Sec. 4)
def test_mri_histogram_and_window_against_library_routines():
    rng = np.random.default_rng(11)
    for n in (1, 5, 10, 997, 4000):
        mri = np.where(rng.random(n) < 0.4, 0, rng.geometric(0.02, n))
        h = mri_histogram(mri, 64)
        assert np.array_equal(h[:63], np.bincount(mri, minlength=4096)[:63])
        assert h[63] == (mri >= 63).sum() and h.sum() == n
        rec = mri[mri >= 1]
        for q in (0.5, 0.8, 0.95, 1.0):
            want = int(np.quantile(rec, q, method="inverted_cdf")) if len(rec) else 0
            assert window_from_mri(mri, q) == want
    assert window_from_mri([0, 0, 0]) == 0
    assert window_from_mri([0, 7]) == 7
    assert window_from_mri([1, 2, 3, 4, 5, 6, 7, 8, 9, 10]) == 8      # 80 % of ten values


def test_window_of_periodic_keys_is_their_period():
    """Six prompt keys re-attended every 37 steps and nothing else: every one of them has
    MRI = 37 (Eq. 1; prompt entries start at TS = 0), so the histogram is a single spike and
    W = 37."""
    u = _scripted_unit(P=6, B=1000, W=1)
    for t in range(1, 120):
        act = np.zeros(len(u) + 1, dtype=bool)
        if t % 37 == 0:
            act[:6] = True
        u.decode_step(t, np.zeros((1, 4)), np.zeros(4), np.zeros(4), act_override=act)
    h = mri_histogram(u.MRI, 64)
    assert h[37] == 6 and h[0] == len(u) - 6 and h.sum() == len(u)
    assert window_from_mri(u.MRI) == 37


# ---------------------------------------------------------------- current-attention ranking
def test_current_attention_with_window_one_is_the_greedy_comparator():
    """Ranking by the step's own weights and evicting after every step (W = 1) is the greedy
    rule (App. C, TOVA): the general eviction path and the separately written comparator must
    keep the same entries at every step, also when the prompt is longer than the budget."""
    rng = np.random.default_rng(3)
    P, d, G, B = 40, 8, 2, 24
    k, v = rng.normal(size=(P, d)), rng.normal(size=(P, d))
    a = OracleUnit(k, v, G, B, 1, alpha=0.05, score_flags=USE_CURRENT_ATTENTION)
    g = GreedyUnit(k, v, G, B)
    for t in range(1, 120):
        q, kn, vn = rng.normal(size=(G, d)) * 3, rng.normal(size=d), rng.normal(size=d)
        oa, _, _ = a.decode_step(t, q, kn, vn)
        og = g.decode_step(t, q, kn, vn)
        a.evict(t)
        assert np.allclose(oa, og) and a.pos.tolist() == g.pos and len(a) == B


def test_current_attention_behind_a_window_by_hand():
    """Five prompt entries, budget 4, window 2: at t = 2 the candidates are the five prompt
    entries, the weights of step 2 decide, the two newest entries stay whatever they got."""
    k = np.zeros((5, 4))
    u = OracleUnit(k, k, 1, 4, 2, alpha=0.5, score_flags=USE_CURRENT_ATTENTION)
    w1 = np.array([[0.9, 0.02, 0.02, 0.02, 0.02, 0.02]])
    w2 = np.array([[0.05, 0.3, 0.01, 0.2, 0.3, 0.04, 0.1]])
    u.decode_step(1, np.zeros((1, 4)), np.zeros(4), np.zeros(4), p_override=w1)
    assert u.evict(1) == []                               # t is not a multiple of W
    u.decode_step(2, np.zeros((1, 4)), np.zeros(4), np.zeros(4), p_override=w2)
    assert u.evict(2) == [0, 2, 3]                        # keeps 4 (tie with 1: the newer) and 1
    assert u.pos.tolist() == [1, 4, 5, 6]


# ---------------------------------------------------------------- invariants on random runs
def test_invariants_over_random_configurations():
    """What Sec. 4, Eq. 1 and Eq. 6 fix whatever the inputs are, on 60 random (P, B, W, alpha)
    with random injected weights: the cache never holds more than max(P, B) + W entries and exactly B
    after a due eviction; an eviction removes nothing younger than W steps and keeps the order;
    per token MRI never shrinks, TS <= t, MRI <= t - birth, MRI = 0 exactly for tokens never
    activated after their birth step, TS = birth for those; statistics travel with the token."""
    rng = np.random.default_rng(2024)
    for case in range(60):
        B = int(rng.integers(3, 40))
        W = int(rng.integers(1, B))
        P = int(rng.integers(0, 60))
        G = int(rng.integers(1, 4))
        alpha = float(rng.choice([0.0, 0.02, 0.1, 0.3, 1.5]))
        u = OracleUnit(np.zeros((P, 2)), np.zeros((P, 2)), G, B, W, alpha,
                       score_flags=int(rng.choice([3, 1, 2, 0, 3 | 16])))
        birth = lambda pos: max(0, pos - P + 1)           # noqa: E731  (step that appended it)
        hist = {}                                          # pos -> (TS, MRI, ever activated later)
        for t in range(1, 3 * W + 25):
            n1 = len(u) + 1
            p = (rng.random((G, n1)) ** 4 * 0.5).astype(np.float32)
            _, _, act = u.decode_step(t, np.zeros((G, 2)), np.zeros(2), np.zeros(2), p_override=p)
            assert len(u) <= max(P, B) + W                 # the capacity a caller has to provide
            for i, pos in enumerate(u.pos.tolist()):
                ts, mri = int(u.TS[i]), int(u.MRI[i])
                old = hist.get(pos, (birth(pos), 0, False))
                later = old[2] or (bool(act[i]) and t > birth(pos))
                assert mri >= old[1] and ts >= old[0] and ts <= t
                assert mri <= t - birth(pos)
                assert (mri == 0) == (not later)
                if not later:
                    assert ts == birth(pos)
                hist[pos] = (ts, mri, later)
            before = u.pos.copy()
            due = t % W == 0 and len(u) > B
            gone = u.evict(t)
            assert bool(gone) == due
            if due:
                assert len(u) == B and all(g < P + t - W for g in gone)
                assert np.all(np.diff(u.pos) > 0) and set(u.pos.tolist()) | set(gone) == set(before.tolist())
                for i, pos in enumerate(u.pos.tolist()):   # (TS, MRI) moved with their token
                    assert (int(u.TS[i]), int(u.MRI[i])) == hist[pos][:2]


# ---------------------------------------------------------------- tracking over the prompt
def test_prefill_tracking_by_hand():
    """Zero queries give uniform weights 1/(i+1) at prompt position i.  With alpha = 0.4 the
    positions 0 and 1 activate everything they see and position 2 (weights 1/3) nothing:
    key 0 is hit at steps -2 (its birth) and -1, key 1 at -1 (birth), key 2 at 0 (birth)."""
    k = np.arange(6, dtype=np.float64).reshape(3, 2)
    q = np.zeros((3, 1, 2))
    ts, mri, n_act = prefill_tracking(k, q, 0.4)
    assert ts.tolist() == [-1, -1, 0] and mri.tolist() == [1, 0, 0] and n_act == 3
    # alpha = 0: every query activates every key it sees: all TS end at 0, every gap is 1
    ts, mri, n_act = prefill_tracking(np.ones((5, 2)), np.zeros((5, 2, 2)), 0.0)
    assert ts.tolist() == [0] * 5 and mri.tolist() == [1, 1, 1, 1, 0] and n_act == 15
    # alpha > 1: nothing is ever active
    ts, mri, n_act = prefill_tracking(np.ones((5, 2)), np.zeros((5, 2, 2)), 1.5)
    assert ts.tolist() == [-4, -3, -2, -1, 0] and mri.tolist() == [0] * 5 and n_act == 0


def test_prefill_tracking_is_the_decode_tracking_fed_with_the_prompt():
    """The same tokens fed one by one as decode steps 1..P to a unit that starts empty and never
    evicts leave the same MRI, and TS shifted by P (its clock starts at 1, the prompt's ends at 0)."""
    rng = np.random.default_rng(5)
    P, G, d = 40, 3, 8
    k, v = rng.standard_normal((P, d)), rng.standard_normal((P, d))
    q = 2.0 * rng.standard_normal((P, G, d))
    alpha = 0.08
    ts, mri, n_act = prefill_tracking(k, q, alpha)
    u = OracleUnit(np.zeros((0, d)), np.zeros((0, d)), G, 10 * P, 4, alpha)
    for t in range(1, P + 1):
        u.decode_step(t, q[t - 1], k[t - 1], v[t - 1])
        assert u.evict(t) == []
    assert np.array_equal(u.TS - P, ts) and np.array_equal(u.MRI, mri) and u.n_activations == n_act
    assert mri.max() > 1 and (mri == 0).sum() > 0               # the case is not degenerate
    # handing the computed weights in as float32 decides the same wherever no weight sits within
    # float32 rounding of alpha (checked), and the override is what is thresholded
    p_all = np.zeros((G, P, P), dtype=np.float32)
    for i in range(P):
        s = (q[i] @ k[:i + 1].T) / np.sqrt(d)
        e = np.exp(s - s.max(axis=1, keepdims=True))
        p_all[:, i, :i + 1] = (e / e.sum(axis=1, keepdims=True)).astype(np.float32)
    assert np.abs(p_all[p_all > 0] - np.float32(alpha)).min() > 1e-6
    ts2, mri2, n2 = prefill_tracking(k, q, alpha, p_override=p_all)
    assert np.array_equal(ts2, ts) and np.array_equal(mri2, mri) and n2 == n_act
    ts3, _, n3 = prefill_tracking(k, q, alpha, p_override=np.zeros_like(p_all))
    assert n3 == 0 and ts3.tolist() == list(range(1 - P, 1))


def test_prefill_tracking_periodic_reader():
    """A key that is read by every 5th prompt position and by nobody else gets MRI = 5."""
    P, d = 31, 4
    k = np.zeros((P, d)); k[:, 1] = 1.0
    k[3] = [6.0, 0.0, 0.0, 0.0]                                  # the key that gets read
    q = np.zeros((P, 1, d)); q[:, 0, 1] = 6.0                    # everybody else: uniform over the rest
    for i in range(8, P, 5):
        q[i, 0] = [12.0, 0.0, 0.0, 0.0]
    ts, mri, _ = prefill_tracking(k, q, 0.5, scale=1.0)
    # (its own query at position 3 spreads e^36 over three older keys: 1/3 < 0.5, so the first
    # hit comes at position 8, five steps after its birth)
    assert mri[3] == 5 and ts[3] == 28 + 1 - P
    assert mri[np.arange(P) != 3].max() <= 1
