"""How sharp the oracle's pins are: plausible mistakes are planted one at a time in a COPY of
the oracle's source (on the CPU, in memory), the pin tests of test_oracle_pins.py are run
against the mutant, and every mutant must fail at least one of them.  The unmodified copy must
pass all of them.  CPU only."""
import importlib.util
import inspect
import os
import sys
import types

import pytest

import test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "lazyev_oracle.py")).read()

# (name, text in the oracle, replacement)
MUTANTS = [
    ("strict threshold", "act = (p >= self.alpha).any(axis=0)", "act = (p > self.alpha).any(axis=0)"),
    ("AND over the group", "act = (p >= self.alpha).any(axis=0)", "act = (p >= self.alpha).all(axis=0)"),
    ("eviction at N == B", "len(self) > self.B", "len(self) >= self.B"),
    ("eviction every step", "return t % self.W == 0 and", "return"),
    ("MRI = last gap", "self.MRI = np.maximum(self.MRI, self.TS - ts_prev)", "self.MRI = np.where(act, self.TS - ts_prev, self.MRI)"),
    ("MRI = min gap", "self.MRI = np.maximum(self.MRI, self.TS - ts_prev)",
     "self.MRI = np.where(act & (self.MRI > 0), np.minimum(self.MRI, self.TS - ts_prev), np.maximum(self.MRI, self.TS - ts_prev))"),
    ("TS one step late", "self.TS[act] = t  ", "self.TS[act] = t - 1  "),
    ("new entry TS = 0", "self.TS = np.append(self.TS, t)", "self.TS = np.append(self.TS, 0)"),
    ("new entry MRI = 1", "self.MRI = np.append(self.MRI, 0)", "self.MRI = np.append(self.MRI, 1)"),
    ("attention before the append", None, None),   # handled below: moves the attention call
    ("no softmax scale", "s = (q @ self.K.T) * self.scale              # [G,N]", "s = (q @ self.K.T)"),
    ("output from K", "return p @ self.V, p", "return p @ self.K, p"),
    ("softmax over heads", "p = e / e.sum(axis=1, keepdims=True)\n        return p @ self.V, p",
     "p = e / e.sum(axis=0, keepdims=True)\n        return p @ self.V, p"),
    ("window not protected", "n_cand = n - self.W  ", "n_cand = n  "),
    ("window one short", "n_cand = n - self.W  ", "n_cand = n - self.W + 1  "),
    ("keeps B - W + 1", "select_survivors(score, self.B - self.W)", "select_survivors(score, self.B - self.W + 1)"),
    ("older entry wins ties", "key=lambda i: (score[i], i), reverse=True", "key=lambda i: (score[i], -i), reverse=True"),
    ("lowest scores kept", "key=lambda i: (score[i], i), reverse=True", "key=lambda i: (-score[i], i), reverse=True"),
    ("H1 increasing", "h1 = np.where(has, f(ratio),", "h1 = np.where(has, 1.0 - f(ratio),"),
    ("H1 = f(MRI / dt)", "ratio = np.divide(dt, m, out=np.zeros_like(dt), where=has)",
     "ratio = np.divide(m, np.maximum(dt, 1.0), out=np.zeros_like(dt), where=has)"),
    ("H2 = f(1 / MRI)", "inv = np.divide(1.0, m - 1.0,", "inv = np.divide(1.0, m,"),
    ("H2 dropped", "return h1 + h2", "return h1"),
    ("sigmoid without the 2", "f = 2.0 / (1.0 + e)", "f = 1.0 / (1.0 + e)"),
    ("exp(-x) for exp(x)", "f = 2.0 / (1.0 + e)", "f = 2.0 / (1.0 + 1.0 / e)"),
    ("polynomial one term short", "p = np.full_like(xs, _EXP_COEF[13])\n    for n in range(12, -1, -1):",
     "p = np.full_like(xs, _EXP_COEF[8])\n    for n in range(7, -1, -1):"),
    ("rows not moved with their token", 'for name in ("K", "V", "pos", "TS", "MRI"):', 'for name in ("V", "pos", "TS", "MRI"):'),
    ("MRI not moved with its token", 'for name in ("K", "V", "pos", "TS", "MRI"):', 'for name in ("K", "V", "pos", "TS"):'),
    ("score from stale TS", "dt = (t - ts).astype(np.float64)", "dt = (t - 1 - ts).astype(np.float64)"),
    ("reflected H2 not reflected", "h2 = np.where(mri >= 1, 1.0 - h2, 0.0)", "h2 = np.where(mri >= 1, h2, 0.0)"),
    ("current attention: smallest over the group", "self.last_weight = p.max(axis=0)", "self.last_weight = p.min(axis=0)"),
    ("current attention: injected weights ignored", "            self.last_weight = pw.max(axis=0).astype(np.float64)\n", "            self.last_weight = p.max(axis=0)\n"),
    ("histogram without overflow bin", "hist[min(int(m), n_bins - 1)] += 1", "hist[int(m) % n_bins] += 1"),
    ("window quantile over all entries", "    v = v[v >= 1]\n", ""),
    ("prompt tracking: query does not see its own key", "s = (q[i] @ k[:i + 1].T) * scale                     # [G, i+1]",
     "s = (q[i] @ k[:max(i, 1)].T) * scale"),
    ("prompt tracking: clock ends at P", "        tau = i + 1 - P\n", "        tau = i + 1\n"),
    ("prompt tracking: MRI = last gap", "MRI[idx] = np.maximum(MRI[idx], tau - TS[idx])           # Eq. 1", "MRI[idx] = tau - TS[idx]"),
    ("prompt tracking: AND over the group", "            act = (p >= alpha).any(axis=0)\n        idx", "            act = (p >= alpha).all(axis=0)\n        idx"),
    ("prompt tracking: injected weights ignored", "        if p_override is not None:\n            pw = np.asarray(p_override)[:, i, :i + 1]", "        if False:\n            pw = np.asarray(p_override)[:, i, :i + 1]"),
]


def _mutated_source(name, old, new):
    if name == "attention before the append":
        src = SOURCE
        a = src.index("        out, p = self.attention(q)\n")
        src = src[:a] + src[a + len("        out, p = self.attention(q)\n"):]
        marker = "        k_new = np.asarray(k_new, dtype=np.float64).reshape(1, self.d)\n"
        # attend over the old cache, then pad the weights with a zero column for the new entry
        return src.replace(marker, "        out, p = self.attention(q)\n"
                                   "        p = np.concatenate([p, np.zeros((self.G, 1))], axis=1)\n" + marker, 1)
    assert SOURCE.count(old) >= 1, "mutation target not found: " + name
    return SOURCE.replace(old, new)


def _load(source, tag):
    mod = types.ModuleType("oracle_mutant_" + tag)
    mod.__file__ = "<mutant %s>" % tag
    sys.modules[mod.__name__] = mod               # dataclasses / typing look the module up
    exec(compile(source, mod.__file__, "exec"), mod.__dict__)
    return mod


PIN_TESTS = [(n, f) for n, f in inspect.getmembers(pins, inspect.isfunction) if n.startswith("test_")]
SWAPPED = ["H2_DECREASING", "USE_CURRENT_ATTENTION", "USE_H1", "USE_H2", "GreedyUnit", "LazyEvictionOracle", "OracleUnit",
           "mri_histogram", "window_from_mri", "mri_centric_score", "select_survivors",
           "two_sigmoid_neg", "two_sigmoid_neg_libm", "prefill_tracking"]


def _run_pins(mod):
    """Runs every pin test with the oracle names of test_oracle_pins bound to `mod`; returns the
    names of the tests that failed."""
    saved = {n: getattr(pins, n) for n in SWAPPED}
    saved_mod = sys.modules.get("oracle.lazyev_oracle")
    failed = []
    try:
        for n in SWAPPED:
            setattr(pins, n, getattr(mod, n))
        sys.modules["oracle.lazyev_oracle"] = mod           # for tests that import it themselves
        import oracle
        saved_attr = getattr(oracle, "lazyev_oracle", None)
        oracle.lazyev_oracle = mod
        for name, fn in PIN_TESTS:
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            cases = [()]
            if marks:
                argnames = [a.strip() for a in marks[0].args[0].split(",")]
                cases = [c if isinstance(c, tuple) else (c,) for c in marks[0].args[1]]
                cases = [c for c in cases if len(c) == len(argnames)]
            for case in cases:
                try:
                    fn(*case)
                except Exception:                            # any failure of the pin counts
                    failed.append(name)
                    break
        oracle.lazyev_oracle = saved_attr
    finally:
        for n, v in saved.items():
            setattr(pins, n, v)
        if saved_mod is not None:
            sys.modules["oracle.lazyev_oracle"] = saved_mod
    return failed


def test_the_unmodified_copy_passes_every_pin():
    assert _run_pins(_load(SOURCE, "identity")) == []


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_every_planted_mistake_fails_a_pin(name, old, new):
    failed = _run_pins(_load(_mutated_source(name, old, new), str(abs(hash(name)))))
    assert failed, "no pin notices: " + name
