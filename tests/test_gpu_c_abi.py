"""The C ABI from a plain C99 program (csrc/abi_example.c, built by the package's build step
with gcc): no Python and no C++ between the caller and the library.  Its printed outputs and
survivor positions are compared with the CPU oracle on the same inputs."""
import os
import subprocess

import numpy as np
import pytest

from oracle.lazyev_oracle import OracleUnit

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HQ, HKV, D, P, B, W, STEPS = 4, 2, 64, 5, 8, 2, 12
ALPHA = 0.125


def _value(stream, pos, head, lane):
    return float((stream * 131 + pos * 31 + head * 17 + lane * 7) % 23 - 11) / 8.0


def _rows(stream, positions, head):
    return np.array([[_value(stream, p, head, l) for l in range(D)] for p in positions])


def test_plain_c_program_against_the_oracle():
    exe = os.path.join(ROOT, "paper_2506_15969_amd", "lib", "abi_example")
    assert os.path.exists(exe), "run `python -m paper_2506_15969_amd.build` first"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    lines = r.stdout.strip().splitlines()
    assert lines[-1] == "ok"
    G = HQ // HKV
    units = [OracleUnit(_rows(1, range(P), h), _rows(2, range(P), h), G, B, W, ALPHA) for h in range(HKV)]
    for t in range(1, STEPS + 1):
        f = lines[t - 1].split()
        assert f[0] == "step" and int(f[1]) == t and f[2] == "evicted" and f[4] == "out"
        got = np.array([float(x) for x in f[5:]]).reshape(HQ, D)          # every output element
        want, gone = [], []
        for h, u in enumerate(units):
            q = np.array([[_value(3, t, h * G + g, l) for l in range(D)] for g in range(G)])
            o, _, _ = u.decode_step(t, q, _rows(1, [P + t - 1], h)[0], _rows(2, [P + t - 1], h)[0])
            want.append(o)
            gone.append(len(u.evict(t)))
        assert int(f[3]) == gone[0] == gone[1]
        want = np.concatenate(want)                                        # [HQ, D] fp64
        # element by element, and the fp32 tolerance of the output rows (1e-5 relative L2)
        assert np.all(np.abs(got - want) <= 1e-5 * np.abs(want).max(axis=1, keepdims=True)), \
            (t, "\n", got, "\n", want)
        err = np.linalg.norm(got - want, axis=1) / np.linalg.norm(want, axis=1)
        assert err.max() <= 1e-5, (t, err)
    f = lines[STEPS].split()
    assert f == ["len", str(len(units[0])), "last_step", str(STEPS), "evict_events",
                 str(units[0].n_evict_events)]
    for h, u in enumerate(units):
        f = lines[STEPS + 1 + h].split()
        assert f[:3] == ["pos", "head", str(h)] and [int(x) for x in f[3:]] == u.pos.tolist()
