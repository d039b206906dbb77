"""The eviction kernels on hand-made recurrence states: the statistics arrays belong to the
caller, so a test can write any (TS, MRI) pattern before an eviction and compare the survivors
with the oracle's scoring and selection (Eq. 3, Eq. 6).  The patterns aim at the radix select:
every key equal, two values, keys that differ only in their low bits, a tie group that
straddles the cut, no ties at all.  (TS may be negative here: only t - TS enters the score.)"""
import numpy as np
import pytest
import torch

from oracle.lazyev_oracle import mri_centric_score, select_survivors

pytestmark = pytest.mark.gpu

B, W, D, HKV = 1500, 20, 64, 12
T = W                                                  # the step of the eviction


def _patterns(rng):
    """One (TS, MRI) pair of arrays over the B candidates per unit."""
    n, t = B, T
    pats = []
    pats.append((np.zeros(n, int), np.zeros(n, int)))                          # all score 0
    pats.append((np.full(n, t - 5), np.full(n, 5)))                            # all equal, non-zero
    pats.append((np.where(rng.integers(0, 2, n), t - 3, t - 9), np.full(n, 4)))   # two values
    pats.append((t - rng.integers(1000, 1004, n), rng.integers(4000, 4003, n)))   # close ratios
    pats.append((t - rng.permutation(n) - 1, np.full(n, 777)))                 # all distinct
    half = np.arange(n) < n // 2                                               # tie group at the cut
    pats.append((np.where(half, t - 50, t - rng.integers(1, 40, n)), np.full(n, 50)))
    pats.append((t - rng.integers(0, 30, n), rng.integers(0, 3, n)))           # MRI in {0, 1, 2}
    pats.append((t - rng.integers(0, 20000, n), rng.integers(0, 5000, n)))     # random
    pats.append((np.full(n, t), np.zeros(n, int)))                             # dt = 0, MRI = 0
    pats.append((t - rng.integers(0, 3, n) * 700, np.ones(n, int)))            # x = 0, 700, 1400
    few = np.zeros(n, int)
    few[rng.choice(n, 7, replace=False)] = 3                                   # 7 scored, rest zero
    pats.append((np.full(n, t - 3), few))
    pats.append((t - np.arange(n) % 37, (np.arange(n) * 7) % 9))               # periodic structure
    assert len(pats) == HKV
    return pats


@pytest.mark.parametrize("flags", [3, 1, 2 | 16])
def test_eviction_on_hand_made_states(lazyev_lib, flags):
    rng = np.random.default_rng(100 + flags)
    eng = lazyev_lib.LazyEviction(1, 1, HKV, HKV, D, B, W, B, alpha=2.0, dtype=torch.float32,
                                  score_flags=flags)
    tag = torch.arange(B, dtype=torch.float32, device="cuda")
    eng.k_cache[0, 0, :, :B, :] = tag.view(1, -1, 1)             # row i holds i in every element
    eng.v_cache[0, 0, :, :B, :] = -tag.view(1, -1, 1)
    eng.init()
    q = torch.zeros((1, HKV, D), device="cuda")
    out = torch.empty_like(q)
    for step in range(1, T + 1):                                 # nothing reaches alpha = 2
        kv = torch.full((1, HKV, D), float(B + step - 1), device="cuda")
        eng.decode_step(0, step, q, kv, -kv, out)
    assert eng.stats()["len"][0] == B + W                        # also applies pending tracking
    pats = _patterns(rng)
    for h, (ts, mri) in enumerate(pats):
        eng.ts[0, 0, h, :B] = torch.from_numpy(ts.astype(np.int32)).cuda()
        eng.mri[0, 0, h, :B] = torch.from_numpy(mri.astype(np.int32)).cuda()
    torch.cuda.synchronize()
    assert eng.evict(0, T) == W
    st = eng.stats()
    assert st["len"][0] == B
    pos = eng.pos[0, 0].cpu().numpy()
    ts_g, mri_g = eng.ts[0, 0].cpu().numpy(), eng.mri[0, 0].cpu().numpy()
    k_g, v_g = eng.k_cache[0, 0].cpu().numpy(), eng.v_cache[0, 0].cpu().numpy()
    moved = 0
    for h, (ts, mri) in enumerate(pats):
        score = mri_centric_score(T, ts, mri, flags)
        keep = select_survivors(score, B - W)
        want = np.concatenate([keep, np.arange(B, B + W)])       # survivors, then the last W
        assert np.array_equal(pos[h, :B], want), ("survivor set", h)
        assert np.array_equal(ts_g[h, :B - W], ts[keep]) and np.array_equal(mri_g[h, :B - W], mri[keep])
        assert np.all(ts_g[h, B - W:B] == np.arange(1, W + 1)) and np.all(mri_g[h, B - W:B] == 0)
        assert np.array_equal(k_g[h, :B, 0], want) and np.array_equal(k_g[h, :B, D - 1], want)
        assert np.array_equal(v_g[h, :B, 5], -want.astype(np.float32))
        moved += int((want != np.arange(B)).sum())
    assert st["n_rows_moved"][0] == moved
