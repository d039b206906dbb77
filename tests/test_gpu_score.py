"""The device's Eq. 3 score against the oracle's, bit for bit."""
import numpy as np
import pytest
import torch

from oracle.lazyev_oracle import mri_centric_score

pytestmark = pytest.mark.gpu


def _check(binding, dt, mri, flags=3):
    d = torch.from_numpy(dt.astype(np.int32)).cuda()
    m = torch.from_numpy(mri.astype(np.int32)).cuda()
    got = binding.score_pairs(d, m, flags).cpu().numpy()
    ref = mri_centric_score(0, -dt.astype(np.int64), mri, flags)
    assert np.array_equal(got.view(np.uint64), ref.view(np.uint64))


def test_exhaustive_grid(lazyev_lib):
    n = 4097
    mri = np.arange(n)
    for lo in range(0, n, 512):
        dt = np.arange(lo, min(n, lo + 512))
        D, M = np.meshgrid(dt, mri, indexing="ij")
        _check(lazyev_lib, D.ravel(), M.ravel())


def test_reflected_h2_grid(lazyev_lib):
    mri = np.arange(0, 40000)
    for dt in (0, 1, 63, 5000):
        _check(lazyev_lib, np.full_like(mri, dt), mri, 3 | 16)
    _check(lazyev_lib, np.zeros_like(mri), mri, 2 | 16)


def test_random_pairs_and_flags(lazyev_lib):
    rng = np.random.default_rng(0)
    dt = rng.integers(0, 32769, 1_000_000)
    mri = rng.integers(0, 32769, 1_000_000)
    for flags in (3, 1, 2, 0, 2 | 16, 3 | 16, 1 | 16):
        _check(lazyev_lib, dt, mri, flags)
    # very stale entries: x = dt/mri beyond the cut-off of the exponential
    _check(lazyev_lib, np.array([2_000_000_000, 700, 699, 1399, 1400]), np.array([1, 1, 1, 2, 2]))
