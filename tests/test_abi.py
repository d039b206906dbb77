"""The C-ABI library loads, exports every declared symbol and rejects bad arguments on the host
(no GPU work is launched here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _good(b):
    return b.Config(n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, budget=64,
                    window=8, prompt_len=16, alpha=0.01, softmax_scale=0.0, dtype=b.DTYPE_BF16,
                    score_flags=3)


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)           # declarations, not prose
    return set(re.findall(r"\b(lazyev_[a-z_]+)\s*\(", header))


def test_every_declared_symbol_is_exported(lazyev_lib):
    """include/lazyev.h is the contract of the path; include/lazyev_bench.h holds the knobs and
    the per-kernel timer (same library) and the streaming probes (liblazyev_bench.so)."""
    declared = _declared("lazyev.h")
    assert declared == set(lazyev_lib.EXPORTS)
    for name in declared:
        assert hasattr(lazyev_lib.lib, name)
    bench = _declared("lazyev_bench.h")
    assert bench == set(lazyev_lib.BENCH_EXPORTS) | set(lazyev_lib.BENCH_LIB_EXPORTS)
    for name in lazyev_lib.BENCH_EXPORTS:
        assert hasattr(lazyev_lib.lib, name)
    probes = lazyev_lib.bench_lib()
    for name in lazyev_lib.BENCH_LIB_EXPORTS:
        assert hasattr(probes, name)
        assert not hasattr(lazyev_lib.lib, name), "the path's library holds no measuring kernels"


def test_struct_layout_matches_header(lazyev_lib):
    # 12 four-byte fields, 6 pointers, a size_t, a pointer
    assert C.sizeof(lazyev_lib.Config) == 12 * 4 + 8 * 8
    assert C.sizeof(lazyev_lib.Stats) == 8 + 6 * 8


def test_capacity_and_workspace(lazyev_lib):
    b = lazyev_lib
    cfg = _good(b)
    assert b.lib.lazyev_capacity(C.byref(cfg)) == 64 + 8
    assert b.lib.lazyev_workspace_size(C.byref(cfg)) > 0
    cfg.prompt_len = 100
    assert b.lib.lazyev_capacity(C.byref(cfg)) == 108


@pytest.mark.parametrize("field,value", [("n_q_heads", 7), ("head_dim", 96), ("window", 0),
                                         ("budget", 8), ("dtype", 5), ("score_flags", 8), ("score_flags", 64),
                                         ("n_layers", 0), ("alpha", float("nan")),
                                         ("n_q_heads", 32), ("prompt_len", -1),
                                         ("budget", 2_000_000)])
def test_invalid_configs_are_rejected(lazyev_lib, field, value):
    b = lazyev_lib
    cfg = _good(b)
    setattr(cfg, field, value)
    assert b.lib.lazyev_capacity(C.byref(cfg)) == 0
    assert b.lib.lazyev_workspace_size(C.byref(cfg)) == 0
    ctx = C.c_void_p()
    assert b.lib.lazyev_init(C.byref(cfg), C.byref(ctx)) == b.EINVAL and not ctx


def test_init_needs_buffers_and_workspace(lazyev_lib):
    b = lazyev_lib
    cfg = _good(b)
    ctx = C.c_void_p()
    assert b.lib.lazyev_init(C.byref(cfg), C.byref(ctx)) == b.EINVAL      # null caches
    for f in ("k_cache", "v_cache", "ts", "mri", "pos"):
        setattr(cfg, f, 256)
    assert b.lib.lazyev_init(C.byref(cfg), C.byref(ctx)) == b.EWORKSPACE  # no workspace
    cfg.workspace, cfg.workspace_bytes = 256, 16
    assert b.lib.lazyev_init(C.byref(cfg), C.byref(ctx)) == b.EWORKSPACE  # too small
    assert b.lib.lazyev_init(C.byref(cfg), None) == b.EINVAL


def test_null_context_calls(lazyev_lib):
    b = lazyev_lib
    assert b.lib.lazyev_decode_step(None, 0, 1, 1, 1, 1, 1, None, None) == b.EINVAL
    assert b.lib.lazyev_evict(None, 0, 1, None) == b.EINVAL and b.lib.lazyev_evict_static(None, 0, 1, None) == b.EINVAL
    assert b.lib.lazyev_evict_all(None, 1, None) == b.EINVAL
    assert b.lib.lazyev_stats(None, None) == b.EINVAL
    assert b.lib.lazyev_set_chunk(None, 128) == b.EINVAL and b.lib.lazyev_set_variant(None, 4) == b.EINVAL
    assert b.lib.lazyev_prefill_track(None, 0, 1, None, None) == b.EINVAL
    assert b.lib.lazyev_prefill_track_seq(None, 0, 0, 1, None, None) == b.EINVAL
    assert b.lib.lazyev_admit(None, 0, 1, 0) == b.EINVAL and b.lib.lazyev_retire(None, 0) == b.EINVAL
    b.lib.lazyev_destroy(None)
    assert b.lib.lazyev_last_hip_error(None) == 0
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert len(b.lib.lazyev_strerror(code)) > 0


def test_window_from_histogram_is_the_quantile(lazyev_lib):
    """Host logic: the window taken from an MRI histogram (Sec. 4, "Observation Window") equals
    the quantile of the raw values as the oracle and numpy define it."""
    import numpy as np
    from oracle.lazyev_oracle import mri_histogram, window_from_mri
    rng = np.random.default_rng(5)
    for n in (1, 10, 1000, 5003):
        mri = np.where(rng.random(n) < 0.5, 0, rng.geometric(0.01, n))
        hist = mri_histogram(mri, 4096).tolist()
        for q in (0.5, 0.8, 0.99, 1.0):
            assert lazyev_lib.window_from_histogram(hist, q) == window_from_mri(mri, q)
    assert lazyev_lib.window_from_histogram([5, 0, 0, 0]) == 0
    assert lazyev_lib.window_from_histogram([0, 0, 3, 1], 0.8) == 3
    assert lazyev_lib.window_from_histogram([0, 4, 1], 0.8) == 1          # 4 of 5 is exactly 80 %
    w = C.c_int32(-7)
    f = lazyev_lib.lib.lazyev_window_from_histogram
    one = (C.c_int64 * 3)(1, 2, 3)
    assert f(None, 3, 0.8, C.byref(w)) == lazyev_lib.EINVAL and f(one, 3, 0.8, None) == lazyev_lib.EINVAL
    assert f(one, 1, 0.8, C.byref(w)) == lazyev_lib.EINVAL and f(one, 3, 0.0, C.byref(w)) == lazyev_lib.EINVAL
    assert f(one, 3, 1.5, C.byref(w)) == lazyev_lib.EINVAL
    assert f((C.c_int64 * 3)(1, -2, 3), 3, 0.8, C.byref(w)) == lazyev_lib.EINVAL
    assert lazyev_lib.lib.lazyev_mri_histogram(None, 0, 16, None) == lazyev_lib.EINVAL


def test_current_attention_ranking_needs_the_bf16_shape(lazyev_lib):
    b = lazyev_lib
    cfg = _good(b)
    cfg.score_flags = b.SCORE_CURRENT_ATTENTION
    assert b.lib.lazyev_capacity(C.byref(cfg)) == 72                   # bf16, head_dim 128: accepted
    cfg.dtype = b.DTYPE_FP32
    assert b.lib.lazyev_capacity(C.byref(cfg)) == 0
    cfg.dtype, cfg.head_dim = b.DTYPE_BF16, 64
    assert b.lib.lazyev_capacity(C.byref(cfg)) == 0


def test_cache_length_formula_against_a_simulation(lazyev_lib):
    """Host logic shared with the kernels: the closed form for a sequence's cache length must
    equal stepping the schedule of Sec. 4 (append; after a step that is a multiple of W, cut to
    B if more than B are cached), for prompts shorter and longer than the budget."""
    import random
    rng = random.Random(9)
    f = lazyev_lib.lib.lazyev_cached_before_step
    for _ in range(400):
        B = rng.randint(2, 70)
        W = rng.randint(1, B - 1)
        P = rng.randint(0, 120)
        n = P
        for tau in range(1, 200):
            assert f(P, tau, B, W) == n, (P, B, W, tau)
            n += 1
            if tau % W == 0 and n > B:
                n = B
    assert f(-1, 1, 8, 2) == -1 and f(4, 0, 8, 2) == -1 and f(4, 1, 2, 2) == -1


def test_benchmark_refuses_more_than_one_gpu():
    """The path has no cross-GPU part: bench.py --gpus 2 says so and exits before touching a GPU."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
