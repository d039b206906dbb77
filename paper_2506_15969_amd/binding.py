"""Thin ctypes binding of the C ABI in include/lazyev.h.

Argument marshalling only: every step of the decode path runs in the HIP library.  torch is
used for device memory and the stream.  Importing this module fails if the library has not
been built (python -m paper_2506_15969_amd.build); there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

# (LAZYEV_LIBRARY names another build of the same library in lib/, e.g. the instrumented
# liblazyev_timeline.so that bench.py --timeline measures with)
_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib",
                         os.path.basename(os.environ.get("LAZYEV_LIBRARY", "liblazyev.so")))
if not os.path.exists(_LIB_PATH):
    raise ImportError("liblazyev.so is not built: run `python -m paper_2506_15969_amd.build` "
                      "(expected at %s)" % _LIB_PATH)
lib = C.CDLL(_LIB_PATH)

OK, EINVAL, ECAPACITY, EWORKSPACE, EHIP, ENOMEM, ESCRATCH, EEXCHANGE = 0, -1, -2, -3, -4, -5, -6, -7
DTYPE_FP32, DTYPE_BF16 = 0, 1
SCORE_H1, SCORE_H2 = 1, 2
SCORE_H2_DECREASING = 16
SCORE_CURRENT_ATTENTION = 32
MAX_HIST_BINS = 8192
LDS_CANDIDATES = 8192


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("budget", C.c_int32),
                ("window", C.c_int32), ("prompt_len", C.c_int32), ("alpha", C.c_float),
                ("softmax_scale", C.c_float), ("dtype", C.c_int32), ("score_flags", C.c_int32),
                ("k_cache", C.c_void_p), ("v_cache", C.c_void_p), ("ts", C.c_void_p),
                ("mri", C.c_void_p), ("pos", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p)]


class Stats(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("len", C.POINTER(C.c_int32)),
                ("last_step", C.POINTER(C.c_int32)), ("n_evict_events", C.POINTER(C.c_int64)),
                ("n_evicted", C.POINTER(C.c_int64)), ("n_activations", C.POINTER(C.c_int64)),
                ("n_rows_moved", C.POINTER(C.c_int64))]


# what include/lazyev.h declares (the contract) ...
EXPORTS = ["lazyev_capacity", "lazyev_workspace_size", "lazyev_init", "lazyev_decode_step",
           "lazyev_prefill_track", "lazyev_prefill_track_seq", "lazyev_evict", "lazyev_evict_all",
           "lazyev_evict_static", "lazyev_stats", "lazyev_admit", "lazyev_retire",
           "lazyev_cached_before_step", "lazyev_mri_histogram", "lazyev_window_from_histogram",
           "lazyev_score_pairs", "lazyev_destroy", "lazyev_strerror", "lazyev_last_hip_error"]
# ... and include/lazyev_bench.h (knobs and the per-kernel timer in the same library; the plain
# streaming probes in liblazyev_bench.so, loaded by bench_lib() when somebody measures)
BENCH_EXPORTS = ["lazyev_set_chunk", "lazyev_set_target_blocks", "lazyev_set_variant", "lazyev_set_spin_ticks",
                 "lazyev_profile_arm", "lazyev_profile_read", "lazyev_log_words", "lazyev_log_peek"]
BENCH_LIB_EXPORTS = ["lazyev_stream_probe", "lazyev_stream_read_probe", "lazyev_event_overhead"]
_BENCH_LIB_PATH = os.path.join(os.path.dirname(_LIB_PATH), "liblazyev_bench.so")
_bench_lib = None


def bench_lib():
    """liblazyev_bench.so (plain streaming probes, event-pair cost), loaded on first use."""
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(_BENCH_LIB_PATH):
            raise ImportError("liblazyev_bench.so is not built: run `python -m paper_2506_15969_amd.build`")
        b = C.CDLL(_BENCH_LIB_PATH)
        b.lazyev_stream_probe.restype = C.c_int
        b.lazyev_stream_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p]
        b.lazyev_stream_read_probe.restype = C.c_int
        b.lazyev_stream_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p]
        b.lazyev_event_overhead.restype = C.c_int
        b.lazyev_event_overhead.argtypes = [C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        _bench_lib = b
    return _bench_lib


lib.lazyev_capacity.restype = C.c_int32
lib.lazyev_capacity.argtypes = [C.POINTER(Config)]
lib.lazyev_workspace_size.restype = C.c_size_t
lib.lazyev_workspace_size.argtypes = [C.POINTER(Config)]
lib.lazyev_init.restype = C.c_int
lib.lazyev_init.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
lib.lazyev_prefill_track.restype = C.c_int
lib.lazyev_prefill_track.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
lib.lazyev_prefill_track_seq.restype = C.c_int
lib.lazyev_prefill_track_seq.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
lib.lazyev_decode_step.restype = C.c_int
lib.lazyev_decode_step.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
lib.lazyev_evict.restype = C.c_int
lib.lazyev_evict.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
lib.lazyev_evict_all.restype = C.c_int
lib.lazyev_evict_all.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
lib.lazyev_evict_static.restype = C.c_int
lib.lazyev_evict_static.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
lib.lazyev_window_from_histogram.restype = C.c_int
lib.lazyev_window_from_histogram.argtypes = [C.POINTER(C.c_int64), C.c_int32, C.c_double, C.POINTER(C.c_int32)]
lib.lazyev_stats.restype = C.c_int
lib.lazyev_stats.argtypes = [C.c_void_p, C.POINTER(Stats)]
lib.lazyev_admit.restype = C.c_int
lib.lazyev_admit.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
lib.lazyev_retire.restype = C.c_int
lib.lazyev_cached_before_step.restype = C.c_int32
lib.lazyev_cached_before_step.argtypes = [C.c_int32] * 4
lib.lazyev_retire.argtypes = [C.c_void_p, C.c_int32]
lib.lazyev_mri_histogram.restype = C.c_int
lib.lazyev_mri_histogram.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int64)]
lib.lazyev_score_pairs.restype = C.c_int
lib.lazyev_score_pairs.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                   C.c_void_p]
lib.lazyev_set_chunk.restype = C.c_int
lib.lazyev_set_chunk.argtypes = [C.c_void_p, C.c_int32]
lib.lazyev_set_target_blocks.restype = C.c_int
lib.lazyev_set_target_blocks.argtypes = [C.c_void_p, C.c_int32]
lib.lazyev_set_variant.restype = C.c_int
lib.lazyev_set_variant.argtypes = [C.c_void_p, C.c_int32]
lib.lazyev_set_spin_ticks.restype = C.c_int
lib.lazyev_set_spin_ticks.argtypes = [C.c_void_p, C.c_uint32]
lib.lazyev_profile_arm.restype = C.c_int
lib.lazyev_profile_arm.argtypes = [C.c_void_p, C.c_int32]
lib.lazyev_log_words.restype = C.c_int32
lib.lazyev_log_words.argtypes = [C.c_void_p]
lib.lazyev_log_peek.restype = C.c_int
lib.lazyev_log_peek.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_uint32), C.POINTER(C.c_int32)]
lib.lazyev_profile_read.restype = C.c_int
lib.lazyev_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
lib.lazyev_destroy.restype = None
lib.lazyev_destroy.argtypes = [C.c_void_p]
lib.lazyev_strerror.restype = C.c_char_p
lib.lazyev_strerror.argtypes = [C.c_int]
lib.lazyev_last_hip_error.restype = C.c_int
lib.lazyev_last_hip_error.argtypes = [C.c_void_p]


class LazyevError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (code %d)" % (where, lib.lazyev_strerror(code).decode(), code))


def _check(code: int, where: str):
    if code != OK:
        raise LazyevError(code, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def score_pairs(delta_t: torch.Tensor, mri: torch.Tensor, score_flags: int = SCORE_H1 | SCORE_H2):
    """lazyev_score_pairs on int32 device tensors; returns a float64 device tensor."""
    assert delta_t.is_cuda and mri.is_cuda and delta_t.dtype == torch.int32 and mri.dtype == torch.int32
    delta_t, mri = delta_t.contiguous(), mri.contiguous()
    out = torch.empty(delta_t.numel(), dtype=torch.float64, device=delta_t.device)
    stream = torch.cuda.current_stream(delta_t.device).cuda_stream
    _check(lib.lazyev_score_pairs(_ptr(delta_t), _ptr(mri), _ptr(out), delta_t.numel(),
                                  score_flags, C.c_void_p(stream)), "lazyev_score_pairs")
    return out.view(delta_t.shape)


def window_from_histogram(hist, quantile: float = 0.8) -> int:
    """lazyev_window_from_histogram on a sequence of counts (host only)."""
    n = len(hist)
    arr = (C.c_int64 * n)(*[int(x) for x in hist])
    w = C.c_int32(0)
    _check(lib.lazyev_window_from_histogram(arr, n, quantile, C.byref(w)), "lazyev_window_from_histogram")
    return w.value


class LazyEviction:
    """Owns the device buffers (as torch tensors) and a library context for them.

    k_cache / v_cache [L,S,Hkv,C,d], ts / mri / pos [L,S,Hkv,C] are attributes; fill the prompt
    rows with `load_prompt` (or write them directly) BEFORE `init()`.
    """

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, budget, window,
                 prompt_len, alpha, dtype=torch.bfloat16, softmax_scale=0.0,
                 score_flags=SCORE_H1 | SCORE_H2, device="cuda:0", stream=None):
        if not torch.cuda.is_available():
            raise RuntimeError("lazyev needs a GPU: no CPU fallback exists")
        self.device = torch.device(device)
        self.dtype = dtype
        self.cfg = Config(n_layers=n_layers, batch=batch, n_q_heads=n_q_heads,
                          n_kv_heads=n_kv_heads, head_dim=head_dim, budget=budget, window=window,
                          prompt_len=prompt_len, alpha=alpha, softmax_scale=softmax_scale,
                          dtype=DTYPE_FP32 if dtype == torch.float32 else DTYPE_BF16,
                          score_flags=score_flags)
        cap = lib.lazyev_capacity(C.byref(self.cfg))
        if cap <= 0:
            raise LazyevError(EINVAL, "lazyev_capacity")
        self.capacity = cap
        L, S, H, d = n_layers, batch, n_kv_heads, head_dim
        self.k_cache = torch.zeros((L, S, H, cap, d), dtype=dtype, device=self.device)
        self.v_cache = torch.zeros((L, S, H, cap, d), dtype=dtype, device=self.device)
        self.ts = torch.zeros((L, S, H, cap), dtype=torch.int32, device=self.device)
        self.mri = torch.zeros((L, S, H, cap), dtype=torch.int32, device=self.device)
        self.pos = torch.zeros((L, S, H, cap), dtype=torch.int32, device=self.device)
        ws_bytes = lib.lazyev_workspace_size(C.byref(self.cfg))
        self.workspace = torch.zeros(ws_bytes, dtype=torch.uint8, device=self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.cfg.k_cache, self.cfg.v_cache = self.k_cache.data_ptr(), self.v_cache.data_ptr()
        self.cfg.ts, self.cfg.mri, self.cfg.pos = (self.ts.data_ptr(), self.mri.data_ptr(),
                                                  self.pos.data_ptr())
        self.cfg.workspace, self.cfg.workspace_bytes = self.workspace.data_ptr(), ws_bytes
        self.cfg.stream = self.stream.cuda_stream
        self._ctx = C.c_void_p()

    def load_prompt(self, layer: int, k: torch.Tensor, v: torch.Tensor):
        """k, v [S,Hkv,P,d] -> entries 0..P-1 of the layer."""
        P = self.cfg.prompt_len
        self.k_cache[layer, :, :, :P].copy_(k)
        self.v_cache[layer, :, :, :P].copy_(v)

    def init(self):
        if self._ctx:
            lib.lazyev_destroy(self._ctx)
            self._ctx = C.c_void_p()
        _check(lib.lazyev_init(C.byref(self.cfg), C.byref(self._ctx)), "lazyev_init")
        return self

    def set_chunk(self, chunk: int):
        _check(lib.lazyev_set_chunk(self._ctx, chunk), "lazyev_set_chunk")

    def decode_step(self, layer, t, q, k_new, v_new, out, p_out=None, p_override=None):
        code = lib.lazyev_decode_step(self._ctx, layer, t, q.data_ptr(), k_new.data_ptr(),
                                      v_new.data_ptr(), out.data_ptr(), _ptr(p_out),
                                      _ptr(p_override))
        if code != OK:
            raise LazyevError(code, "lazyev_decode_step")

    def prefill_track(self, layer, q_prompt, p_out=None, p_override=None):
        """lazyev_prefill_track.  q_prompt [S,P,Hq,d]; p_out / p_override [S,Hq,P,P] fp32."""
        code = lib.lazyev_prefill_track(self._ctx, layer, q_prompt.data_ptr(), _ptr(p_out), _ptr(p_override))
        if code != OK:
            raise LazyevError(code, "lazyev_prefill_track")

    def prefill_track_seq(self, layer, seq, q_prompt, p_out=None, p_override=None):
        """lazyev_prefill_track_seq.  q_prompt [P,Hq,d]; p_out / p_override [Hq,P,P] fp32."""
        code = lib.lazyev_prefill_track_seq(self._ctx, layer, seq, q_prompt.data_ptr(), _ptr(p_out),
                                            _ptr(p_override))
        if code != OK:
            raise LazyevError(code, "lazyev_prefill_track_seq")

    def evict(self, layer, t) -> int:
        n = C.c_int32(0)
        code = lib.lazyev_evict(self._ctx, layer, t, C.byref(n))
        if code != OK:
            raise LazyevError(code, "lazyev_evict")
        return n.value

    def evict_static(self, layer, t) -> int:
        """lazyev_evict_static: lazyev_evict with the gather list in the library's own static
        device array instead of the workspace."""
        n = C.c_int32(0)
        code = lib.lazyev_evict_static(self._ctx, layer, t, C.byref(n))
        if code != OK:
            raise LazyevError(code, "lazyev_evict_static")
        return n.value

    def evict_all(self, t) -> int:
        """lazyev_evict_all: the eviction check of every layer after step t."""
        n = C.c_int32(0)
        code = lib.lazyev_evict_all(self._ctx, t, C.byref(n))
        if code != OK:
            raise LazyevError(code, "lazyev_evict_all")
        return n.value

    def stats(self) -> dict:
        L = self.cfg.n_layers
        a32 = lambda: (C.c_int32 * L)()
        a64 = lambda: (C.c_int64 * L)()
        bufs = dict(len=a32(), last_step=a32(), n_evict_events=a64(), n_evicted=a64(),
                    n_activations=a64(), n_rows_moved=a64())
        st = Stats(n_layers=L, **{k: C.cast(v, C.POINTER(C.c_int32 if k in ("len", "last_step")
                                                         else C.c_int64)) for k, v in bufs.items()})
        _check(lib.lazyev_stats(self._ctx, C.byref(st)), "lazyev_stats")
        return {k: list(v) for k, v in bufs.items()}

    def admit(self, seq: int, prompt_len: int, t0: int, k=None, v=None):
        """lazyev_admit.  k, v [L,Hkv,prompt_len,d] (optional): the prompt rows, copied into the
        slot's units of every layer first."""
        if k is not None:
            self.k_cache[:, seq, :, :prompt_len].copy_(k)
            self.v_cache[:, seq, :, :prompt_len].copy_(v)
        _check(lib.lazyev_admit(self._ctx, seq, prompt_len, t0), "lazyev_admit")

    def retire(self, seq: int):
        _check(lib.lazyev_retire(self._ctx, seq), "lazyev_retire")

    def mri_histogram(self, layer: int = -1, n_bins: int = MAX_HIST_BINS):
        """lazyev_mri_histogram: counts of cached entries by MRI (last bin: MRI >= n_bins - 1)
        over the units of `layer` (-1: all layers), as a list of ints."""
        hist = (C.c_int64 * n_bins)()
        _check(lib.lazyev_mri_histogram(self._ctx, layer, n_bins, hist), "lazyev_mri_histogram")
        return list(hist)

    def set_target_blocks(self, n_blocks: int):
        _check(lib.lazyev_set_target_blocks(self._ctx, n_blocks), "lazyev_set_target_blocks")

    def set_variant(self, variant: int):
        _check(lib.lazyev_set_variant(self._ctx, variant), "lazyev_set_variant")

    def set_spin_ticks(self, ticks: int):
        _check(lib.lazyev_set_spin_ticks(self._ctx, ticks), "lazyev_set_spin_ticks")

    def log_peek(self, layer: int, units, back: int = 0):
        """lazyev_log_peek for the (sequence, kv_head) pairs in `units`: (step, bool array
        [len(units), 32 * log_words]) of a logged call, or None if the layer has no such call in
        its activation log."""
        import numpy as np
        words = lib.lazyev_log_words(self._ctx)
        if words <= 0:
            return None
        buf = (C.c_uint32 * words)()
        t = C.c_int32(0)
        rows = []
        for (seq, kvh) in units:
            if lib.lazyev_log_peek(self._ctx, layer, back, seq * self.cfg.n_kv_heads + kvh, buf, C.byref(t)) != 0:
                return None
            a = np.frombuffer(buf, dtype=np.uint32).copy()
            rows.append(np.unpackbits(a.view(np.uint8), bitorder="little").astype(bool))
        return t.value, np.stack(rows)

    def profile_arm(self, n_calls: int):
        _check(lib.lazyev_profile_arm(self._ctx, n_calls), "lazyev_profile_arm")

    def profile_read(self) -> dict:
        """{kernel: (total ms, launches)} of the armed calls since the last read."""
        ms, n = (C.c_double * 4)(), (C.c_int64 * 4)()
        _check(lib.lazyev_profile_read(self._ctx, ms, n), "lazyev_profile_read")
        names = ("split", "combine", "select", "move")
        return {k: (ms[i], n[i]) for i, k in enumerate(names)}

    def close(self):
        if self._ctx:
            lib.lazyev_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
