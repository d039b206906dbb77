"""The synthetic input generator: stateless, sliceable, and the same on every device."""
import numpy as np
import pytest
import torch

from paper_2506_15969_amd.workload import CONFIGS, Workload


def test_slices_equal_the_full_batch():
    w = Workload(CONFIGS["cfg3"])
    G = w.cfg.group
    qf, kf, vf = w.step_inputs(2, 300, 303)
    q, k, v = w.step_inputs(2, 301, 302, seq=[4, 9], kv_head=[3, 0])
    heads = [3 * G + g for g in range(G)] + list(range(G))
    assert torch.equal(qf[1:2][:, [4, 9]][:, :, heads], q)
    assert torch.equal(kf[1:2][:, [4, 9]][:, :, [3, 0]], k)
    assert torch.equal(vf[1:2][:, [4, 9]][:, :, [3, 0]], v)
    # the row generated at step t is the row "by position" P+t-1
    K, V = w.kv_rows(2, [w.cfg.prompt_len + 301 - 1])
    assert torch.equal(K[:, :, 0], kf[1]) and torch.equal(V[:, :, 0], vf[1])


def test_prompt_queries_slice_and_read_the_first_keys_periodically():
    cfg = CONFIGS["cfg2"].scaled(batch=3, prompt_len=100, steps=4, budget=200, window=32)
    w = Workload(cfg)
    G, d = cfg.group, cfg.head_dim
    qa = w.prompt_queries(0)                                      # [S, P, Hq, d]
    assert qa.shape == (3, 100, cfg.n_q_heads, d)
    q1 = w.prompt_queries(0, seq=[2, 0], kv_head=[3, 1])
    heads = [3 * G + g for g in range(G)] + [G + g for g in range(G)]
    assert torch.equal(qa[[2, 0]][:, :, heads], q1)
    # position i >= 32 reads key (5 i) mod 32 on head i mod G: its logit dominates the row
    k, _ = w.prompt_kv(0, seq=[1], kv_head=[2])
    k = k[0, 0].double()
    for i in (32, 57, 99):
        s = (qa[1, i, 2 * G + i % G].double() @ k[:i + 1].T) / d ** 0.5
        assert int(s.argmax()) == (5 * i) % 32 and float(s.max()) > 30.0
    # the same key again 32 positions later, on another head
    assert (5 * 57) % 32 == (5 * 89) % 32


def test_values_look_standard_normal_and_differ_across_streams():
    w = Workload(CONFIGS["cfg2"])
    K, V = w.prompt_kv(0)
    for x in (K.float(), V.float()):
        assert abs(x.mean()) < 0.01 and abs(x.std() - 1) < 0.01 and x.abs().max() < 4.95
    assert not torch.equal(K, V)
    K1, _ = Workload(CONFIGS["cfg2"].scaled(seed=99)).prompt_kv(0)
    assert not torch.equal(K, K1)


def test_planted_key_dominates_its_firing_step():
    w = Workload(CONFIGS["cfg1"])
    c = w.cfg
    ev_t, ev_j = w.firings(1, c.steps + 1)
    assert len(w.planted) == 8 and set(ev_j) == set(w.planted.tolist())
    assert np.all((w.period >= 40) & (w.period <= 90))
    K, _ = w.prompt_kv(0)
    t, j = int(ev_t[3]), int(ev_j[3])
    q, _, _ = w.step_inputs(0, t, t + 1)
    g = j % c.group                                     # G = 1 here: every head is boosted
    logits = (K[0, 0].double() @ q[0, 0, g].double()) / np.sqrt(c.head_dim)
    assert int(logits.argmax()) == j and logits[j] > 20


def test_sink_boost_raises_sink_logits():
    w = Workload(CONFIGS["cfg3"])
    K, _ = w.prompt_kv(0, seq=[0], kv_head=[0])
    q, _, _ = w.step_inputs(0, 10, 40, seq=[0], kv_head=[0])
    logits = torch.einsum("nhd,pd->nhp", q[:, 0].double(), K[0, 0].double()) / np.sqrt(128)
    assert logits[:, :, :4].mean() > 4.0 and abs(logits[:, :, 8:].mean()) < 0.3


@pytest.mark.gpu
def test_gpu_generation_is_bit_identical_to_cpu():
    for name in ("cfg1", "cfg3", "cfg4"):
        w = Workload(CONFIGS[name])
        t0 = 2000 if name != "cfg1" else 50
        a = w.step_inputs(0, t0, t0 + 8)
        b = w.step_inputs(0, t0, t0 + 8, device="cuda")
        for x, y in zip(a, b):
            assert torch.equal(x, y.cpu())
        ka, va = w.prompt_kv(0)
        kb, vb = w.prompt_kv(0, device="cuda")
        assert torch.equal(ka, kb.cpu()) and torch.equal(va, vb.cpu())
        assert torch.equal(w.prompt_queries(0), w.prompt_queries(0, device="cuda").cpu())
