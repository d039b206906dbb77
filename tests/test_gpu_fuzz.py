"""Random call sequences.  Engine A is driven plainly, exports its weights at every step and is
followed by oracle units that threshold those weights (exact comparison).  Engine B gets the
same inputs but a random mix of what must not change any result: weights exported or not
(immediate or deferred tracking), lazyev_stats / lazyev_mri_histogram in between, evictions
asked for when none is due, the block split and the format the logits are kept in for the
deferred tracking changed between calls, layers advanced in random order.  B's caches, statistics and outputs must equal A's bit for bit."""
import numpy as np
import pytest
import torch

from oracle.lazyev_oracle import OracleUnit

pytestmark = pytest.mark.gpu


def _case(rng):
    hkv = int(rng.integers(1, 3))
    g = int(rng.choice([1, 2, 4, 5, 7, 8]))
    b = int(rng.integers(8, 70))
    return dict(L=int(rng.integers(1, 4)), S=int(rng.integers(1, 4)), HKV=hkv, G=g,
                P=int(rng.integers(0, 90)), B=b, W=int(rng.integers(1, min(b, 17))),
                steps=int(rng.integers(30, 80)), alpha=float(rng.choice([0.01, 0.03, 0.1])))


@pytest.mark.parametrize("seed", range(8))
def test_random_call_sequences(lazyev_lib, seed):
    rng = np.random.default_rng(1000 + seed)
    c = _case(rng)
    L, S, HKV, G, P, B, W = (c[k] for k in ("L", "S", "HKV", "G", "P", "B", "W"))
    HQ, D = HKV * G, 128
    print("\ncase", seed, c, flush=True)
    gen = torch.Generator().manual_seed(seed)
    rnd = lambda *shape: torch.randn(shape, generator=gen).to(torch.bfloat16)   # noqa: E731
    kp, vp = rnd(L, S, HKV, P, D), rnd(L, S, HKV, P, D)
    engines = []
    for _ in range(2):
        e = lazyev_lib.LazyEviction(L, S, HQ, HKV, D, B, W, P, c["alpha"], dtype=torch.bfloat16)
        for l in range(L):
            if P:
                e.load_prompt(l, kp[l].cuda(), vp[l].cuda())
        engines.append(e.init())
    A, Bn = engines
    orc = {(l, s, h): OracleUnit(kp[l, s, h].double().numpy(), vp[l, s, h].double().numpy(), G, B, W,
                                 c["alpha"]) for l in range(L) for s in range(S) for h in range(HKV)}
    cap = A.capacity
    out_a = torch.empty((S, HQ, D), dtype=torch.bfloat16, device="cuda")
    out_b = torch.empty_like(out_a)
    p_a = torch.zeros((S, HQ, cap), dtype=torch.float32, device="cuda")
    p_b = torch.zeros_like(p_a)
    ins = [[(rnd(S, HQ, D).cuda(), rnd(S, HKV, D).cuda(), rnd(S, HKV, D).cuda()) for _ in range(L)]
           for _ in range(c["steps"])]
    # A: plain order, followed by the oracle
    for t in range(1, c["steps"] + 1):
        for l in range(L):
            q, kn, vn = ins[t - 1][l]
            A.decode_step(l, t, q, kn, vn, out_a, p_out=p_a)
            pg = p_a.cpu().numpy()
            qd, kd, vd = q.double().cpu().numpy(), kn.double().cpu().numpy(), vn.double().cpu().numpy()
            for s in range(S):
                for h in range(HKV):
                    u = orc[(l, s, h)]
                    rows = slice(h * G, (h + 1) * G)
                    u.decode_step(t, qd[s, rows], kd[s, h], vd[s, h],
                                  p_override=np.ascontiguousarray(pg[s, rows, :len(u) + 1]))
            n_ev = A.evict(l, t)
            for s in range(S):
                for h in range(HKV):
                    assert len(orc[(l, s, h)].evict(t)) == n_ev
    A.stats()
    for (l, s, h), u in orc.items():
        n = len(u)
        assert np.array_equal(A.pos[l, s, h, :n].cpu().numpy(), u.pos)
        assert np.array_equal(A.ts[l, s, h, :n].cpu().numpy(), u.TS)
        assert np.array_equal(A.mri[l, s, h, :n].cpu().numpy(), u.MRI)
        assert np.array_equal(A.k_cache[l, s, h, :n].double().cpu().numpy(), u.K)
    # B: the same steps, layers advanced in random order, with harmless extras thrown in
    done = [0] * L
    outs_b = {}
    while min(done) < c["steps"]:
        l = int(rng.choice([i for i in range(L) if done[i] < c["steps"]]))
        t = done[l] + 1
        q, kn, vn = ins[t - 1][l]
        if rng.random() < 0.3:
            Bn.set_target_blocks(int(rng.choice([1, S * HKV, 4 * S * HKV, 40 * S * HKV, 512])))
        if rng.random() < 0.3:                            # every logit kept for the tracking, or candidate lists
            Bn.set_variant(int(rng.choice([5, 6])))
        Bn.decode_step(l, t, q, kn, vn, out_b, p_out=p_b if rng.random() < 0.3 else None)
        outs_b[(l, t)] = out_b.clone()
        r = rng.random()
        if r < 0.15:
            Bn.stats()
        elif r < 0.25:
            Bn.mri_histogram(int(rng.integers(-1, L)), 16)
        Bn.evict(l, t)
        if rng.random() < 0.2:
            assert Bn.evict(l, t) == 0                    # a second request finds nothing due
        done[l] = t
    st_a, st_b = A.stats(), Bn.stats()
    assert st_a == st_b
    for name in ("k_cache", "v_cache", "ts", "mri", "pos"):
        assert torch.equal(getattr(A, name), getattr(Bn, name)), name
    # outputs: a third engine in plain order without exported weights, against what B produced
    A2 = lazyev_lib.LazyEviction(L, S, HQ, HKV, D, B, W, P, c["alpha"], dtype=torch.bfloat16)
    for l in range(L):
        if P:
            A2.load_prompt(l, kp[l].cuda(), vp[l].cuda())
    A2.init()
    for t in range(1, c["steps"] + 1):
        for l in range(L):
            q, kn, vn = ins[t - 1][l]
            A2.decode_step(l, t, q, kn, vn, out_a)
            A2.evict(l, t)
            # B ran with other block splits: its rows may differ in the order of the fp32 sums
            diff = (out_a.float() - outs_b[(l, t)].float()).abs().max().item()
            assert diff <= 2e-2, (l, t, diff)
