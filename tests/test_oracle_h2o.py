"""Pins of the oracle's H2O policy (Section 3 "Comparison systems"; Appendix A.1 "Baseline
Settings") against a hand-worked example, a pure-Python replay and the policy's invariants."""
import math

import numpy as np

import oracle
from test_oracle_pins import bits, val, rand_bits, brute_attention


def _empty(B, Hkv, D):
    z = np.zeros((B, Hkv, 0, D), dtype=np.uint16)
    return z, z.copy(), np.zeros((B, Hkv, 0), np.float32), np.zeros((B, Hkv, 0), np.int64), [0] * B


def test_uniform_attention_worked_example():
    """Equal keys: a step over n cached tokens gives each 1/n.  Budget 3, one recent token, empty
    start.  Totals after step t (n = t + 1 tokens until the budget is hit, 4 from then on):
      t=0: {0: 1}            t=1: {0: 1.5, 1: .5}          t=2: {0: 11/6, 1: 5/6, 2: 1/3}
      t=3: four tokens, 1/4 each: {0: 25/12, 1: 13/12, 2: 7/12, 3: 1/4}; token 3 is recent, so the
           lowest old one, 2, goes.  t=4: {0: 7/3, 1: 4/3, 3: 1/2, 4: 1/4}: 3 goes.  t=5: 4 goes.
    The output is the mean of the cached value rows."""
    T, D = 6, 2
    k0, v0, tot0, pos0, n0 = _empty(1, 1, D)
    nk = bits(np.ones((T, 1, 1, D)))
    vrows = np.array([[float(t + 1), float(-t)] for t in range(T)])
    nv = bits(vrows.reshape(T, 1, 1, D))
    q = bits(np.full((T, 1, 1, D), 0.75))
    res = oracle.h2o_decode_loop(q, k0, v0, tot0, pos0, n0, nk, nv, 0.5, budget=3, recent=1)
    assert res["dropped"][:, 0, 0].tolist() == [-1, -1, -1, 2, 3, 4]
    final = res["final"][0][0]
    assert sorted(final) == [0, 1, 5]
    want0 = 1 + 1 / 2 + 1 / 3 + 3 * (1 / 4)
    want1 = 1 / 2 + 1 / 3 + 3 * (1 / 4)
    assert abs(final[0] - want0) < 1e-6 and abs(final[1] - want1) < 1e-6 and abs(final[5] - 0.25) < 1e-7
    kept = [[0], [0, 1], [0, 1, 2], [0, 1, 2, 3], [0, 1, 3, 4], [0, 1, 4, 5]]
    for t in range(T):
        assert np.allclose(val(res["outs"][t, 0, 0]), vrows[kept[t]].mean(axis=0), rtol=2 ** -8)


def _replay(q, k0, v0, tot0, pos0, n0, nk, nv, scale, budget, recent, G):
    """The same policy in pure-Python floats, one (sequence, KV head) at a time."""
    T, B, Hq, D = q.shape
    Hkv = k0.shape[1]
    drops = np.full((T, B, Hkv), -1, dtype=np.int64)
    outs = np.zeros((T, B, Hq, D))
    finals = {}
    for b in range(B):
        for g in range(Hkv):
            toks = {int(pos0[b, g, j]): [val(k0[b, g, j]).tolist(), val(v0[b, g, j]).tolist(), float(tot0[b, g, j])]
                    for j in range(n0[b])}
            p = max(toks, default=-1)
            for t in range(T):
                p += 1
                toks[p] = [val(nk[t, b, g]).tolist(), val(nv[t, b, g]).tolist(), 0.0]
                order = sorted(toks)
                best = [0.0] * len(order)
                for h in range(g * G, (g + 1) * G):
                    o, a, _ = brute_attention(val(q[t, b, h]).tolist(), [toks[x][0] for x in order],
                                              [toks[x][1] for x in order], scale)
                    outs[t, b, h] = o
                    best = [max(u, float(np.float32(w))) for u, w in zip(best, a)]
                for x, w in zip(order, best):
                    toks[x][2] = float(np.float32(np.float32(toks[x][2]) + np.float32(w)))
                if len(toks) > budget:
                    old = [x for x in order if x <= p - recent]
                    victim = min(old, key=lambda x: (toks[x][2], x))
                    drops[t, b, g] = victim
                    del toks[victim]
            finals[(b, g)] = {x: toks[x][2] for x in toks}
    return outs, drops, finals


def test_random_case_matches_pure_python_replay_and_invariants():
    rng = np.random.default_rng(5)
    B, Hq, Hkv, D, T = 2, 4, 2, 8, 14
    budget, recent = 8, 4
    n0 = [6, 3]
    k0, v0 = rand_bits(rng, (B, Hkv, 6, D), 1.5), rand_bits(rng, (B, Hkv, 6, D))
    tot0 = rng.random((B, Hkv, 6)).astype(np.float32)
    pos0 = np.tile(np.array([0, 1, 5, 6, 8, 9]), (B, Hkv, 1))          # gaps: what a prefill-side selection leaves
    pos0[1, :, :3] = [2, 3, 4]
    q = rand_bits(rng, (T, B, Hq, D), 1.5)
    nk, nv = rand_bits(rng, (T, B, Hkv, D), 1.5), rand_bits(rng, (T, B, Hkv, D))
    res = oracle.h2o_decode_loop(q, k0, v0, tot0, pos0, n0, nk, nv, 0.4, budget, recent)
    outs, drops, finals = _replay(q, k0, v0, tot0, pos0, n0, nk, nv, 0.4, budget, recent, Hq // Hkv)
    assert (res["dropped"] == drops).all()
    assert (drops >= 0).any() and (drops == -1).any()
    assert np.allclose(val(res["outs"]), outs, rtol=2 ** -8, atol=1e-30)
    for b in range(B):
        last = max(pos0[b, 0, :n0[b]]) + T
        for g in range(Hkv):
            got = res["final"][b][g]
            assert sorted(got) == sorted(finals[(b, g)])
            for x in got:
                assert abs(float(got[x]) - finals[(b, g)][x]) <= 1e-6 * abs(finals[(b, g)][x])
            assert len(got) == budget                                   # full, never above the budget
            assert all(x in got for x in range(last - recent + 1, last + 1))   # the recent ones are all there
    # totals of one step add up to 1 per head at most, so a token's total never exceeds its steps in the cache
    assert all(float(v) <= T + 1 for b in range(B) for g in range(Hkv) for v in res["final"][b][g].values())


def test_budget_never_reached_is_full_attention():
    rng = np.random.default_rng(9)
    B, Hq, Hkv, D, T = 1, 2, 1, 8, 5
    k0, v0, tot0, pos0, n0 = _empty(B, Hkv, D)
    q = rand_bits(rng, (T, B, Hq, D))
    nk, nv = rand_bits(rng, (T, B, Hkv, D)), rand_bits(rng, (T, B, Hkv, D))
    res = oracle.h2o_decode_loop(q, k0, v0, tot0, pos0, n0, nk, nv, 0.3, budget=T, recent=2)
    assert (res["dropped"] == -1).all()
    Kc, Vc = np.moveaxis(nk[:, 0], 0, 1)[None], np.moveaxis(nv[:, 0], 0, 1)[None]       # [1, Hkv, T, D]
    for t in range(T):
        out, _, _ = oracle.full_attn(q[t], Kc, Vc, [t + 1], 0.3)
        assert (out == res["outs"][t]).all()


def test_heavy_hitter_survives_and_ties_drop_the_older():
    D, T = 4, 9
    k0, v0, tot0, pos0, n0 = _empty(1, 1, D)
    keys = np.zeros((T, 1, 1, D)); keys[2, 0, 0, 0] = 30.0              # token 2 draws every later query
    q = bits(np.tile([1.0, 0, 0, 0], (T, 1, 1, 1)))
    res = oracle.h2o_decode_loop(q, k0, v0, tot0, pos0, n0, bits(keys), bits(np.ones((T, 1, 1, D))), 1.0,
                                 budget=4, recent=2)
    assert 2 in res["final"][0][0] and 2 not in res["dropped"]
    assert res["final"][0][0][2] > T - 3 - 1e-3
    # before token 2 arrives nothing is dropped; afterwards the others' totals stop growing (their share is
    # e^-30), and the lowest old one goes each time
    assert res["dropped"][:4, 0, 0].tolist() == [-1, -1, -1, -1]
    # exact ties: all-zero queries make every step uniform; two tokens entering with equal totals
    k0 = bits(np.zeros((1, 1, 3, D))); v0 = k0.copy()
    tot0 = np.array([[[0.5, 0.5, 0.5]]], np.float32); pos0 = np.array([[[4, 2, 7]]])
    r = oracle.h2o_decode_loop(bits(np.zeros((1, 1, 1, D))), k0, v0, tot0, pos0, [3], bits(np.zeros((1, 1, 1, D))),
                               bits(np.zeros((1, 1, 1, D))), 1.0, budget=3, recent=1)
    assert r["dropped"][0, 0, 0] == 2
