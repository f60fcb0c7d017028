"""Pins of the CPU oracle against things other than itself (no GPU needed).

Closed forms, pure-Python brute force on tiny inputs, the schedule printed in the paper's
Figure 1 caption, the cost model of its Appendix A.2 table, and the invariants Section 2.2
states.  Each test is chosen so that one plausible mistake in the oracle (dropped scale,
wrong head->group map, transposed operand, wrong tie order, pool off by one, ...) fails it.
"""
import math
import os

import numpy as np
import pytest
import torch

import gen
import oracle
from oracle.bf16 import bf16_bits_to_f64, f64_to_bf16_bits


# ----------------------------------------------------------------------------- helpers
def bits(x) -> np.ndarray:
    """fp values -> bf16 bit patterns through torch's own conversion (independent of oracle)."""
    return gen.bf16_bits(torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


def val(b) -> np.ndarray:
    """bf16 bit patterns -> python floats through torch (independent of oracle)."""
    return gen.bits_to_bf16(np.asarray(b, dtype=np.uint16)).to(torch.float64).numpy()


def rand_bits(rng, shape, gain=1.0):
    return bits(rng.standard_normal(shape) * gain)


def brute_attention(q, keys, values, scale):
    """Textbook softmax attention for one query in pure Python floats (lists of lists)."""
    n, D = len(keys), len(q)
    s = [scale * sum(q[d] * keys[j][d] for d in range(D)) for j in range(n)]
    m = max(s)
    e = [math.exp(x - m) for x in s]
    z = sum(e)
    a = [x / z for x in e]
    o = [sum(a[j] * values[j][d] for j in range(n)) for d in range(D)]
    return o, a, m + math.log(z)


# ----------------------------------------------------------------------------- bf16
def test_bf16_widening_matches_torch():
    allbits = np.arange(0, 1 << 16, dtype=np.uint16)
    mine = bf16_bits_to_f64(allbits)
    ref = val(allbits)
    ok = (mine == ref) | (np.isnan(mine) & np.isnan(ref))
    assert ok.all()


def test_bf16_rounding_matches_torch_and_ties_to_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 3, rng.standard_normal(2000) * 1e-3,
                        np.array([0.0, -0.0, 1.0, -1.0, 65504.0])]).astype(np.float32)
    assert (f64_to_bf16_bits(x.astype(np.float64)) == bits(x)).all()
    # exact halfway points between neighbours: 1 + 2^-8 lies between 1 (even) and 1 + 2^-7
    assert f64_to_bf16_bits(np.array([1.0 + 2.0 ** -8]))[0] == 0x3F80
    # 1 + 3*2^-8 lies between 1+2^-7 (odd mantissa) and 1+2^-6 (even) -> up
    assert f64_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 0x3F82
    # single rounding: just above the halfway point in fp64, not representable in fp32
    assert f64_to_bf16_bits(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 0x3F81
    assert f64_to_bf16_bits(np.array([-(1.0 + 2.0 ** -8 + 2.0 ** -40)]))[0] == 0xBF81


# ----------------------------------------------------------------------------- full attention
def test_full_attn_matches_pure_python_brute_force_gqa():
    rng = np.random.default_rng(1)
    B, Hq, Hkv, D, cap = 2, 6, 2, 8, 11
    lens = np.array([9, 5])
    q, K, V = rand_bits(rng, (B, Hq, D)), rand_bits(rng, (B, Hkv, cap, D)), rand_bits(rng, (B, Hkv, cap, D))
    scale = 0.3
    out, w, lse = oracle.full_attn(q, K, V, lens, scale)
    qv, Kv, Vv = val(q), val(K), val(V)
    G = Hq // Hkv
    for b in range(B):
        n = lens[b]
        for h in range(Hq):
            g = h // G          # heads of a group are contiguous
            o, a, l = brute_attention(list(qv[b, h]), Kv[b, g, :n].tolist(), Vv[b, g, :n].tolist(), scale)
            assert np.allclose(w[b, h, :n], a, rtol=1e-12, atol=0)
            assert (w[b, h, n:] == 0).all()
            assert abs(lse[b, h] - l) < 1e-12
            assert (out[b, h] == bits(np.array(o))).all() or np.allclose(val(out[b, h]), o, rtol=2 ** -8)
            assert abs(w[b, h, :n].sum() - 1.0) < 1e-12


def test_full_attn_two_key_closed_form_pins_scale_and_sign():
    # q = e0 * 2, k0 = e0 * 3, k1 = -e0: s = scale*(6, -2); a0 = 1/(1+exp(-8*scale))
    D = 4
    q = bits(np.array([[[2.0, 0, 0, 0]]]))
    K = bits(np.array([[[[3.0, 0, 0, 0], [-1.0, 0, 0, 0]]]]))
    V = bits(np.array([[[[1.0, 0, 0, 0], [0, 1.0, 0, 0]]]]))
    for scale in (1.0, 0.25):
        out, w, lse = oracle.full_attn(q, K, V, [2], scale)
        a0 = 1.0 / (1.0 + math.exp(-8.0 * scale))
        assert abs(w[0, 0, 0] - a0) < 1e-14 and abs(w[0, 0, 1] - (1 - a0)) < 1e-14
        assert abs(lse[0, 0] - (6 * scale + math.log1p(math.exp(-8 * scale)))) < 1e-13
        assert (out[0, 0] == bits(np.array([a0, 1 - a0, 0, 0]))).all()


def test_full_attn_uniform_and_zero_query_give_mean_of_values():
    rng = np.random.default_rng(2)
    n, D = 37, 16
    V = rand_bits(rng, (1, 1, n, D))
    same = np.repeat(rand_bits(rng, (1, 1, 1, D)), n, axis=2)
    q = rand_bits(rng, (1, 1, D))
    mean_v = val(V)[0, 0].mean(axis=0)
    for (qq, KK) in ((q, same), (bits(np.zeros((1, 1, D))), rand_bits(rng, (1, 1, n, D)))):
        out, w, lse = oracle.full_attn(qq, KK, V, [n], 0.5)
        assert np.allclose(w[0, 0], 1.0 / n, rtol=1e-13)
        assert (out[0, 0] == f64_to_bf16_bits(mean_v)).all()


def test_full_attn_dominant_key_and_len_one():
    rng = np.random.default_rng(3)
    n, D = 20, 8
    K = rand_bits(rng, (1, 1, n, D), gain=0.01)
    V = rand_bits(rng, (1, 1, n, D))
    qf = np.zeros((1, 1, D)); qf[0, 0, 0] = 16.0
    Kf = val(K); Kf[0, 0, 13, 0] = 16.0
    out, w, _ = oracle.full_attn(bits(qf), bits(Kf), V, [n], 1.0)
    assert w[0, 0, 13] > 1 - 1e-50 or w[0, 0, 13] == 1.0
    assert (out[0, 0] == V[0, 0, 13]).all()
    out1, w1, lse1 = oracle.full_attn(bits(qf), K, V, [1], 1.0)
    assert (out1[0, 0] == V[0, 0, 0]).all() and w1[0, 0, 0] == 1.0


def test_full_attn_ignores_rows_beyond_len():
    rng = np.random.default_rng(4)
    q, K, V = rand_bits(rng, (1, 4, 8)), rand_bits(rng, (1, 2, 12, 8)), rand_bits(rng, (1, 2, 12, 8))
    a = oracle.full_attn(q, K, V, [7], 0.4)
    K2, V2 = K.copy(), V.copy()
    K2[:, :, 7:] = 0x7F80  # +inf beyond the valid rows must not matter
    V2[:, :, 7:] = 0x7F80
    b = oracle.full_attn(q, K2, V2, [7], 0.4)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()


# ----------------------------------------------------------------------------- selection
def brute_topk(weights_group, n, k, pool_w):
    """Pure-Python statement: group max, clipped window max, sort by (-score, position)."""
    G = len(weights_group)
    A = [max(weights_group[h][j] for h in range(G)) for j in range(n)]
    half = (pool_w - 1) // 2
    P = [max(A[i] for i in range(max(0, j - half), min(n, j + half + 1))) for j in range(n)]
    order = sorted(range(n), key=lambda j: (-P[j], j))
    return order[:min(k, n)], P


@pytest.mark.parametrize("kind", ["lognormal", "ties"])
@pytest.mark.parametrize("pool_w", [1, 3, 7])
def test_topk_matches_pure_python(kind, pool_w):
    B, Hq, Hkv, n, k = 2, 6, 2, 61, 17
    w = gen.make_weights(B, Hq, n, seed=11, kind=kind).numpy()
    lens = [61, 40]
    idx, sel = oracle.topk_select(w, lens, Hkv, k, pool_w)
    G = Hq // Hkv
    for b in range(B):
        for g in range(Hkv):
            grp = [w[b, g * G + i, :lens[b]].tolist() for i in range(G)]
            want, P = brute_topk(grp, lens[b], k, pool_w)
            assert idx[b, g, :len(want)].tolist() == want
            assert sel[b, g, :len(want)].tolist() == [np.float32(P[j]) for j in want]
            assert idx.dtype == np.int32


def test_topk_one_hot_with_pool7_selects_the_window_then_lowest_positions():
    n, p = 50, 20
    w = np.zeros((1, 1, n), dtype=np.float32); w[0, 0, p] = 1.0
    idx, sel = oracle.topk_select(w, [n], 1, 10, 7)
    assert idx[0, 0].tolist() == [17, 18, 19, 20, 21, 22, 23, 0, 1, 2]
    assert sel[0, 0].tolist() == [1.0] * 7 + [0.0] * 3
    # clipped at the left edge: a peak at 1 covers positions 0..4 only
    w[:] = 0; w[0, 0, 1] = 1.0
    assert oracle.topk_select(w, [n], 1, 6, 7)[0][0, 0].tolist() == [0, 1, 2, 3, 4, 5]
    # pool 1: only the peak itself, then ties by position
    assert oracle.topk_select(w, [n], 1, 3, 1)[0][0, 0].tolist() == [1, 0, 2]


def test_topk_monotone_constant_and_k_ge_len():
    n = 12
    dec = np.linspace(1.0, 0.1, n, dtype=np.float32)[None, None]
    assert oracle.topk_select(dec, [n], 1, 5, 1)[0][0, 0].tolist() == [0, 1, 2, 3, 4]
    inc = dec[..., ::-1].copy()
    assert oracle.topk_select(inc, [n], 1, 5, 1)[0][0, 0].tolist() == [11, 10, 9, 8, 7]
    const = np.full((1, 1, n), 0.25, dtype=np.float32)
    assert oracle.topk_select(const, [n], 1, 5, 7)[0][0, 0].tolist() == [0, 1, 2, 3, 4]
    idx, sel = oracle.topk_select(inc, [7], 1, 10, 1)       # K >= len: everything, then -1
    assert idx[0, 0].tolist() == [6, 5, 4, 3, 2, 1, 0, -1, -1, -1]
    assert (sel[0, 0, 7:] == 0).all()


def test_topk_group_max_not_mean_or_first():
    # head 0 prefers token 0 weakly, head 1 prefers token 3 strongly: max picks 3 first;
    # the mean would pick 1 (0.45 avg) and the first head alone would pick 0.
    w = np.array([[[0.50, 0.45, 0.05, 0.00],
                   [0.00, 0.45, 0.00, 0.55]]], dtype=np.float32)
    assert oracle.topk_select(w, [4], 1, 2, 1)[0][0, 0].tolist() == [3, 0]
    # two groups of one head each select independently
    assert oracle.topk_select(w, [4], 2, 1, 1)[0][0, :, 0].tolist() == [0, 3]


def test_topk_mean_and_first_aggregation_match_pure_python():
    """Appendix A.3: mean over the group and first head of the group instead of the max."""
    rng = np.random.default_rng(44)
    G, n, k = 3, 40, 9
    w = rng.random((1, 2 * G, n)).astype(np.float64)
    for agg in ("mean", "first"):
        for pool_w in (1, 5):
            idx, sel = oracle.topk_select(w, [n], 2, k, pool_w, agg=agg)
            for g in range(2):
                rows = [w[0, g * G + h].tolist() for h in range(G)]
                A = [sum(r[j] for r in rows) / G if agg == "mean" else rows[0][j] for j in range(n)]
                half = (pool_w - 1) // 2
                P = [max(A[max(0, j - half):min(n, j + half + 1)]) for j in range(n)]
                order = sorted(range(n), key=lambda j: (-P[j], j))[:k]
                assert idx[0, g].tolist() == order
                assert np.allclose(sel[0, g], [P[j] for j in order], rtol=1e-15)
    # the three aggregations differ where they should: one head dominates one position
    w2 = np.full((1, 2, 6), 0.1); w2[0, 1, 4] = 0.9                   # only the second head sees position 4
    assert oracle.topk_select(w2, [6], 1, 1, 1, agg="max")[0][0, 0, 0] == 4
    assert oracle.topk_select(w2, [6], 1, 1, 1, agg="mean")[0][0, 0, 0] == 4
    assert oracle.topk_select(w2, [6], 1, 1, 1, agg="first")[0][0, 0, 0] == 0
    # fp32 in, fp32 arithmetic: the mean is the fp32 sum in head order divided in fp32
    w3 = np.array([[[1.0], [2.0 ** -24], [2.0 ** -24]]], dtype=np.float32)
    s3 = oracle.topk_select(w3, [1], 1, 1, 1, agg="mean")[1]
    assert s3.dtype == np.float32 and s3[0, 0, 0] == np.float32(1.0) / np.float32(3.0)


def test_topk_selected_dominate_unselected():
    w = gen.make_weights(1, 4, 500, seed=5).numpy()
    idx, sel = oracle.topk_select(w, [500], 1, 64, 7)
    P = oracle.pooled_group_scores(w[0], 7)
    chosen = set(idx[0, 0].tolist())
    assert len(chosen) == 64
    rest = [P[j] for j in range(500) if j not in chosen]
    assert min(P[j] for j in chosen) >= max(rest)
    assert all(sel[0, 0, i] >= sel[0, 0, i + 1] for i in range(63))


# ----------------------------------------------------------------------------- gather
def test_gather_is_a_bit_copy_and_skips_minus_one():
    rng = np.random.default_rng(6)
    K, V = rand_bits(rng, (2, 3, 20, 8)), rand_bits(rng, (2, 3, 20, 8))
    idx = rng.integers(0, 20, size=(2, 3, 5)).astype(np.int32)
    idx[1, 2, 3:] = -1
    sk = np.full((2, 3, 6, 8), 0xABCD, dtype=np.uint16); sv = sk.copy()
    oracle.gather_small_kv(K, V, idx, sk, sv)
    for b in range(2):
        for g in range(3):
            for i in range(5):
                j = idx[b, g, i]
                if j >= 0:
                    assert sk[b, g, i].tolist() == K[b, g, j].tolist()
                    assert sv[b, g, i].tolist() == V[b, g, j].tolist()
                else:
                    assert (sk[b, g, i] == 0xABCD).all() and (sv[b, g, i] == 0xABCD).all()
            assert (sk[b, g, 5] == 0xABCD).all()      # beyond k: untouched


# ----------------------------------------------------------------------------- partial attention
def _setup_partial(rng, B=2, Hq=4, Hkv=2, D=8, cap=40, lens=(30, 22), k=6, r=(3, 0)):
    q, K, V = rand_bits(rng, (B, Hq, D)), rand_bits(rng, (B, Hkv, cap, D)), rand_bits(rng, (B, Hkv, cap, D))
    lens = np.array(lens); tail = lens - np.array(r)
    idx = np.stack([np.stack([rng.permutation(tail[b])[:k] for _ in range(Hkv)]) for b in range(B)]).astype(np.int32)
    sk = np.zeros((B, Hkv, k, D), dtype=np.uint16); sv = sk.copy()
    oracle.gather_small_kv(K, V, idx, sk, sv)
    return q, K, V, lens, tail, idx, sk, sv


def test_partial_equals_masked_full_attention_brute_force():
    rng = np.random.default_rng(7)
    q, K, V, lens, tail, idx, sk, sv = _setup_partial(rng)
    scale = 0.35
    out = oracle.partial_attn(q, sk, sv, 6, K, V, tail, lens, scale)
    qv, Kv, Vv = val(q), val(K), val(V)
    for b in range(2):
        for h in range(4):
            g = h // 2
            rows = idx[b, g].tolist() + list(range(tail[b], lens[b]))
            o, _, _ = brute_attention(qv[b, h].tolist(), [Kv[b, g, j].tolist() for j in rows],
                                      [Vv[b, g, j].tolist() for j in rows], scale)
            assert np.allclose(val(out[b, h]), o, rtol=2 ** -8, atol=1e-30)
            assert (out[b, h] == f64_to_bf16_bits(np.array(o))).mean() > 0.8


def test_partial_with_whole_context_selected_equals_full():
    rng = np.random.default_rng(8)
    B, Hq, Hkv, D, n = 1, 4, 2, 8, 25
    q, K, V = rand_bits(rng, (B, Hq, D)), rand_bits(rng, (B, Hkv, 32, D)), rand_bits(rng, (B, Hkv, 32, D))
    w = oracle.full_attn(q, K, V, [n], 0.3)[1].astype(np.float32)
    idx, _ = oracle.topk_select(w, [n], Hkv, n + 4, 7)         # K > len
    sk = np.zeros((B, Hkv, n + 4, D), dtype=np.uint16); sv = sk.copy()
    oracle.gather_small_kv(K, V, idx, sk, sv)
    full = oracle.full_attn(q, K, V, [n], 0.3)[0]
    part = oracle.partial_attn(q, sk, sv, n + 4, K, V, [n], [n], 0.3)
    # same rows in another order: equal up to fp64 summation order, i.e. at most one bf16 ulp
    assert np.allclose(val(part), val(full), rtol=2 ** -7, atol=0)
    assert (part == full).mean() > 0.9


def test_partial_invariant_under_row_permutation_and_single_row():
    rng = np.random.default_rng(9)
    q, K, V, lens, tail, idx, sk, sv = _setup_partial(rng)
    a = oracle.partial_attn(q, sk, sv, 6, K, V, tail, lens, 0.3)
    perm = rng.permutation(6)
    b = oracle.partial_attn(q, sk[:, :, perm], sv[:, :, perm], 6, K, V, tail, lens, 0.3)
    assert np.allclose(val(a), val(b), rtol=2 ** -7)
    # one selected row, nothing recent: the output is that value row whatever the query
    one = oracle.partial_attn(q, sk, sv, 1, K, V, lens, lens, 0.3)
    for h in range(4):
        assert (one[0, h] == sv[0, h // 2, 0]).all()
    # n_sel larger than the context at refresh is clamped to it
    c = oracle.partial_attn(q[:1], sk[:1], sv[:1], 6, K[:1], V[:1], [4], [5], 0.3)
    d = oracle.partial_attn(q[:1], sk[:1], sv[:1], 4, K[:1], V[:1], [4], [5], 0.3)
    assert (c == d).all()


# ----------------------------------------------------------------------------- trigger
def test_query_sim_closed_forms():
    rng = np.random.default_rng(10)
    D, Hq = 16, 4
    qf = rng.standard_normal((1, Hq, D))
    q = bits(qf)
    qbar = val(q)[0].mean(axis=0)
    sim, need, ref = oracle.query_sim(q, qbar[None], 0.9)
    assert abs(sim[0] - 1) < 1e-15 and not need[0]
    sim, need, ref = oracle.query_sim(q, -3.0 * qbar[None], 0.9)
    assert abs(sim[0] + 1) < 1e-15 and need[0] and np.allclose(ref[0], qbar)
    orth = np.zeros(D); orth[0], orth[1] = qbar[1], -qbar[0]
    assert abs(oracle.query_sim(q, orth[None], 0.0)[0][0]) < 1e-16
    # cosine of the MEAN vector, not the mean of per-head cosines
    e = np.zeros((1, 2, 2)); e[0, 0] = [1, 0]; e[0, 1] = [0, 4]
    sim = oracle.query_sim(bits(e), np.array([[1.0, 0.0]]), 0.5)[0][0]
    assert abs(sim - 0.5 / math.sqrt(0.25 + 4.0)) < 1e-15     # mean = (0.5, 2)


def test_query_sim_threshold_edge_and_force():
    q = bits(np.array([[[3.0, 4.0]]]))
    ref = np.array([[1.0, 0.0]])                 # sim = 0.6 exactly representable? use compare
    sim = oracle.query_sim(q, ref, 0.0)[0][0]
    _, need_eq, _ = oracle.query_sim(q, ref, sim)          # sim == s  -> full
    _, need_lo, new_lo = oracle.query_sim(q, ref, sim - 1e-9)   # sim > s -> partial
    assert need_eq[0] and not need_lo[0]
    assert (new_lo == ref).all()                 # partial: reference kept
    _, need_f, new_f = oracle.query_sim(q, ref, sim - 1e-9, force_full=True)
    assert need_f[0] and np.allclose(new_f, [[3.0, 4.0]])
    # zero vectors do not divide by zero
    assert oracle.query_sim(bits(np.zeros((1, 1, 2))), np.zeros((1, 2)), 0.5)[0][0] == 0.0


# ----------------------------------------------------------------------------- schedule / loop
def _read_rows(path):
    with open(path) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def test_fig1_schedule(golden_dir):
    (line,) = _read_rows(os.path.join(golden_dir, "fig1_schedule.txt"))
    head, modes = line.split("|")
    L, K, S, T = map(int, head.split())
    want = {int(t): m for t, m in (tok.split(":") for tok in modes.split())}
    assert {t: ("F" if oracle.is_full_step(t, S) else "P") for t in range(1, T + 1)} == want
    # and the loop itself follows it
    rng = np.random.default_rng(12)
    D = 4
    res = oracle.decode_loop(rand_bits(rng, (T + 1, 1, 2, D)), rand_bits(rng, (1, 1, L + T, D)),
                             rand_bits(rng, (1, 1, L + T, D)), rand_bits(rng, (T, 1, 1, D)),
                             rand_bits(rng, (T, 1, 1, D)), [L], 0.5, K, S, pool_w=1, evict_lowest=True)
    assert ["F" if f else "P" for f in res["full"][1:, 0]] == [want[t] for t in range(1, T + 1)]
    assert res["full"][0, 0]                                   # prefill attends to everything
    # cache sizes of the figure: partial steps attend K rows, the full step L + 3
    assert res["rows"][:, 0].tolist() == [L, K, K, L + 3, K]


def test_cost_model_rows(golden_dir):
    for line in _read_rows(os.path.join(golden_dir, "cost_model.txt")):
        L, K, S, T = map(int, line.split())
        rng = np.random.default_rng(L)
        D = 4
        res = oracle.decode_loop(rand_bits(rng, (T + 1, 1, 1, D)), rand_bits(rng, (1, 1, L + T, D)),
                                 rand_bits(rng, (1, 1, L + T, D)), rand_bits(rng, (T, 1, 1, D)),
                                 rand_bits(rng, (T, 1, 1, D)), [L], 0.5, K, S, pool_w=1, evict_lowest=True)
        rows = res["rows"][1:, 0]
        n_full = T // S
        model = T * L / S + T * K                         # the paper's table
        exact = n_full * L + sum(S * i for i in range(1, n_full + 1)) + (T - n_full) * K
        assert rows.sum() == exact
        assert abs(rows.sum() - model) / model < 0.05
        van = oracle.decode_loop(rand_bits(rng, (T + 1, 1, 1, D)), rand_bits(rng, (1, 1, L + T, D)),
                                 rand_bits(rng, (1, 1, L + T, D)), rand_bits(rng, (T, 1, 1, D)),
                                 rand_bits(rng, (T, 1, 1, D)), [L], 0.5, K, 1, pool_w=1)
        assert van["rows"][1:, 0].sum() == T * L + T * (T + 1) // 2     # T x L, plus growth


def _small_loop_inputs(seed, T=9, B=2, Hq=4, Hkv=2, D=8, L=(21, 17)):
    rng = np.random.default_rng(seed)
    cap = max(L) + T + 1
    return dict(q=rand_bits(rng, (T + 1, B, Hq, D)), K=rand_bits(rng, (B, Hkv, cap, D)),
                V=rand_bits(rng, (B, Hkv, cap, D)), nk=rand_bits(rng, (T, B, Hkv, D)),
                nv=rand_bits(rng, (T, B, Hkv, D)), lens=np.array(L))


def test_stride_one_is_vanilla_attention():
    x = _small_loop_inputs(13)
    res = oracle.decode_loop(x["q"], x["K"], x["V"], x["nk"], x["nv"], x["lens"], 0.4, 5, 1)
    assert res["full"].all()
    # vanilla: attend over everything written so far, computed here with the brute force
    Kv, Vv = val(res["k"]), val(res["v"])
    for t in (0, 4, 9):
        for b in range(2):
            n = x["lens"][b] + t
            for h in range(4):
                o, _, _ = brute_attention(val(x["q"][t, b, h]).tolist(), Kv[b, h // 2, :n].tolist(),
                                          Vv[b, h // 2, :n].tolist(), 0.4)
                assert np.allclose(val(res["outs"][t, b, h]), o, rtol=2 ** -8, atol=1e-30)


def test_never_refreshed_keeps_the_initial_selection():
    x = _small_loop_inputs(14)
    res = oracle.decode_loop(x["q"], x["K"], x["V"], x["nk"], x["nv"], x["lens"], 0.4, 5, 0)
    assert res["full"][0].all() and not res["full"][1:].any()
    for snap in res["idx"][1:]:
        assert (snap == res["idx"][0]).all()
    # and that selection is the top-K of the first query's scores
    w = oracle.full_attn(x["q"][0], x["K"], x["V"], x["lens"], 0.4)[1].astype(np.float32)
    assert (oracle.topk_select(w, x["lens"], 2, 5, 7)[0] == res["idx"][0]).all()


def test_loop_refresh_changes_selection_and_tail_is_attended():
    x = _small_loop_inputs(15, T=8)
    res = oracle.decode_loop(x["q"], x["K"], x["V"], x["nk"], x["nv"], x["lens"], 0.4, 5, 4, pool_w=1)
    assert res["full"][:, 0].tolist() == [True, False, False, False, True, False, False, False, True]
    # rows: K + r on partial steps (all K selected rows kept + r appended ones)
    assert res["rows"][:, 0].tolist() == [21, 6, 7, 8, 25, 6, 7, 8, 29]
    # a partial step equals brute-force attention over idx rows + appended rows
    t, b = 6, 1
    Kv, Vv = val(res["k"]), val(res["v"])
    n = x["lens"][b] + t
    tail0 = x["lens"][b] + 4
    for h in range(4):
        g = h // 2
        rows = res["idx"][4][b, g].tolist() + list(range(tail0, n))
        o, _, _ = brute_attention(val(x["q"][t, b, h]).tolist(), [Kv[b, g, j].tolist() for j in rows],
                                  [Vv[b, g, j].tolist() for j in rows], 0.4)
        assert np.allclose(val(res["outs"][t, b, h]), o, rtol=2 ** -8, atol=1e-30)


def test_attn_scores_match_pure_python_and_closed_forms():
    """Scores-only pass (Section 4.3, "w/o full attention"): softmax of scale * q.K over the
    valid rows, keys only."""
    rng = np.random.default_rng(31)
    B, Hq, Hkv, D, cap = 2, 6, 2, 8, 12
    lens = [11, 5]
    q, K = rand_bits(rng, (B, Hq, D)), rand_bits(rng, (B, Hkv, cap, D), 1.5)
    w, lse = oracle.attn_scores(q, K, lens, 0.37)
    assert w.shape == (B, Hq, 11)
    for b in range(B):
        for h in range(Hq):
            g = h // 3                                     # G = 3: heads 0-2 -> KV head 0
            keys = val(K[b, g, :lens[b]]).tolist()
            _, a, l = brute_attention(val(q[b, h]).tolist(), keys, keys, 0.37)
            assert np.allclose(w[b, h, :lens[b]], a, rtol=1e-12, atol=0)
            assert (w[b, h, lens[b]:] == 0).all()
            assert abs(lse[b, h] - l) < 1e-12
    # two keys, closed form: a0 = 1 / (1 + exp(scale * q.(k1 - k0)))
    q2 = bits([[[1.0, 2.0]]]); K2 = bits([[[[0.5, -1.0], [0.25, 0.5]]]])
    w2, _ = oracle.attn_scores(q2, K2, [2], 0.5)
    s0, s1 = 0.5 * (0.5 - 2.0), 0.5 * (0.25 + 1.0)
    assert abs(w2[0, 0, 0] - 1 / (1 + math.exp(s1 - s0))) < 1e-15
    # equal keys: uniform scores; an empty sequence: nothing, lse = -inf
    Ku = bits(np.ones((1, 1, 7, 2)))
    wu, _ = oracle.attn_scores(q2, Ku, [7], 3.0)
    assert np.allclose(wu, 1 / 7, rtol=1e-15)
    w0, l0 = oracle.attn_scores(q2, Ku, [0], 3.0)
    assert w0.shape == (1, 1, 0) and l0[0, 0] == -np.inf


def test_scores_only_refresh_loop():
    """Section 4.3, "w/o full attention": at a refresh step the output is attention over the
    rebuilt small cache alone; the selections, and every partial step, are those of the
    normal schedule."""
    x = _small_loop_inputs(17, T=8)
    args = (x["q"], x["K"], x["V"], x["nk"], x["nv"], x["lens"], 0.4, 5, 4)
    ref = oracle.decode_loop(*args, pool_w=1)
    res = oracle.decode_loop(*args, pool_w=1, scores_only_refresh=True)
    assert (res["full"] == ref["full"]).all()
    for a, c in zip(res["idx"], ref["idx"]):
        assert (a == c).all()
    partial = ~res["full"][:, 0]
    assert (res["outs"][partial] == ref["outs"][partial]).all()
    assert not (res["outs"][~partial] == ref["outs"][~partial]).all()     # refresh steps differ
    assert res["rows"][:, 0].tolist() == [5, 6, 7, 8, 5, 6, 7, 8, 5]
    # a refresh step equals brute-force attention over exactly the selected rows
    Kv, Vv = val(res["k"]), val(res["v"])
    for t in (0, 4, 8):
        for b in range(2):
            for h in range(4):
                g = h // 2
                rows = res["idx"][t][b, g].tolist()
                assert len(set(rows)) == 5 and min(rows) >= 0
                o, _, _ = brute_attention(val(x["q"][t, b, h]).tolist(), [Kv[b, g, j].tolist() for j in rows],
                                          [Vv[b, g, j].tolist() for j in rows], 0.4)
                assert np.allclose(val(res["outs"][t, b, h]), o, rtol=2 ** -8, atol=1e-30)
    # a small cache as large as the context selects everything: the step is full attention again
    big = oracle.decode_loop(x["q"], x["K"], x["V"], x["nk"], x["nv"], x["lens"], 0.4, 40, 1,
                             scores_only_refresh=True)
    van = oracle.decode_loop(x["q"], x["K"], x["V"], x["nk"], x["nv"], x["lens"], 0.4, 40, 1)
    assert (big["outs"] == van["outs"]).all()


def test_dynamic_trigger_in_loop():
    x = _small_loop_inputs(16, T=8, B=1, L=(21,))
    # identical queries at every step: similarity 1 > s, so no full step after t=0
    q_same = np.repeat(x["q"][:1], 9, axis=0)
    res = oracle.decode_loop(q_same, x["K"][:1], x["V"][:1], x["nk"][:, :1], x["nv"][:, :1], [21], 0.4, 5, 2,
                             dynamic=True, threshold=0.9)
    assert res["full"][:, 0].tolist() == [True] + [False] * 8
    assert np.allclose(res["sims"][[2, 4, 6, 8], 0], 1.0) and np.isnan(res["sims"][[1, 3, 5, 7], 0]).all()
    # independent random queries: similarity ~0 <= s at every tested step -> full on every 2nd
    res = oracle.decode_loop(x["q"][:, :1], x["K"][:1], x["V"][:1], x["nk"][:, :1], x["nv"][:, :1], [21], 0.4, 5, 2,
                             dynamic=True, threshold=0.9)
    assert res["full"][:, 0].tolist() == [True, False, True, False, True, False, True, False, True]


def test_window_votes_match_pure_python_and_closed_forms():
    """Observation window of W prompt tokens (Section 2.2 "Prefilling stage"; Section 3 on the
    SnapKV baseline; Appendix A.1 "Baseline Settings"): per query head, the sum over the
    window's queries of the causal post-softmax scores."""
    rng = np.random.default_rng(77)
    B, W, Hq, Hkv, D, cap = 2, 3, 4, 2, 8, 12
    lens = [10, 2]                                             # the second prompt is shorter than the window
    qw, K = rand_bits(rng, (B, W, Hq, D)), rand_bits(rng, (B, Hkv, cap, D), 1.5)
    votes = oracle.window_votes(qw, K, lens, 0.41)
    assert votes.shape == (B, Hq, 10)
    for b in range(B):
        for h in range(Hq):
            want = [0.0] * 10
            for i in range(W):
                pos = lens[b] - W + i                          # query i sits at this position
                if pos < 0:
                    continue
                keys = val(K[b, h // 2, :pos + 1]).tolist()
                _, a, _ = brute_attention(val(qw[b, i, h]).tolist(), keys, keys, 0.41)
                for j in range(pos + 1):
                    want[j] += a[j]
            assert np.allclose(votes[b, h], want, rtol=1e-12, atol=1e-300)
    # every existing query hands out one vote in all: 3 for the long prompt, 2 for the short one
    assert np.allclose(votes[0].sum(axis=1), 3.0, rtol=1e-12)
    assert np.allclose(votes[1].sum(axis=1), 2.0, rtol=1e-12)
    # equal keys: query at position p gives 1/(p+1) to rows 0..p, so row j collects a harmonic tail
    Ku = bits(np.ones((1, 1, 9, 2)))
    qu = rand_bits(rng, (1, 4, 1, 2))
    vu = oracle.window_votes(qu, Ku, [9], 2.0)[0, 0]
    for j in range(9):
        assert abs(vu[j] - sum(1.0 / (p + 1) for p in range(5, 9) if p >= j)) < 1e-14
    # causality: the last row is seen by the last query only; a window of one is the plain score pass
    one, _ = oracle.attn_scores(qw[:, -1], K, lens, 0.41)
    assert np.array_equal(oracle.window_votes(qw[:, -1:], K, lens, 0.41), one)
    last = oracle.window_votes(qw, K, lens, 0.41)[0, :, 9]
    assert np.allclose(last, one[0, :, 9], rtol=1e-14)
    # a dominant key inside every query's view collects the whole window
    Kd = np.zeros((1, 1, 6, 2)); Kd[0, 0, 1] = [40.0, 0.0]
    qd = bits(np.tile([[1.0, 0.0]], (1, 3, 1, 1)))
    vd = oracle.window_votes(qd, bits(Kd), [6], 1.0)[0, 0]
    assert abs(vd[1] - 3.0) < 1e-12 and vd[[0, 2, 3, 4, 5]].max() < 1e-15
