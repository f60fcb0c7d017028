"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle.

Same seeded inputs on both sides; the oracle never sees anything the GPU produced.
Tolerances: outputs <= 2e-2 max-abs (and one bf16 step); attention weights 1e-5 relative
(sanity; measured error is ~1e-6); indices exact except across oracle score gaps <= 1e-6
relative; gathers bit-exact.
"""
import sys

import numpy as np
import pytest
import torch

import gen
import oracle
from helpers import assert_out_close, assert_idx_equivalent

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_05787_amd as lib     # raises if the HIP library is not built
    return lib


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def rand_case(seed, B, Hq, Hkv, cap, gain=1.0, D=128):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Hq, D, generator=g).to(torch.bfloat16)
    K = (torch.randn(B, Hkv, cap, D, generator=g) * gain).to(torch.bfloat16)
    V = torch.randn(B, Hkv, cap, D, generator=g).to(torch.bfloat16)
    return q, K, V


def gpu_full(rk, geom, q, K, V, lens, max_len, want_weights=True, pred=None, pred_val=0, out_init=None):
    dev = "cuda"
    B, Hq = geom.batch, geom.n_q_heads
    ws = rk.Workspace(geom, K.shape[2], 16)
    out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device=dev) if out_init is None else out_init.clone().to(dev)
    w = torch.full((B, Hq, K.shape[2]), -7.0, dtype=torch.float32, device=dev) if want_weights else None
    lse = torch.full((B, Hq), 123.0, dtype=torch.float32, device=dev)
    sl = torch.tensor(lens, dtype=torch.int32, device=dev)
    rk.rk_full_attn(geom, q.to(dev), K.to(dev), V.to(dev), sl, max_len, out, weights=w, lse=lse,
                    pred=None if pred is None else torch.tensor(pred, dtype=torch.int32, device=dev),
                    pred_val=pred_val, workspace=ws)
    torch.cuda.synchronize()
    return gen.bf16_bits(out), (None if w is None else w.cpu().numpy()), lse.cpu().numpy()


FULL_CASES = [
    # name, B, Hq, Hkv, lens, cap        (row counts chosen to hit ragged tails and every tile path)
    ("llama_ragged", 2, 32, 8, [700, 333], 768),
    ("qwen_g7", 1, 28, 4, [1000], 1024),
    ("mha_g1", 1, 4, 4, [130], 256),
    ("g2", 2, 8, 4, [65, 64], 128),
    ("g8", 1, 16, 2, [517], 640),
    ("g3_g5_like", 1, 15, 3, [97], 128),
    ("len1_and_len0", 3, 8, 2, [1, 0, 17], 64),
    ("tiles2_path", 4, 32, 8, [2100, 1500, 2099, 64], 2112),     # chunk 128
    ("tiles4_path", 4, 32, 8, [4200, 4100, 255, 257], 4224),     # chunk 256
    # long rows: without weights the wide split + the separate merge launch
    ("long_two_heads", 1, 8, 2, [20000], 20032),
    ("long_llama", 1, 32, 8, [9001], 9024),
    # ragged batches: the workgroups of a launch are shared out by length (2..64 sequences); 65 take the even split
    ("ragged_16", 16, 8, 2, [3000, 1, 0, 129, 2999, 640, 77, 1500, 128, 127, 2048, 5, 900, 31, 3000, 256], 3008),
    ("ragged_64", 64, 4, 1, [((i * 37) % 19) * 61 + (i % 3) for i in range(64)], 1152),
    ("ragged_65_even_split", 65, 4, 1, [((i * 37) % 19) * 61 + (i % 3) for i in range(65)], 1152),
    ("ragged_one_long", 3, 8, 2, [6000, 40, 200], 6016),
    ("ragged_64_one_long", 64, 4, 1, [3000] + [1] * 62 + [0], 3008),     # shares capped by the rows a sequence has
]


@pytest.mark.parametrize("case", FULL_CASES, ids=[c[0] for c in FULL_CASES])
def test_full_attn_matches_oracle(rk, case):
    name, B, Hq, Hkv, lens, cap = case
    say("full_attn case", case)
    q, K, V = rand_case(100 + len(name), B, Hq, Hkv, cap)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    out, w, lse = gpu_full(rk, geom, q, K, V, lens, max(max(lens), 1))
    o_ref, w_ref, lse_ref = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), lens, scale)
    assert_out_close(out, o_ref, name)
    for b in range(B):
        n = lens[b]
        if n == 0:
            assert (lse[b] == -np.inf).all() and (out[b] == 0).all()
            continue
        rel = np.abs(w[b, :, :n] - w_ref[b, :, :n]) / w_ref[b, :, :n]
        assert rel.max() < 1e-5, "weights rel err %.3g" % rel.max()
        assert np.abs(w[b, :, :n].sum(axis=1) - 1).max() < 1e-5
        assert (w[b, :, n:] == -7.0).all(), "weights beyond len must not be written"
        assert np.abs(lse[b] - lse_ref[b]).max() < 1e-5
    # without weights (single launch, merged inside the kernel in another summation order)
    out2, _, lse2 = gpu_full(rk, geom, q, K, V, lens, max(max(lens), 1), want_weights=False)
    assert_out_close(out2, o_ref, name + " (no weights)")
    finite = np.isfinite(lse_ref)
    assert np.abs(lse2[finite] - lse_ref[finite]).max(initial=0.0) < 1e-5 and (lse2[~finite] == -np.inf).all()


def test_full_attn_planted_keys_and_max_len_clamp(rk):
    say("full_attn planted / clamp")
    B, Hq, Hkv, cap = 1, 32, 8, 2048
    q, K, V = rand_case(7, B, Hq, Hkv, cap)
    K[:, :, ::131] *= 4.0                                   # a few dominant keys per head
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    out, w, _ = gpu_full(rk, geom, q, K, V, [2048], 2048)
    o_ref, w_ref, _ = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), [2048], scale)
    assert_out_close(out, o_ref)
    assert (np.abs(w[0, :, :2048] - w_ref[0]) / w_ref[0]).max() < 1e-5
    # a sequence longer than max_len is processed up to max_len
    out_c, _, _ = gpu_full(rk, geom, q, K, V, [2048], 1000)
    o_c, _, _ = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), [1000], scale)
    assert_out_close(out_c, o_c)


def test_full_attn_predicate_skips_sequences(rk):
    say("full_attn predicate")
    B, Hq, Hkv, cap = 3, 8, 2, 256
    q, K, V = rand_case(9, B, Hq, Hkv, cap)
    scale = 0.1
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    init = torch.full((B, Hq, 128), 5.0, dtype=torch.bfloat16)
    out, w, lse = gpu_full(rk, geom, q, K, V, [200, 100, 256], 256, pred=[1, 0, 1], pred_val=1, out_init=init)
    o_ref, _, _ = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), [200, 100, 256], scale)
    assert_out_close(out[[0, 2]], o_ref[[0, 2]])
    assert (out[1] == gen.bf16_bits(init)[1]).all() and (w[1] == -7.0).all() and (lse[1] == 123.0).all()


def test_full_attn_scores_phase_alone(rk):
    """rk_full_attn_scores: the streaming kernel by itself leaves scale * q.k in the buffer."""
    say("full_attn_scores")
    B, Hq, Hkv, cap = 2, 8, 2, 1100
    lens = [1100, 37]
    q, K, V = rand_case(33, B, Hq, Hkv, cap)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    ws = rk.Workspace(geom, cap, 16)
    sc = torch.full((B, Hq, cap), -7.0, dtype=torch.float32, device="cuda")
    rk.rk_full_attn_scores(geom, q.cuda(), K.cuda(), V.cuda(), torch.tensor(lens, dtype=torch.int32, device="cuda"),
                           cap, sc, workspace=ws)
    torch.cuda.synchronize()
    _, w_ref, lse_ref = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), lens, scale)
    got = sc.cpu().numpy()
    for b in range(B):
        n = lens[b]
        s_ref = np.log(w_ref[b, :, :n]) + lse_ref[b][:, None]          # s = ln a + lse
        assert np.abs(got[b, :, :n] - s_ref).max() < 2e-6
        assert (got[b, :, n:] == -7.0).all()


TOPK_CASES = [
    # name, B, Hq, Hkv, lens, k, pool_w, kind
    ("lognormal_pool7", 2, 8, 2, [5000, 3777], 256, 7, "lognormal"),
    ("lognormal_pool1", 1, 4, 1, [4096], 100, 1, "lognormal"),
    ("ties_pool7", 2, 6, 2, [3000, 2999], 333, 7, "ties"),
    ("ties_pool1_k1", 1, 2, 2, [1500], 1, 1, "ties"),
    ("k_ge_len", 2, 4, 2, [50, 7], 64, 7, "lognormal"),
    ("len0", 2, 4, 2, [0, 20], 8, 3, "lognormal"),
    ("big_k", 1, 4, 1, [40000], 8192, 7, "lognormal"),
    ("max_k_ties", 1, 2, 1, [33000], 16384, 7, "ties"),
    ("pool63", 1, 2, 1, [2000], 128, 63, "lognormal"),
    ("refine_path", 1, 2, 1, [90000], 14000, 1, "lognormal"),     # more candidates than LDS holds: bin cut again
    ("ragged_batch", 5, 8, 2, [70000, 3, 1025, 64, 31999], 1024, 7, "lognormal"),
    ("many_candidates_128k", 1, 4, 1, [131072], 8192, 7, "lognormal"),    # buckets laid out from the histogram
    ("many_candidates_pool1", 2, 2, 1, [60000, 20000], 8192, 1, "lognormal"),
    # more candidate positions than LDS holds, but their runs of equal pooled scores fit: no second cut
    ("runs_fit_positions_do_not_128k", 1, 4, 1, [131072], 16000, 7, "lognormal"),
    ("runs_fit_one_workgroup", 2, 4, 2, [8100, 6000], 1100, 7, "lognormal"),
    ("dense_one_workgroup_ties", 1, 4, 1, [8192], 1500, 7, "ties"),
    ("pool3_runs_cut_by_k", 1, 2, 2, [20000], 999, 3, "lognormal"),
    # score distributions far from a softmax row's: stretches of one value, one histogram bin, rare spikes, all equal
    ("plateaus_70k", 2, 4, 2, [70000, 41234], 5000, 7, "plateaus"),
    ("narrow_band_40k", 1, 4, 1, [40000], 8192, 7, "narrow"),
    ("spiky_140k", 1, 7, 1, [140000], 2048, 15, "spiky"),
    ("all_zero_9k", 2, 2, 2, [9000, 5], 1000, 7, "zeros"),
]


@pytest.mark.parametrize("case", TOPK_CASES, ids=[c[0] for c in TOPK_CASES])
def test_topk_select_exact(rk, case):
    name, B, Hq, Hkv, lens, k, pool_w, kind = case
    say("topk case", case)
    n = max(max(lens), 1)
    w = gen.make_weights(B, Hq, n, seed=len(name) * 13 + k, kind=kind)
    geom = rk.Geom(B, Hq, Hkv, 128, 1.0)
    ws = rk.Workspace(geom, n, k)
    idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    sel = torch.full((B, Hkv, k), -5.0, dtype=torch.float32, device="cuda")
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    rk.rk_topk_select(geom, w.cuda(), sl, n, k, pool_w, idx, sel_scores=sel, workspace=ws)
    torch.cuda.synchronize()
    i_ref, s_ref = oracle.topk_select(w.numpy(), lens, Hkv, k, pool_w)
    assert (idx.cpu().numpy() == i_ref).all()
    assert (sel.cpu().numpy() == s_ref).all()
    # same call again: deterministic
    idx2 = torch.empty_like(idx)
    rk.rk_topk_select(geom, w.cuda(), sl, n, k, pool_w, idx2, workspace=ws)
    torch.cuda.synchronize()
    assert (idx2 == idx).all()


FUSED_CASES = [
    # name, B, Hq, Hkv, lens, cap, k, pool_w
    ("llama_ragged", 2, 32, 8, [3100, 1029], 3200, 256, 7),          # several pooling tiles, ragged
    ("qwen_g7", 1, 28, 4, [2500], 2560, 128, 7),
    ("g8_pool1", 1, 16, 2, [1300], 1408, 64, 1),
    ("mha_g1_pool63", 1, 4, 4, [1024], 1024, 100, 63),               # halo as wide as allowed, tile-aligned length
    ("short_and_empty", 3, 8, 2, [5, 0, 1025], 1100, 16, 7),         # k > len, len 0, one position past a tile
    ("g5", 1, 15, 3, [700], 704, 32, 3),
]


@pytest.mark.parametrize("case", FUSED_CASES, ids=[c[0] for c in FUSED_CASES])
def test_full_attn_select_matches_oracle(rk, case):
    """rk_full_attn_select = rk_full_attn + rk_topk_select: out, lse, weights and idx against the
    oracle, with and without the weights returned, twice in a row (workspace left clean)."""
    name, B, Hq, Hkv, lens, cap, k, pool_w = case
    say("full_attn_select case", case)
    q, K, V = rand_case(200 + len(name), B, Hq, Hkv, cap)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    ws = rk.Workspace(geom, cap, k)
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    qd, Kd, Vd = q.cuda(), K.cuda(), V.cuda()
    o_ref, w_ref, lse_ref = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), lens, scale)
    i_ref, s_ref = oracle.topk_select(w_ref.astype(np.float32), lens, Hkv, k, pool_w)
    G = Hq // Hkv
    max_len = max(max(lens), 1)
    for rep, want_w in enumerate([True, False, True]):
        out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
        wt = torch.full((B, Hq, cap), -7.0, dtype=torch.float32, device="cuda") if want_w else None
        lse = torch.full((B, Hq), 123.0, dtype=torch.float32, device="cuda")
        idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
        sel = torch.full((B, Hkv, k), -5.0, dtype=torch.float32, device="cuda")
        rk.rk_full_attn_select(geom, qd, Kd, Vd, sl, max_len, out, k, pool_w, idx, weights=wt, lse=lse,
                               sel_scores=sel, workspace=ws)
        torch.cuda.synchronize()
        assert_out_close(gen.bf16_bits(out), o_ref, "%s rep %d" % (name, rep))
        idx_n, sel_n, lse_n = idx.cpu().numpy(), sel.cpu().numpy(), lse.cpu().numpy()
        for b in range(B):
            n = lens[b]
            if n == 0:
                assert (lse_n[b] == -np.inf).all() and (idx_n[b] == -1).all()
                continue
            assert np.abs(lse_n[b] - lse_ref[b]).max() < 1e-5
            if want_w:
                wn = wt[b].cpu().numpy()
                assert (np.abs(wn[:, :n] - w_ref[b, :, :n]) / w_ref[b, :, :n]).max() < 1e-5
                assert (wn[:, n:] == -7.0).all(), "weights beyond len must not be written"
            for g in range(Hkv):
                P = oracle.pooled_group_scores(w_ref[b, g * G:(g + 1) * G, :n].astype(np.float32), pool_w)
                assert_idx_equivalent(idx_n[b, g], i_ref[b, g], P, n, k, "%s b=%d g=%d" % (name, b, g))
                kk = min(k, n)
                assert np.abs(sel_n[b, g, :kk] - s_ref[b, g, :kk]).max() <= 1e-5 * s_ref[b, g, :kk].max()
                assert (sel_n[b, g, kk:] == 0).all()
    # and the same indices as the two separate calls on the same inputs
    out2 = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    wt2 = torch.zeros(B, Hq, cap, dtype=torch.float32, device="cuda")
    idx2 = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    rk.rk_full_attn(geom, qd, Kd, Vd, sl, max_len, out2, weights=wt2, workspace=ws)
    rk.rk_topk_select(geom, wt2, sl, max_len, k, pool_w, idx2, workspace=ws)
    torch.cuda.synchronize()
    for b in range(B):
        for g in range(Hkv):
            n = lens[b]
            if n == 0:
                continue
            P = oracle.pooled_group_scores(w_ref[b, g * G:(g + 1) * G, :n].astype(np.float32), pool_w)
            assert_idx_equivalent(idx2[b, g].cpu().numpy(), idx_n[b, g], P, n, k, "two calls vs one")


def test_full_attn_select_predicate(rk):
    say("full_attn_select predicate")
    B, Hq, Hkv, cap, k = 3, 8, 2, 1500, 32
    lens = [1200, 900, 1500]
    q, K, V = rand_case(77, B, Hq, Hkv, cap)
    geom = rk.Geom(B, Hq, Hkv, 128, 0.1)
    ws = rk.Workspace(geom, cap, k)
    out = torch.full((B, Hq, 128), 5.0, dtype=torch.bfloat16, device="cuda")
    idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    pred = torch.tensor([1, 0, 1], dtype=torch.int32, device="cuda")
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    rk.rk_full_attn_select(geom, q.cuda(), K.cuda(), V.cuda(), sl, cap, out, k, 7, idx, pred=pred, pred_val=1, workspace=ws)
    torch.cuda.synchronize()
    o_ref, w_ref, _ = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), lens, 0.1)
    i_ref, _ = oracle.topk_select(w_ref.astype(np.float32), lens, Hkv, k, 7)
    got = gen.bf16_bits(out)
    assert_out_close(got[[0, 2]], o_ref[[0, 2]])
    assert (out[1] == 5.0).all() and (idx[1] == -5).all()
    G = Hq // Hkv
    for b in (0, 2):
        for g in range(Hkv):
            P = oracle.pooled_group_scores(w_ref[b, g * G:(g + 1) * G, :lens[b]].astype(np.float32), 7)
            assert_idx_equivalent(idx[b, g].cpu().numpy(), i_ref[b, g], P, lens[b], k, "pred b=%d" % b)


@pytest.mark.parametrize("agg", ["mean", "first"])
def test_topk_select_other_aggregations_exact(rk, agg):
    """Appendix A.3: mean over the group / first head of the group; same fp32 weights on both sides,
    so the result is exact, the mean included (fp32 sum in head order, fp32 division)."""
    code = {"mean": rk.RK_AGG_MEAN, "first": rk.RK_AGG_FIRST}[agg]
    for name, B, Hq, Hkv, lens, k, pool_w, kind in [("g4", 2, 8, 2, [5000, 3777], 256, 7, "lognormal"),
                                                     ("g7_ties", 1, 7, 1, [3000], 333, 7, "ties"),
                                                     ("g3_pool1", 1, 6, 2, [1500], 100, 1, "lognormal")]:
        say("topk", agg, name)
        n = max(lens)
        w = gen.make_weights(B, Hq, n, seed=len(name) * 7 + k, kind=kind)
        geom = rk.Geom(B, Hq, Hkv, 128, 1.0)
        ws = rk.Workspace(geom, n, k)
        idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
        sel = torch.full((B, Hkv, k), -5.0, dtype=torch.float32, device="cuda")
        rk.rk_topk_select(geom, w.cuda(), torch.tensor(lens, dtype=torch.int32, device="cuda"), n, k, pool_w, idx,
                          sel_scores=sel, agg=code, workspace=ws)
        torch.cuda.synchronize()
        i_ref, s_ref = oracle.topk_select(w.numpy(), lens, Hkv, k, pool_w, agg=agg)
        assert (idx.cpu().numpy() == i_ref).all()
        assert (sel.cpu().numpy() == s_ref).all()


def test_full_attn_select_mean_aggregation(rk):
    say("full_attn_select, mean aggregation")
    B, Hq, Hkv, cap, k = 1, 8, 2, 2600, 128
    lens = [2500]
    q, K, V = rand_case(515, B, Hq, Hkv, cap)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    ws = rk.Workspace(geom, cap, k)
    out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    rk.rk_full_attn_select(geom, q.cuda(), K.cuda(), V.cuda(), torch.tensor(lens, dtype=torch.int32, device="cuda"),
                           2500, out, k, 7, idx, agg=rk.RK_AGG_MEAN, workspace=ws)
    torch.cuda.synchronize()
    o_ref, w_ref, _ = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), lens, scale)
    w32 = w_ref.astype(np.float32)
    i_ref, _ = oracle.topk_select(w32, lens, Hkv, k, 7, agg="mean")
    assert_out_close(gen.bf16_bits(out), o_ref)
    for g in range(Hkv):
        P = oracle.pooled_group_scores(w32[0, g * 4:(g + 1) * 4, :2500], 7, "mean")
        assert_idx_equivalent(idx[0, g].cpu().numpy(), i_ref[0, g], P, 2500, k, "g=%d" % g)
    i_max, _ = oracle.topk_select(w32, lens, Hkv, k, 7)
    assert (i_ref != i_max).any(), "the case should tell mean from max"


def test_gather_bit_exact(rk):
    say("gather")
    B, Hkv, cap, k = 3, 4, 500, 77
    _, K, V = rand_case(21, B, 4, Hkv, cap)
    g = torch.Generator().manual_seed(3)
    idx = torch.randint(0, cap, (B, Hkv, k), generator=g, dtype=torch.int32)
    idx[1, 2, 50:] = -1
    geom = rk.Geom(B, 4, Hkv, 128, 1.0)
    sK = torch.full((B, Hkv, k + 3, 128), 9.0, dtype=torch.bfloat16, device="cuda")
    sV = torch.full((B, Hkv, k + 3, 128), 9.0, dtype=torch.bfloat16, device="cuda")
    rk.rk_gather_small_kv(geom, K.cuda(), V.cuda(), idx.cuda(), k, sK, sV)
    torch.cuda.synchronize()
    rK = np.full((B, Hkv, k + 3, 128), gen.bf16_bits(torch.tensor(9.0, dtype=torch.bfloat16)), dtype=np.uint16)
    rV = rK.copy()
    oracle.gather_small_kv(gen.bf16_bits(K), gen.bf16_bits(V), idx.numpy(), rK, rV)
    assert (gen.bf16_bits(sK) == rK).all() and (gen.bf16_bits(sV) == rV).all()
    # refresh bookkeeping in the same launch, honouring the predicate
    sl = torch.tensor([400, 410, 420], dtype=torch.int32, device="cuda")
    tail = torch.tensor([1, 2, 3], dtype=torch.int32, device="cuda")
    pred = torch.tensor([1, 0, 1], dtype=torch.int32, device="cuda")
    sK2 = torch.full_like(sK, 9.0); sV2 = torch.full_like(sV, 9.0)
    rk.rk_gather_small_kv(geom, K.cuda(), V.cuda(), idx.cuda(), k, sK2, sV2, seq_lens=sl, tail_start=tail,
                          pred=pred, pred_val=1)
    torch.cuda.synchronize()
    assert tail.tolist() == [400, 2, 420]
    got = gen.bf16_bits(sK2)
    assert (got[[0, 2]] == rK[[0, 2]]).all() and (got[1] == gen.bf16_bits(torch.tensor(9.0, dtype=torch.bfloat16))).all()
    tail2 = torch.tensor([7, 7, 7], dtype=torch.int32, device="cuda")
    rk.rk_mark_refresh(geom, sl, tail2, pred=pred, pred_val=0)
    torch.cuda.synchronize()
    assert tail2.tolist() == [7, 410, 7]


PARTIAL_CASES = [
    # name, B, Hq, Hkv, lens, recent, k, n_sel
    ("llama_k256_r3", 2, 32, 8, [900, 650], [3, 0], 256, 256),
    ("qwen_k100_r17", 1, 28, 4, [700], [17], 100, 100),
    ("evict_lowest", 1, 8, 2, [600], [5], 64, 59),
    ("recent_only", 1, 8, 2, [300], [9], 16, 0),
    ("clamped_n_sel", 2, 4, 4, [40, 500], [2, 1], 128, 128),
    ("k2048_many_chunks", 1, 32, 8, [5000], [10], 2048, 2048),
    ("tiles2", 4, 32, 8, [4000, 3000, 2500, 2600], [20, 1, 0, 7], 2080, 2080),
]


@pytest.mark.parametrize("case", PARTIAL_CASES, ids=[c[0] for c in PARTIAL_CASES])
def test_partial_attn_matches_oracle(rk, case):
    name, B, Hq, Hkv, lens, recent, k, n_sel = case
    say("partial case", case)
    cap = max(lens) + 8
    q, K, V = rand_case(300 + len(name), B, Hq, Hkv, cap)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    tail = [l - r for l, r in zip(lens, recent)]
    g = torch.Generator().manual_seed(5)
    idx = torch.full((B, Hkv, k), -1, dtype=torch.int32)
    for b in range(B):
        kk = min(k, tail[b])
        for h in range(Hkv):
            idx[b, h, :kk] = torch.randperm(tail[b], generator=g)[:kk].to(torch.int32)
    sK = torch.zeros(B, Hkv, k, 128, dtype=torch.bfloat16, device="cuda")
    sV = torch.zeros_like(sK)
    Kd, Vd = K.cuda(), V.cuda()
    rk.rk_gather_small_kv(geom, Kd, Vd, idx.cuda(), k, sK, sV)
    ws = rk.Workspace(geom, cap, k)
    out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    rk.rk_partial_attn(geom, q.cuda(), sK, sV, n_sel, Kd, Vd, torch.tensor(tail, dtype=torch.int32, device="cuda"),
                       torch.tensor(lens, dtype=torch.int32, device="cuda"), max(max(recent), 1), out, workspace=ws)
    torch.cuda.synchronize()
    rK = np.zeros((B, Hkv, k, 128), dtype=np.uint16); rV = rK.copy()
    oracle.gather_small_kv(gen.bf16_bits(K), gen.bf16_bits(V), idx.numpy(), rK, rV)
    o_ref = oracle.partial_attn(gen.bf16_bits(q), rK, rV, n_sel, gen.bf16_bits(K), gen.bf16_bits(V), tail, lens, scale)
    assert_out_close(gen.bf16_bits(out), o_ref, name)
    # an output that is only 2-byte aligned (the kernel stores 8 bytes at a time where it can): same bits
    raw = torch.zeros(B * Hq * 128 + 1, dtype=torch.bfloat16, device="cuda")
    out_odd = raw[1:].view(B, Hq, 128)
    assert out_odd.data_ptr() % 4 == 2
    rk.rk_partial_attn(geom, q.cuda(), sK, sV, n_sel, Kd, Vd, torch.tensor(tail, dtype=torch.int32, device="cuda"),
                       torch.tensor(lens, dtype=torch.int32, device="cuda"), max(max(recent), 1), out_odd, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out_odd, out) and raw[0].item() == 0


def test_partial_attn_fixed_size_per_sequence(rk):
    """rk_partial_attn_fixed: every sequence drops one selected row per row decoded since ITS refresh."""
    say("partial, fixed-size small cache, ragged")
    B, Hq, Hkv, k = 4, 8, 2, 200
    lens, recent = [900, 650, 300, 150], [0, 7, 31, 3]        # the last one: fewer than k rows were ever selected
    cap = max(lens) + 8
    q, K, V = rand_case(321, B, Hq, Hkv, cap)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    tail = [l - r for l, r in zip(lens, recent)]
    g = torch.Generator().manual_seed(6)
    idx = torch.full((B, Hkv, k), -1, dtype=torch.int32)
    for b in range(B):
        kk = min(k, tail[b])
        for h in range(Hkv):
            idx[b, h, :kk] = torch.randperm(tail[b], generator=g)[:kk].to(torch.int32)
    sK = torch.zeros(B, Hkv, k, 128, dtype=torch.bfloat16, device="cuda")
    sV = torch.zeros_like(sK)
    Kd, Vd = K.cuda(), V.cuda()
    rk.rk_gather_small_kv(geom, Kd, Vd, idx.cuda(), k, sK, sV)
    ws = rk.Workspace(geom, cap, k)
    out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    rk.rk_partial_attn_fixed(geom, q.cuda(), sK, sV, k, Kd, Vd, torch.tensor(tail, dtype=torch.int32, device="cuda"),
                             torch.tensor(lens, dtype=torch.int32, device="cuda"), max(recent), out, workspace=ws)
    torch.cuda.synchronize()
    rK = np.zeros((B, Hkv, k, 128), dtype=np.uint16); rV = rK.copy()
    oracle.gather_small_kv(gen.bf16_bits(K), gen.bf16_bits(V), idx.numpy(), rK, rV)
    got = gen.bf16_bits(out)
    for b in range(B):
        sl = slice(b, b + 1)
        o_ref = oracle.partial_attn(gen.bf16_bits(q)[sl], rK[sl], rV[sl], max(k - recent[b], 0), gen.bf16_bits(K)[sl],
                                    gen.bf16_bits(V)[sl], tail[sl], lens[sl], scale)
        assert_out_close(got[sl], o_ref, "b=%d" % b)


LAZY_CASES = [
    # name, B, Hq, Hkv, k, lens, recent, fixed
    ("llama_first_step", 2, 32, 8, 256, [3000, 1400], [1, 1], False),
    ("qwen_g7", 1, 28, 4, 300, [2500], [1], False),
    ("ragged_short_and_later", 4, 8, 2, 200, [900, 650, 300, 150], [1, 7, 31, 3], False),    # the last: fewer than k rows exist
    ("fixed_size", 3, 8, 2, 200, [900, 650, 150], [1, 5, 2], True),
    ("big_k_tail", 1, 8, 2, 2048, [9000], [9], False),
]


@pytest.mark.parametrize("case", LAZY_CASES, ids=[c[0] for c in LAZY_CASES])
def test_partial_attn_lazy_gathers_on_the_way(rk, case):
    """rk_partial_attn_lazy: the step's output equals the partial step on a gathered small cache, and the
    small cache it leaves equals the gather (bit for bit) on every row the step attended to."""
    name, B, Hq, Hkv, k, lens, recent, fixed = case
    say("lazy partial case", name)
    cap = max(lens) + 8
    q, K, V = rand_case(777 + len(name), B, Hq, Hkv, cap)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    tail = [l - r for l, r in zip(lens, recent)]
    g = torch.Generator().manual_seed(6)
    idx = torch.full((B, Hkv, k), -1, dtype=torch.int32)
    for b in range(B):
        kk = min(k, tail[b])
        for h in range(Hkv):
            idx[b, h, :kk] = torch.randperm(tail[b], generator=g)[:kk].to(torch.int32)
    marker_val = 0x7fc1                       # a NaN pattern: rows the step does not write must keep it
    sK = torch.full((B, Hkv, k, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    sV = torch.full_like(sK, float("nan"))
    Kd, Vd = K.cuda(), V.cuda()
    ws = rk.Workspace(geom, cap, k)
    out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    rk.rk_partial_attn_lazy(geom, q.cuda(), sK, sV, idx.cuda(), k, Kd, Vd, torch.tensor(tail, dtype=torch.int32, device="cuda"),
                            torch.tensor(lens, dtype=torch.int32, device="cuda"), max(recent), out, fixed_size=fixed,
                            workspace=ws)
    torch.cuda.synchronize()
    rK = np.zeros((B, Hkv, k, 128), dtype=np.uint16); rV = rK.copy()
    oracle.gather_small_kv(gen.bf16_bits(K), gen.bf16_bits(V), idx.numpy(), rK, rV)
    got, gK, gV = gen.bf16_bits(out), gen.bf16_bits(sK), gen.bf16_bits(sV)
    for b in range(B):
        sl = slice(b, b + 1)
        n_sel = max(k - recent[b], 0) if fixed else k
        o_ref = oracle.partial_attn(gen.bf16_bits(q)[sl], rK[sl], rV[sl], n_sel, gen.bf16_bits(K)[sl],
                                    gen.bf16_bits(V)[sl], tail[sl], lens[sl], scale)
        assert_out_close(got[sl], o_ref, "%s b=%d" % (name, b))
        n1 = min(n_sel, tail[b])
        assert (gK[b, :, :n1] == rK[b, :, :n1]).all() and (gV[b, :, :n1] == rV[b, :, :n1]).all()
        assert np.isnan(gen.bits_to_bf16(gK[b, :, n1:]).float().numpy()).all(), "rows beyond the attended ones were written"
        assert np.isnan(gen.bits_to_bf16(gV[b, :, n1:]).float().numpy()).all()
    # the next step runs on the small cache the lazy step left (only where it is complete: not the fixed-size case)
    if not fixed:
        lens2 = [l + 1 for l in lens]
        q2 = torch.randn(B, Hq, 128, generator=g).to(torch.bfloat16)
        sK2, sV2 = torch.nan_to_num(sK), torch.nan_to_num(sV)
        rk.rk_partial_attn(geom, q2.cuda(), sK2, sV2, k, Kd, Vd, torch.tensor(tail, dtype=torch.int32, device="cuda"),
                           torch.tensor(lens2, dtype=torch.int32, device="cuda"), max(recent) + 1, out, workspace=ws)
        torch.cuda.synchronize()
        o2 = oracle.partial_attn(gen.bf16_bits(q2), rK, rV, k, gen.bf16_bits(K), gen.bf16_bits(V), tail, lens2, scale)
        assert_out_close(gen.bf16_bits(out), o2, name + " next step")


def test_streaming_llm_policy_through_partial_attn(rk):
    """The StreamingLLM baseline of Appendix A.1 (4 sink tokens + K - 4 recent tokens) needs no kernel
    of its own: the sinks are a 4-row small cache, the recent tokens the tail of the full cache."""
    say("StreamingLLM policy on rk_partial_attn")
    B, Hq, Hkv, k, sinks = 2, 32, 8, 512, 4
    lens = [3000, 700]
    cap = 3008
    q, K, V = rand_case(612, B, Hq, Hkv, cap)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    idx = torch.arange(sinks, dtype=torch.int32).repeat(B, Hkv, 1).cuda()
    sK = torch.zeros(B, Hkv, sinks, 128, dtype=torch.bfloat16, device="cuda")
    sV = torch.zeros_like(sK)
    Kd, Vd = K.cuda(), V.cuda()
    rk.rk_gather_small_kv(geom, Kd, Vd, idx, sinks, sK, sV)
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    tail = sl - (k - sinks)                                   # the window slides with the sequence
    ws = rk.Workspace(geom, cap, k)
    out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    rk.rk_partial_attn(geom, q.cuda(), sK, sV, sinks, Kd, Vd, tail, sl, k - sinks, out, workspace=ws)
    torch.cuda.synchronize()
    # reference: plain attention over rows {0..3} and the last k - 4 rows, from the oracle's full-attention step
    got = gen.bf16_bits(out)
    Kb, Vb, qb = gen.bf16_bits(K), gen.bf16_bits(V), gen.bf16_bits(q)
    for b in range(B):
        rows = list(range(sinks)) + list(range(lens[b] - (k - sinks), lens[b]))
        o_ref, _, _ = oracle.full_attn(qb[b:b + 1], Kb[b:b + 1][:, :, rows], Vb[b:b + 1][:, :, rows], [len(rows)], scale)
        assert_out_close(got[b:b + 1], o_ref, "b=%d" % b)


def test_rows_past_the_end_are_never_used(rk):
    """Cache rows at and beyond seq_lens (and small-cache rows beyond the selected ones) hold NaN:
    nothing of them may reach the outputs, the weights or the selection."""
    say("NaN beyond the end")
    B, Hq, Hkv, cap, k = 2, 8, 2, 1400, 160       # k >= 128: the early loads of the first rows are taken
    lens = [1210, 70]
    q, K, V = rand_case(91, B, Hq, Hkv, cap)
    nan = torch.tensor(float("nan"), dtype=torch.bfloat16)
    for b in range(B):
        K[b, :, lens[b]:] = nan
        V[b, :, lens[b]:] = nan
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    ws = rk.Workspace(geom, cap, k)
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    Kd, Vd, qd = K.cuda(), V.cuda(), q.cuda()
    Kb, Vb = gen.bf16_bits(K), gen.bf16_bits(V)
    o_ref, w_ref, _ = oracle.full_attn(gen.bf16_bits(q), Kb, Vb, lens, scale)
    for want_w in (True, False):
        out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
        wt = torch.zeros(B, Hq, cap, dtype=torch.float32, device="cuda") if want_w else None
        rk.rk_full_attn(geom, qd, Kd, Vd, sl, cap, out, weights=wt, workspace=ws)
        torch.cuda.synchronize()
        assert_out_close(gen.bf16_bits(out), o_ref, "full, weights=%s" % want_w)
        if want_w:
            assert torch.isfinite(wt).all()
    out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    rk.rk_full_attn_select(geom, qd, Kd, Vd, sl, cap, out, k, 7, idx, workspace=ws)
    torch.cuda.synchronize()
    assert_out_close(gen.bf16_bits(out), o_ref, "fused")
    i_ref, _ = oracle.topk_select(w_ref.astype(np.float32), lens, Hkv, k, 7)
    G = Hq // Hkv
    for b in range(B):
        for g in range(Hkv):
            P = oracle.pooled_group_scores(w_ref[b, g * G:(g + 1) * G, :lens[b]].astype(np.float32), 7)
            assert_idx_equivalent(idx[b, g].cpu().numpy(), i_ref[b, g], P, lens[b], k, "b=%d g=%d" % (b, g))
    # partial step: the small cache holds NaN beyond the min(k, tail_start) gathered rows
    sK = torch.full((B, Hkv, k, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    sV = sK.clone()
    rk.rk_gather_small_kv(geom, Kd, Vd, idx, k, sK, sV)
    tail = [lens[0] - 4, lens[1] - 1]
    out = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    rk.rk_partial_attn(geom, qd, sK, sV, k, Kd, Vd, torch.tensor(tail, dtype=torch.int32, device="cuda"), sl, 4, out,
                       workspace=ws)
    torch.cuda.synchronize()
    rK = np.zeros((B, Hkv, k, 128), dtype=np.uint16); rV = rK.copy()
    oracle.gather_small_kv(Kb, Vb, idx.cpu().numpy(), rK, rV)
    o_part = oracle.partial_attn(gen.bf16_bits(q), rK, rV, k, Kb, Vb, tail, lens, scale)
    assert_out_close(gen.bf16_bits(out), o_part, "partial")


def test_query_sim_matches_oracle(rk):
    say("query_sim")
    B, Hq = 4, 28
    g = torch.Generator().manual_seed(8)
    q = torch.randn(B, Hq, 128, generator=g).to(torch.bfloat16)
    ref = torch.randn(B, 128, generator=g)
    ref[0] = q[0].float().mean(0)                    # sim = 1
    ref[1] = -q[1].float().mean(0) * 2               # sim = -1
    geom = rk.Geom(B, Hq, 4, 128, 1.0)
    for thr, force in ((0.5, False), (-2.0, False), (0.5, True)):
        q_ref = ref.clone().cuda()
        sim = torch.zeros(B, device="cuda"); need = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        rk.rk_query_sim(geom, q.cuda(), q_ref, thr, force, sim, need)
        torch.cuda.synchronize()
        s_ref, n_ref, r_ref = oracle.query_sim(gen.bf16_bits(q), ref.double().numpy(), thr, force)
        assert np.abs(sim.cpu().numpy() - s_ref).max() < 1e-5
        assert (need.cpu().numpy().astype(bool) == n_ref).all()
        assert np.abs(q_ref.cpu().numpy() - r_ref).max() < 1e-6


@pytest.mark.parametrize("heads", [(32, 8), (28, 4)], ids=["g4_tagged", "g7_ticketed"])
@pytest.mark.parametrize("fixed_size", [False, True], ids=["growing", "fixed_size"])
def test_partial_attn_triggered_equals_test_then_step(rk, heads, fixed_size):
    """rk_partial_attn_triggered against rk_query_sim followed by the partial step under its predicate
    (bit for bit: output, similarity, decision, reference), and the decisions against the oracle; sequences
    that fire and that do not in one batch; twice in a row on one workspace (the test's ticket is left clean)."""
    Hq, Hkv = heads
    B, k, cap = 5, 600, 2048
    say("partial_attn_triggered", heads, "fixed_size" if fixed_size else "growing")
    g = torch.Generator().manual_seed(77 + Hq)
    q = torch.randn(B, Hq, 128, generator=g).to(torch.bfloat16)
    ref = torch.randn(B, 128, generator=g)
    ref[0] = q[0].float().mean(0)                    # sim = 1: no full step
    ref[2] = q[2].float().mean(0) * 3 + 0.01 * ref[2]
    ref[3] = -q[3].float().mean(0)                   # sim = -1: full step
    K = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16).cuda()
    V = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16).cuda()
    sK = torch.randn(B, Hkv, k, 128, generator=g).to(torch.bfloat16).cuda()
    sV = torch.randn(B, Hkv, k, 128, generator=g).to(torch.bfloat16).cuda()
    lens = torch.tensor([1500, 1400, 2000, 900, 1207], dtype=torch.int32, device="cuda")
    tail = lens - torch.tensor([3, 9, 1, 5, 0], dtype=torch.int32, device="cuda")
    geom = rk.Geom(B, Hq, Hkv, 128, float(np.float32(1 / np.sqrt(128))))
    ws = rk.Workspace(geom, cap, k)
    thr = 0.5
    s_ref, n_ref, r_ref = oracle.query_sim(gen.bf16_bits(q), ref.double().numpy(), thr, False)
    assert n_ref.any() and not n_ref.all()
    qd = q.cuda()
    # the two calls
    q_ref_a = ref.clone().cuda(); sim_a = torch.zeros(B, device="cuda")
    need_a = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    out_a = torch.full((B, Hq, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    rk.rk_query_sim(geom, qd, q_ref_a, thr, False, sim_a, need_a)
    step = rk.rk_partial_attn_fixed if fixed_size else rk.rk_partial_attn
    step(geom, qd, sK, sV, k, K, V, tail, lens, 16, out_a, pred=need_a, pred_val=0, workspace=ws)
    torch.cuda.synchronize()
    assert (need_a.cpu().numpy().astype(bool) == n_ref).all()
    for rep in range(2):
        q_ref_b = ref.clone().cuda(); sim_b = torch.zeros(B, device="cuda")
        need_b = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        out_b = torch.full((B, Hq, 128), 7.0, dtype=torch.bfloat16, device="cuda")
        rk.rk_partial_attn_triggered(geom, qd, sK, sV, k, K, V, tail, lens, 16, out_b, q_ref_b, thr, sim_b, need_b,
                                     fixed_size=fixed_size, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(need_b, need_a) and torch.equal(sim_b, sim_a), rep
        assert torch.equal(q_ref_b, q_ref_a), rep
        assert torch.equal(out_b, out_a), rep
        assert np.abs(sim_b.cpu().numpy() - s_ref).max() < 1e-5
        assert np.abs(q_ref_b.cpu().numpy() - r_ref).max() < 1e-6
        fired = need_b.cpu().numpy().astype(bool)
        assert (gen.bf16_bits(out_b.cpu())[fired] == gen.bf16_bits(torch.tensor(7.0, dtype=torch.bfloat16))).all()
    # the workspace serves an ordinary step afterwards
    out_c = torch.zeros_like(out_a)
    step(geom, qd, sK, sV, k, K, V, tail, lens, 16, out_c, workspace=ws)
    torch.cuda.synchronize()
    keep = ~need_a.cpu().numpy().astype(bool)
    assert torch.equal(out_c[torch.from_numpy(keep).cuda()], out_a[torch.from_numpy(keep).cuda()])


@pytest.mark.parametrize("shape", [(1, 32, 8, 2048, 5), (1, 28, 4, 4096, 3), (4, 32, 8, 700, 9), (2, 8, 8, 1500, 0), (1, 32, 8, 2048, 40)],
                         ids=["llama_k2048", "qwen_k4096_two_rounds", "batch4_k700", "g1_k1500_no_tail", "llama_k2048_long_tail"])
def test_partial_attn_merge_by_slices_handover(rk, shape):
    """The merge by slices of the partial step with the bound on its re-reads at 0 (every workgroup leaves its share
    to the one that publishes last), at 1 and 2 (some do, some do not) and at its default: the same bits every time,
    against the oracle once, and the workspace left clean for the next call (also rk_full_attn without weights)."""
    B, Hq, Hkv, k, recent = shape
    say("merge_by_slices_handover", shape)
    cap = 6000
    g = torch.Generator().manual_seed(500 + k + B)
    q = torch.randn(B, Hq, 128, generator=g).to(torch.bfloat16)
    K = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16)
    sK = torch.randn(B, Hkv, k, 128, generator=g).to(torch.bfloat16)
    sV = torch.randn(B, Hkv, k, 128, generator=g).to(torch.bfloat16)
    lens_h = np.array([5000 - 37 * b for b in range(B)], dtype=np.int32)
    tail_h = lens_h - recent
    geom = rk.Geom(B, Hq, Hkv, 128, float(np.float32(1 / np.sqrt(128))))
    ws = rk.Workspace(geom, cap, k)
    dK, dV, dsK, dsV, dq = K.cuda(), V.cuda(), sK.cuda(), sV.cuda(), q.cuda()
    lens, tail = torch.from_numpy(lens_h).cuda(), torch.from_numpy(tail_h).cuda()
    outs = []
    try:
        for spin in (256, 0, 1, 2, 0, 256):
            rk.rk_debug_set_slice_spin(spin)
            out = torch.full((B, Hq, 128), 3.0, dtype=torch.bfloat16, device="cuda")
            rk.rk_partial_attn(geom, dq, dsK, dsV, k, dK, dV, tail, lens, max(recent, 1), out, workspace=ws)
            torch.cuda.synchronize()
            outs.append(out.cpu())
        # rk_full_attn without weights over short rows takes the same merge
        full = []
        for spin in (256, 0, 1):
            rk.rk_debug_set_slice_spin(spin)
            out = torch.full((B, Hq, 128), 3.0, dtype=torch.bfloat16, device="cuda")
            rk.rk_full_attn(geom, dq, dK, dV, lens, int(lens_h.max()), out, workspace=ws)
            torch.cuda.synchronize()
            full.append(out.cpu())
    finally:
        rk.rk_debug_set_slice_spin(256)
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
    for o in full[1:]:
        assert torch.equal(o, full[0])
    o_ref = oracle.partial_attn(gen.bf16_bits(q), gen.bf16_bits(sK), gen.bf16_bits(sV), k, gen.bf16_bits(K), gen.bf16_bits(V),
                                tail_h.tolist(), lens_h.tolist(), geom.scale)
    assert_out_close(gen.bf16_bits(outs[0]), o_ref, "merge by slices")
    f_ref, _, _ = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), lens_h.tolist(), geom.scale)
    assert_out_close(gen.bf16_bits(full[0]), f_ref, "full attention, merge by slices")


def test_partial_attn_on_two_streams_at_once(rk):
    """Partial steps of two independent caches enqueued on two streams, so that their launches can share the chip:
    a workgroup of the merge by slices then may find its compute unit only after others of its launch have waited
    for it; the waits are bounded and hand over, and the results are those of the same calls one after the other."""
    say("partial_attn_two_streams")
    B, Hq, Hkv, k, cap = 1, 32, 8, 2048, 6000
    geom = rk.Geom(B, Hq, Hkv, 128, float(np.float32(1 / np.sqrt(128))))
    g = torch.Generator(device="cuda").manual_seed(91)
    sets = []
    for i in range(2):
        K = torch.randn(B, Hkv, cap, 128, generator=g, device="cuda").to(torch.bfloat16)
        V = torch.randn(B, Hkv, cap, 128, generator=g, device="cuda").to(torch.bfloat16)
        sK = torch.randn(B, Hkv, k, 128, generator=g, device="cuda").to(torch.bfloat16)
        sV = torch.randn(B, Hkv, k, 128, generator=g, device="cuda").to(torch.bfloat16)
        q = torch.randn(B, Hq, 128, generator=g, device="cuda").to(torch.bfloat16)
        lens = torch.full((B,), 5000 + i, dtype=torch.int32, device="cuda")
        sets.append(dict(K=K, V=V, sK=sK, sV=sV, q=q, lens=lens, tail=lens - 7, ws=rk.Workspace(geom, cap, k),
                         out=torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")))

    def step(d, stream=None):
        rk.rk_partial_attn(geom, d["q"], d["sK"], d["sV"], k, d["K"], d["V"], d["tail"], d["lens"], 8, d["out"],
                           workspace=d["ws"], stream=stream)
    want = []
    for d in sets:
        step(d)
        torch.cuda.synchronize()
        want.append(d["out"].clone())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(20):
        for d in sets:
            d["out"].zero_()
        torch.cuda.synchronize()
        for _ in range(8):                      # a few launches deep on either stream
            for d, st in zip(sets, streams):
                step(d, stream=st)
        torch.cuda.synchronize()
        for d, w in zip(sets, want):
            assert torch.equal(d["out"], w), rep


# ----------------------------------------------------------------------------- whole loop
def run_gpu_loop(rk, w: gen.Workload, layer: int, K, V, q_steps, new_k, new_v, lens0, evict_lowest=False,
                 scores_only=False):
    """Drive the library through the decode schedule; returns per-step outputs and snapshots."""
    dev = "cuda"
    geom = rk.Geom(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.scale)
    Kd, Vd = K.to(dev).clone(), V.to(dev).clone()
    sl = lens0.to(dev).clone()
    lay = rk.RefreshKVLayer(geom, Kd, Vd, sl, int(lens0.max()), w.k_small, w.stride, pool_w=w.pool_w,
                            dynamic=w.dynamic, threshold=w.threshold, evict_lowest=evict_lowest,
                            scores_only_refresh=scores_only)
    qd, nk, nv = q_steps.to(dev), new_k.to(dev), new_v.to(dev)
    outs, idxs, needs, sims, kinds = [], [], [], [], []
    for t in range(w.n_steps + 1):
        if t >= 1:
            lay.append(nk[t - 1], nv[t - 1])
        kinds.append(lay.step(t, qd[t]))
        outs.append(lay.out.clone()); idxs.append(lay.idx.clone())
        needs.append(lay.need_full.clone()); sims.append(lay.sim.clone())
    torch.cuda.synchronize()
    return dict(outs=np.stack([gen.bf16_bits(o) for o in outs]), idx=[i.cpu().numpy() for i in idxs],
                need=np.stack([n.cpu().numpy() for n in needs]), sims=np.stack([s.cpu().numpy() for s in sims]),
                kinds=kinds, K=gen.bf16_bits(Kd), V=gen.bf16_bits(Vd), lens=sl.cpu().numpy())


def compare_with_oracle(w: gen.Workload, layer: int, got, K, V, q, nk, nv, lens0, evict_lowest=False, scores_only=False):
    """One layer's GPU run against the oracle's decode loop on the same inputs."""
    ref = oracle.decode_loop(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), gen.bf16_bits(nk),
                             gen.bf16_bits(nv), lens0.numpy(), w.scale, w.k_small, w.stride, pool_w=w.pool_w,
                             dynamic=w.dynamic, threshold=w.threshold, evict_lowest=evict_lowest,
                             scores_only_refresh=scores_only)
    assert (got["K"] == ref["k"]).all() and (got["V"] == ref["v"]).all() and (got["lens"] == ref["lens"]).all()
    G = w.group
    n_diff = 0
    lens = lens0.numpy().astype(np.int64).copy()
    last_full_scores = {}
    for t in range(w.n_steps + 1):
        if t >= 1:
            lens += 1
        for b in range(w.batch):
            if ref["full"][t, b]:
                # oracle pooled scores of this refresh, for the gap test on indices
                wts = oracle.full_attn(gen.bf16_bits(q[t, b:b + 1]), ref["k"][b:b + 1], ref["v"][b:b + 1],
                                       [lens[b]], w.scale)[1].astype(np.float32)
                for g in range(w.n_kv_heads):
                    last_full_scores[(b, g)] = (oracle.pooled_group_scores(wts[0, g * G:(g + 1) * G], w.pool_w),
                                                int(lens[b]))
            if w.dynamic and t >= 1 and t % w.stride == 0:
                s_ref = ref["sims"][t, b]
                assert abs(got["sims"][t, b] - s_ref) < 1e-5
                if abs(s_ref - w.threshold) > 1e-5:
                    assert bool(got["need"][t, b]) == bool(ref["full"][t, b]), "trigger decision differs at t=%d" % t
            for g in range(w.n_kv_heads):
                P, n = last_full_scores[(b, g)]
                n_diff += assert_idx_equivalent(got["idx"][t][b, g], ref["idx"][t][b, g], P, n, w.k_small,
                                                "layer %d t=%d b=%d g=%d" % (layer, t, b, g))
        assert_out_close(got["outs"][t], ref["outs"][t], "%s layer %d t=%d" % (w.name, layer, t))
    return ref, n_diff


def check_loop(rk, w: gen.Workload, evict_lowest=False, scores_only=False):
    K, V = gen.make_kv(w, 0)
    q = gen.make_queries(w, 0)
    nk, nv = gen.make_new_rows(w, 0)
    lens0 = gen.seq_lens(w)
    got = run_gpu_loop(rk, w, 0, K, V, q, nk, nv, lens0, evict_lowest, scores_only)
    ref, n_diff = compare_with_oracle(w, 0, got, K, V, q, nk, nv, lens0, evict_lowest, scores_only)
    return got, ref, n_diff


def check_model_loop(rk, w: gen.Workload, n_layers: int, evict_lowest=False, scores_only=False, overlap=False,
                     gen_device="cpu"):
    """The same schedule through rk_decode_step: all layers of a step in one call.  gen_device="cuda":
    the caches are drawn on the GPU (large workloads) and copied to the host for the oracle."""
    dev = "cuda"
    geom = rk.Geom(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.scale)
    lens0 = gen.seq_lens(w)
    data, kv = [], []
    for l in range(n_layers):
        Kg, Vg = gen.make_kv(w, l, device=gen_device)
        data.append(((Kg.cpu(), Vg.cpu()) if gen_device != "cpu" else (Kg, Vg), gen.make_queries(w, l), gen.make_new_rows(w, l)))
        kv.append((Kg.to(dev).clone(), Vg.to(dev).clone()) if gen_device == "cpu" else (Kg, Vg))
    sl = lens0.to(dev).clone()
    model = rk.RefreshKVModel(geom, kv, sl, int(lens0.max()), w.k_small, w.stride, pool_w=w.pool_w, dynamic=w.dynamic,
                              threshold=w.threshold, evict_lowest=evict_lowest, scores_only_refresh=scores_only)
    if overlap == "batched":
        model.batched_refresh()
    elif overlap:
        model.overlap_refresh(2)
    q_all = torch.stack([d[1] for d in data], dim=1).to(dev).contiguous()            # [T+1, n_layers, B, Hq, D]
    nk_all = [d[2][0].to(dev) for d in data]
    nv_all = [d[2][1].to(dev) for d in data]
    B, Hkv, D = w.batch, w.n_kv_heads, w.head_dim
    outs, idxs, needs, sims, kinds = [], [], [], [], []
    for t in range(w.n_steps + 1):
        if t >= 1:
            pos = sl.to(torch.int64)[:, None, None, None].expand(B, Hkv, 1, D)
            for l in range(n_layers):
                kv[l][0].scatter_(2, pos, nk_all[l][t - 1][:, :, None, :])
                kv[l][1].scatter_(2, pos, nv_all[l][t - 1][:, :, None, :])
            sl += 1
            model.advance()
        kinds.append(model.step(t, q_all[t]))
        outs.append(model.out.clone()); idxs.append(model.idx.clone())
        needs.append(model.need_full.clone()); sims.append(model.sim.clone())
    torch.cuda.synchronize()
    n_full = model.n_full.cpu().numpy()
    refs = []
    for l in range(n_layers):
        got = dict(outs=np.stack([gen.bf16_bits(o[l]) for o in outs]), idx=[i[l].cpu().numpy() for i in idxs],
                   need=np.stack([n[l].cpu().numpy() for n in needs]), sims=np.stack([s_[l].cpu().numpy() for s_ in sims]),
                   kinds=kinds, K=gen.bf16_bits(kv[l][0]), V=gen.bf16_bits(kv[l][1]), lens=sl.cpu().numpy())
        (K, V), q, (nk, nv) = data[l]
        ref, _ = compare_with_oracle(w, l, got, K, V, q, nk, nv, lens0, evict_lowest, scores_only)
        # refresh counters kept on the GPU: wherever no decision sat on the threshold
        near = np.zeros(w.batch, dtype=bool)
        if w.dynamic:
            sims_ref = ref["sims"]
            near = (np.abs(np.nan_to_num(sims_ref, nan=9.0) - w.threshold) <= 1e-5).any(axis=0)
        assert (n_full[l][~near] == ref["full"].sum(axis=0)[~near]).all(), "refresh count of layer %d" % l
        refs.append(ref)
    return kinds, n_full, refs


def test_score_select_matches_oracle(rk):
    """rk_score_select: weights, lse and selection from the keys alone (no value pointer at all)."""
    cases = [("llama_ragged", 2, 32, 8, [3100, 1029], 3200, 256, 7), ("qwen_g7", 1, 28, 4, [2500], 2560, 128, 7),
             ("g8_pool1_short_empty", 3, 16, 2, [130, 0, 5], 256, 16, 1), ("two_rounds", 1, 4, 1, [40000], 40064, 512, 7)]
    for name, B, Hq, Hkv, lens, cap, k, pool_w in cases:
        say("score_select case", name)
        q, K, _ = rand_case(400 + len(name), B, Hq, Hkv, cap)
        K[:, :, ::97] *= 3.0
        for b in range(B):
            K[b, :, lens[b]:] = float("nan")             # rows past the end must not matter
        scale = float(np.float32(1 / np.sqrt(128)))
        geom = rk.Geom(B, Hq, Hkv, 128, scale)
        ws = rk.Workspace(geom, cap, k)
        sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
        w_ref, lse_ref = oracle.attn_scores(gen.bf16_bits(q), gen.bf16_bits(K), lens, scale)
        i_ref, _ = oracle.topk_select(w_ref.astype(np.float32), lens, Hkv, k, pool_w)
        G = Hq // Hkv
        for want_w in (True, False):
            wt = torch.full((B, Hq, cap), -7.0, dtype=torch.float32, device="cuda") if want_w else None
            lse = torch.full((B, Hq), 123.0, dtype=torch.float32, device="cuda")
            idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
            rk.rk_score_select(geom, q.cuda(), K.cuda(), sl, max(max(lens), 1), k, pool_w, idx, weights=wt, lse=lse,
                               workspace=ws)
            torch.cuda.synchronize()
            idx_n, lse_n = idx.cpu().numpy(), lse.cpu().numpy()
            for b in range(B):
                n = lens[b]
                if n == 0:
                    assert (lse_n[b] == -np.inf).all() and (idx_n[b] == -1).all()
                    continue
                assert np.abs(lse_n[b] - lse_ref[b]).max() < 1e-5
                if want_w:
                    wn = wt[b].cpu().numpy()
                    assert (np.abs(wn[:, :n] - w_ref[b, :, :n]) / w_ref[b, :, :n]).max() < 1e-5
                    assert (wn[:, n:] == -7.0).all()
                for g in range(Hkv):
                    P = oracle.pooled_group_scores(w_ref[b, g * G:(g + 1) * G, :n].astype(np.float32), pool_w)
                    assert_idx_equivalent(idx_n[b, g], i_ref[b, g], P, n, k, "%s b=%d g=%d" % (name, b, g))


def test_window_select_matches_oracle(rk):
    """rk_window_select: votes of the last W prompt tokens (causal, summed per head) and the selection
    on them; W = 1 must select what rk_score_select selects."""
    cases = [("llama_w8", 2, 32, 8, [3100, 1029], 3200, 256, 7, 8), ("qwen_g7_w5", 1, 28, 4, [2500], 2560, 128, 7, 5),
             ("g8_w32_short_empty", 3, 16, 2, [130, 0, 5], 256, 16, 1, 32), ("w1", 1, 8, 2, [5000], 5056, 64, 7, 1),
             ("two_rounds_w32", 1, 4, 1, [40000], 40064, 512, 7, 32), ("mha_w3", 1, 4, 4, [700], 768, 32, 7, 3),
             ("g3_w4", 1, 6, 2, [1000], 1024, 50, 7, 4)]
    for name, B, Hq, Hkv, lens, cap, k, pool_w, W in cases:
        say("window_select case", name)
        _, K, _ = rand_case(500 + len(name), B, Hq, Hkv, cap)
        gq = torch.Generator().manual_seed(900 + W)
        qw = torch.randn(B, W, Hq, 128, generator=gq).to(torch.bfloat16)
        K[:, :, ::97] *= 3.0
        for b in range(B):
            K[b, :, lens[b]:] = float("nan")             # rows past the end must not matter
        scale = float(np.float32(1 / np.sqrt(128)))
        geom = rk.Geom(B, Hq, Hkv, 128, scale)
        ws = rk.Workspace(geom, cap, k)
        sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
        v_ref = oracle.window_votes(gen.bf16_bits(qw), gen.bf16_bits(K), lens, scale)
        i_ref, _ = oracle.topk_select(v_ref.astype(np.float32), lens, Hkv, k, pool_w)
        G = Hq // Hkv
        max_len = max(max(lens), 1)
        for want_v in (True, False):
            vt = torch.full((B, Hq, cap), -7.0, dtype=torch.float32, device="cuda") if want_v else None
            idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
            rk.rk_window_select(geom, qw.cuda(), K.cuda(), sl, max_len, k, pool_w, idx, votes=vt, workspace=ws)
            torch.cuda.synchronize()
            idx_n = idx.cpu().numpy()
            for b in range(B):
                n = lens[b]
                if n == 0:
                    assert (idx_n[b] == -1).all()
                    continue
                if want_v:
                    vn = vt[b].cpu().numpy()
                    assert (np.abs(vn[:, :n] - v_ref[b, :, :n]) / v_ref[b, :, :n]).max() < 1e-5
                    assert (vn[:, n:] == -7.0).all()
                for g in range(Hkv):
                    P = oracle.pooled_group_scores(v_ref[b, g * G:(g + 1) * G, :n].astype(np.float32), pool_w)
                    assert_idx_equivalent(idx_n[b, g], i_ref[b, g], P, n, k, "%s b=%d g=%d" % (name, b, g))
        if W == 1:
            idx1 = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
            rk.rk_score_select(geom, qw[:, 0].contiguous().cuda(), K.cuda(), sl, max_len, k, pool_w, idx1, workspace=ws)
            torch.cuda.synchronize()
            P = oracle.pooled_group_scores(v_ref[0, :G, :lens[0]].astype(np.float32), pool_w)
            assert_idx_equivalent(idx1.cpu().numpy()[0, 0], idx_n[0, 0], P, lens[0], k, "w1 vs score_select")


def test_window_select_predicate(rk):
    """A sequence the predicate switches off keeps its idx and votes; the other one is selected as usual."""
    B, Hq, Hkv, cap, k, W = 2, 8, 2, 1536, 64, 4
    lens = [1500, 1400]
    _, K, _ = rand_case(61, B, Hq, Hkv, cap)
    qw = torch.randn(B, W, Hq, 128, generator=torch.Generator().manual_seed(62)).to(torch.bfloat16)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    ws = rk.Workspace(geom, cap, k)
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    pred = torch.tensor([1, 0], dtype=torch.int32, device="cuda")
    idx = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    votes = torch.full((B, Hq, cap), -7.0, dtype=torch.float32, device="cuda")
    rk.rk_window_select(geom, qw.cuda(), K.cuda(), sl, max(lens), k, 7, idx, votes=votes, pred=pred, pred_val=1, workspace=ws)
    torch.cuda.synchronize()
    assert (idx[1] == -5).all() and (votes[1] == -7.0).all()
    v_ref = oracle.window_votes(gen.bf16_bits(qw), gen.bf16_bits(K), lens, scale)
    i_ref, _ = oracle.topk_select(v_ref.astype(np.float32), lens, Hkv, k, 7)
    G = Hq // Hkv
    for g in range(Hkv):
        P = oracle.pooled_group_scores(v_ref[0, g * G:(g + 1) * G, :lens[0]].astype(np.float32), 7)
        assert_idx_equivalent(idx.cpu().numpy()[0, g], i_ref[0, g], P, lens[0], k, "g=%d" % g)
    # the workspace is left clean: the same call without a predicate selects both sequences correctly
    rk.rk_window_select(geom, qw.cuda(), K.cuda(), sl, max(lens), k, 7, idx, workspace=ws)
    torch.cuda.synchronize()
    for b in range(B):
        for g in range(Hkv):
            P = oracle.pooled_group_scores(v_ref[b, g * G:(g + 1) * G, :lens[b]].astype(np.float32), 7)
            assert_idx_equivalent(idx.cpu().numpy()[b, g], i_ref[b, g], P, lens[b], k, "b=%d g=%d" % (b, g))


def test_prefill_init_window_one_equals_initial_full_step(rk):
    """Section 2.2 "Prefilling stage": with an observation window of one, starting the small cache
    from the last prompt token's query is what the t = 0 full step of the schedule does."""
    from paper_2411_05787_amd.schedule import RefreshKVLayer
    B, Hq, Hkv, cap, k = 2, 16, 4, 2304, 96
    lens = [2200, 517]
    q, K, V = rand_case(77, B, Hq, Hkv, cap)
    geom = rk.Geom(B, Hq, Hkv, 128, float(np.float32(1 / np.sqrt(128))))
    layers = []
    for _ in range(2):
        sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
        layers.append(RefreshKVLayer(geom, K.cuda(), V.cuda(), sl, max(lens), k, 4, dynamic=True, threshold=0.5))
    layers[0].step(0, q.cuda())
    layers[1].prefill_init(q[:, None].contiguous().cuda())
    torch.cuda.synchronize()
    a, b = layers
    w_ref, _ = oracle.attn_scores(gen.bf16_bits(q), gen.bf16_bits(K), lens, geom.scale)
    ia, ib = a.idx.cpu().numpy(), b.idx.cpu().numpy()
    for bi in range(B):
        for g in range(Hkv):
            P = oracle.pooled_group_scores(w_ref[bi, g * 4:(g + 1) * 4, :lens[bi]].astype(np.float32), 7)
            assert_idx_equivalent(ib[bi, g], ia[bi, g], P, lens[bi], k, "b=%d g=%d" % (bi, g))
    same = torch.from_numpy(ia == ib).cuda()                 # rows may differ only where near-ties swapped
    assert same.float().mean().item() > 0.95
    assert torch.equal(a.small_K[same], b.small_K[same]) and torch.equal(a.small_V[same], b.small_V[same])
    assert torch.equal(a.tail_start, b.tail_start) and torch.equal(a.q_ref, b.q_ref)


def test_loop_scores_only_refresh(rk):
    """Section 4.3 "w/o full attention": refresh steps attend to the rebuilt small cache alone."""
    w = gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], n_steps=12)
    say("loop, scores-only refresh", w)
    got, ref, n_diff = check_loop(rk, w, scores_only=True)
    assert got["kinds"][0] == "full" and got["kinds"][4] == "full" and got["kinds"][5] == "partial"
    wq = gen.shrink(gen.WORKLOADS["cfg3_qwen_64k_dynamic"], context=3000, k_small=256, n_steps=22, n_layers=1)
    say("loop, scores-only refresh, dynamic", wq)
    got, ref, _ = check_loop(rk, wq, scores_only=True)
    assert "both" in got["kinds"]


def test_decode_step_driver_fixed_and_dynamic(rk):
    """rk_decode_step: three layers per call, fixed stride and the trigger, against the oracle."""
    w = gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], n_steps=9)
    say("decode_step driver, fixed stride", w.name)
    kinds, n_full, _ = check_model_loop(rk, w, 3)
    assert kinds[:5] == ["full", "partial", "partial", "partial", "full"]
    assert (n_full == 3).all()                       # t = 0, 4, 8
    wq = gen.shrink(gen.WORKLOADS["cfg3_qwen_64k_dynamic"], context=3000, k_small=256, n_steps=25, batch=2)
    say("decode_step driver, dynamic, fixed-size small cache", wq.name)
    kinds, n_full, refs = check_model_loop(rk, wq, 3, evict_lowest=True)
    assert kinds.count("both") == 5 and kinds[0] == "full"
    fired = np.stack([r["full"][1:].sum(axis=0) for r in refs])
    say("  refreshes per (layer, sequence) after the initialisation:", fired.tolist())
    assert fired.min() < fired.max() or fired.max() < 5, "layers decide on their own"
    say("decode_step driver, refresh on a second stream (native events)")
    kinds, n_full, _ = check_model_loop(rk, gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], n_steps=9), 5, overlap=True)
    assert kinds[:5] == ["full", "partial", "partial", "partial", "full"] and (n_full == 3).all()
    check_model_loop(rk, wq, 3, evict_lowest=True, overlap=True)
    say("decode_step driver, refreshes batched over the layers")
    kinds, n_full, _ = check_model_loop(rk, gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], n_steps=9), 5, overlap="batched")
    assert kinds[:5] == ["full", "partial", "partial", "partial", "full"] and (n_full == 3).all()
    check_model_loop(rk, wq, 3, evict_lowest=True, overlap="batched")
    check_model_loop(rk, gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], n_steps=9, batch=3), 34, overlap="batched")   # two launches of 32 + 2 layers
    say("decode_step driver, scores-only refresh")
    check_model_loop(rk, gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], n_steps=5), 2, scores_only=True)


def test_host_bounds_under_the_trigger_schedule(rk):
    """Under the trigger's schedule the host never learns of a refresh, so its bound on the rows decoded since
    one grows by a row per step: a partial step given a bound far beyond the real count must still fit a
    workspace sized for the context (what it uses does not grow with the bound) and give the result of the
    tight bound (another launch shape: equal to within the bar, not bit for bit), and tighten_recent_bound()
    brings the bound back from the GPU's own counts."""
    say("host bounds under the trigger schedule")
    w = gen.shrink(gen.WORKLOADS["cfg3_qwen_64k_dynamic"], context=3000, k_small=256, n_steps=12)
    geom = rk.Geom(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.scale)
    lens0 = gen.seq_lens(w)
    kv = [tuple(t.cuda() for t in gen.make_kv(w, l)) for l in range(2)]
    sl = lens0.cuda()
    model = rk.RefreshKVModel(geom, kv, sl, int(lens0.max()), w.k_small, w.stride, pool_w=w.pool_w, dynamic=True,
                              threshold=w.threshold)
    q_all = torch.stack([gen.make_queries(w, l) for l in range(2)], dim=1).cuda().contiguous()
    for t in range(w.n_steps + 1):
        if t >= 1:
            sl += 1
            model.advance()
        model.step(t, q_all[t])
    torch.cuda.synchronize()
    assert model.recent_bound == w.n_steps                       # grew with every step: no full step by schedule after t = 0
    real = int((sl.unsqueeze(0) - model.tail_start).max().item())
    assert model.tighten_recent_bound() == real <= w.n_steps
    out_tight = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.bfloat16, device="cuda")
    out_loose = torch.zeros_like(out_tight)
    args = (geom, q_all[w.n_steps, 0], model.small_K[0], model.small_V[0], w.k_small, kv[0][0], kv[0][1], model.tail_start[0], sl)
    rk.rk_partial_attn(*args, max(real, 1), out_tight, workspace=model.ws)
    rk.rk_partial_attn(*args, 1_000_000, out_loose, workspace=model.ws)     # a bound far beyond the context
    torch.cuda.synchronize()
    assert_out_close(gen.bf16_bits(out_loose), gen.bf16_bits(out_tight), "loose against tight bound")


def test_deferred_pooling_and_batched_refresh(rk):
    """rk_full_attn_deferred per layer + rk_refresh_batched(pool_w): out, lse, idx, small cache, tail_start and
    refresh counters against the oracle and, bit for bit, against rk_full_attn_select + rk_gather_small_kv per
    layer; ragged batch with an empty sequence, three layers, then once more with every layer's need_full as
    the predicate (workspaces left clean by the first pass)."""
    import ctypes as C
    from paper_2411_05787_amd.binding import _LayerState, layer_state
    B, Hq, Hkv, cap, k, pool_w, n_layers = 3, 8, 2, 2300, 96, 7, 3
    lens = [2300, 0, 1111]
    say("deferred pooling + batched refresh", B, Hq, Hkv, lens, k)
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    G = Hq // Hkv
    data = [rand_case(900 + l, B, Hq, Hkv, cap) for l in range(n_layers)]
    dev = [tuple(x.cuda() for x in d) for d in data]
    refs = []
    for q, K, V in data:
        o_ref, w_ref, lse_ref = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), lens, scale)
        i_ref, _ = oracle.topk_select(w_ref.astype(np.float32), lens, Hkv, k, pool_w)
        refs.append((o_ref, w_ref, lse_ref, i_ref))

    def fresh():
        return dict(out=[torch.full((B, Hq, 128), 3.0, dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)],
                    lse=[torch.full((B, Hq), 9.0, dtype=torch.float32, device="cuda") for _ in range(n_layers)],
                    idx=[torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda") for _ in range(n_layers)],
                    sK=[torch.zeros(B, Hkv, k, 128, dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)],
                    sV=[torch.zeros(B, Hkv, k, 128, dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)],
                    tail=[torch.full((B,), -3, dtype=torch.int32, device="cuda") for _ in range(n_layers)],
                    n_full=[torch.zeros(B, dtype=torch.int32, device="cuda") for _ in range(n_layers)])

    wss = [rk.Workspace(geom, cap, k) for _ in range(n_layers)]
    ws_ptrs = (C.c_void_p * n_layers)(*[w_.ptr for w_ in wss])
    ws_bytes = min(w_.nbytes for w_ in wss)
    need = [torch.tensor(v, dtype=torch.int32, device="cuda") for v in ([1, 1, 0], [0, 0, 1], [1, 0, 1])]
    for use_pred, agg in ((False, "max"), (True, "max"), (False, "mean")):
        agg_id = {"max": rk.RK_AGG_MAX, "mean": rk.RK_AGG_MEAN}[agg]
        a, b_ = fresh(), fresh()
        states = (_LayerState * n_layers)(*[layer_state(geom, dev[l][1], dev[l][2], a["sK"][l], a["sV"][l], a["idx"][l],
                                                        a["tail"][l], need_full=need[l], n_full=a["n_full"][l], k=k)
                                            for l in range(n_layers)])
        for l in range(n_layers):
            pr = need[l] if use_pred else None
            rk.rk_full_attn_deferred(geom, dev[l][0], dev[l][1], dev[l][2], sl, cap, a["out"][l], lse=a["lse"][l],
                                     pred=pr, pred_val=1, workspace=wss[l])
        rk.rk_refresh_batched(geom, states, ws_ptrs, ws_bytes, sl, cap, k, pool_w=pool_w, agg=agg_id, by_need_full=use_pred)
        for l in range(n_layers):       # the per-layer path on the first workspace
            pr = need[l] if use_pred else None
            rk.rk_full_attn_select(geom, dev[l][0], dev[l][1], dev[l][2], sl, cap, b_["out"][l], k, pool_w, b_["idx"][l],
                                   lse=b_["lse"][l], agg=agg_id, pred=pr, pred_val=1, workspace=wss[0])
            rk.rk_gather_small_kv(geom, dev[l][1], dev[l][2], b_["idx"][l], k, b_["sK"][l], b_["sV"][l], seq_lens=sl,
                                  tail_start=b_["tail"][l], pred=pr, pred_val=1)
        torch.cuda.synchronize()
        for l in range(n_layers):
            o_ref, w_ref, lse_ref, i_ref = refs[l]
            for key in ("out", "idx", "sK", "sV", "tail"):
                assert torch.equal(a[key][l], b_[key][l]), "layer %d: %s differs from the per-layer path" % (l, key)
            assert (a["lse"][l] - b_["lse"][l]).abs().nan_to_num(0.0).max().item() <= 1e-6
            on = need[l].cpu().numpy() == 1 if use_pred else np.ones(B, bool)
            got, idx_n = gen.bf16_bits(a["out"][l]), a["idx"][l].cpu().numpy()
            for b in range(B):
                if not on[b]:
                    assert (a["out"][l][b] == 3.0).all() and (idx_n[b] == -5).all() and a["tail"][l][b].item() == -3
                    assert a["n_full"][l][b].item() == 0
                    continue
                assert a["tail"][l][b].item() == lens[b] and a["n_full"][l][b].item() == 1
                assert_out_close(got[b:b + 1], o_ref[b:b + 1], "layer %d b %d" % (l, b))
                n = lens[b]
                if n == 0:
                    assert (idx_n[b] == -1).all()
                    continue
                for g in range(Hkv):
                    P = oracle.pooled_group_scores(w_ref[b, g * G:(g + 1) * G, :n].astype(np.float32), pool_w, agg=agg)
                    i_want = i_ref[b, g] if agg == "max" else oracle.topk_select(w_ref[b:b + 1, g * G:(g + 1) * G].astype(np.float32),
                                                                                 [n], 1, k, pool_w, agg=agg)[0][0, 0]
                    assert_idx_equivalent(idx_n[b, g], i_want, P, n, k, "deferred %s l=%d b=%d g=%d" % (agg, l, b, g))


def test_refresh_on_second_stream_stack(rk):
    """RefreshKVStack: selection and gather of a full step on a second stream (two workspaces in turn), or
    for all layers at once after the last layer's attention (rk_refresh_batched, with the pooling done per
    layer or deferred to it as well); eager and replayed from a HIP graph."""
    w = gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], n_steps=9)
    n_layers, dev = 5, "cuda"
    geom = rk.Geom(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.scale)
    lens0 = gen.seq_lens(w)
    data = [(gen.make_kv(w, l), gen.make_queries(w, l), gen.make_new_rows(w, l)) for l in range(n_layers)]
    for use_graph, batched, deferred in ((False, False, False), (True, False, False), (False, True, False),
                                         (True, True, False), (False, True, True), (True, True, True)):
        say("refresh of a layer stack, graph =", use_graph, "batched =", batched, "pooling deferred =", deferred)
        kv = [(d[0][0].to(dev).clone(), d[0][1].to(dev).clone()) for d in data]
        sl = lens0.to(dev).clone()
        ws = rk.Workspace(geom, w.capacity, w.k_small)
        layers = [rk.RefreshKVLayer(geom, kv[l][0], kv[l][1], sl, int(lens0.max()), w.k_small, w.stride, pool_w=w.pool_w,
                                    workspace=ws) for l in range(n_layers)]
        stack = rk.RefreshKVStack(layers, n_workspaces=2 if use_graph else 0, batched=batched,
                                  deferred=deferred)   # with and without workspace reuse
        q_all = torch.stack([d[1] for d in data], dim=1).to(dev).contiguous()
        q_cur = torch.empty_like(q_all[0])
        B, Hkv, D = w.batch, w.n_kv_heads, w.head_dim
        graphs = {}
        if use_graph:
            for lay in layers:
                lay.use_static_bounds(int(lens0.max()) + w.n_steps + 1, w.stride)
        outs, idxs = [], []
        for t in range(w.n_steps + 1):
            if t >= 1:
                pos = sl.to(torch.int64)[:, None, None, None].expand(B, Hkv, 1, D)
                for l in range(n_layers):
                    kv[l][0].scatter_(2, pos, data[l][2][0][t - 1].to(dev)[:, :, None, :])
                    kv[l][1].scatter_(2, pos, data[l][2][1][t - 1].to(dev)[:, :, None, :])
                sl += 1
                if not use_graph:
                    for lay in layers:
                        lay.advance()
            q_cur.copy_(q_all[t])
            kind = "full" if (t % w.stride == 0) else "partial"
            if use_graph and t >= 1:
                if kind not in graphs:
                    torch.cuda.synchronize()
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        stack.step(t, q_cur)
                    graphs[kind] = g
                graphs[kind].replay()
            else:
                assert stack.step(t, q_cur) == kind
            torch.cuda.synchronize()
            outs.append(torch.stack([lay.out for lay in layers]).clone())
            idxs.append(torch.stack([lay.idx for lay in layers]).clone())
        for l in range(n_layers):
            got = dict(outs=np.stack([gen.bf16_bits(o[l]) for o in outs]), idx=[i[l].cpu().numpy() for i in idxs],
                       K=gen.bf16_bits(kv[l][0]), V=gen.bf16_bits(kv[l][1]), lens=sl.cpu().numpy())
            (K, V), q, (nk, nv) = data[l]
            compare_with_oracle(w, l, got, K, V, q, nk, nv, lens0)


def test_hybrid_driver_native_partial_steps_graph_full_steps(rk):
    """The launch configuration bench.py times by default: partial steps through rk_decode_step (one
    call for all layers), full steps as the replayed two-stream HIP graph of RefreshKVStack, both on
    the same per-layer state."""
    w = gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], n_steps=11)
    n_layers, dev = 4, "cuda"
    geom = rk.Geom(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.scale)
    lens0 = gen.seq_lens(w)
    data = [(gen.make_kv(w, l), gen.make_queries(w, l), gen.make_new_rows(w, l)) for l in range(n_layers)]
    kv = [(d[0][0].to(dev).clone(), d[0][1].to(dev).clone()) for d in data]
    sl = lens0.to(dev).clone()
    ws = rk.Workspace(geom, w.capacity, w.k_small)
    bound = int(lens0.max()) + w.n_steps + 1
    driver = rk.RefreshKVModel(geom, kv, sl, int(lens0.max()), w.k_small, w.stride, pool_w=w.pool_w, workspace=ws)
    driver.use_static_bounds(bound, w.stride)
    layers = [rk.RefreshKVLayer(geom, kv[l][0], kv[l][1], sl, int(lens0.max()), w.k_small, w.stride, pool_w=w.pool_w,
                                workspace=ws) for l in range(n_layers)]
    for l, lay in enumerate(layers):
        lay.small_K, lay.small_V, lay.idx = driver.small_K[l], driver.small_V[l], driver.idx[l]
        lay.tail_start, lay.out = driver.tail_start[l], driver.out[l]
        lay.use_static_bounds(bound, w.stride)
    stack = rk.RefreshKVStack(layers, n_workspaces=3)
    q_all = torch.stack([d[1] for d in data], dim=1).to(dev).contiguous()
    q_cur = torch.empty_like(q_all[0])
    B, Hkv, D = w.batch, w.n_kv_heads, w.head_dim
    full_graph = None
    outs, idxs = [], []
    for t in range(w.n_steps + 1):
        if t >= 1:
            pos = sl.to(torch.int64)[:, None, None, None].expand(B, Hkv, 1, D)
            for l in range(n_layers):
                kv[l][0].scatter_(2, pos, data[l][2][0][t - 1].to(dev)[:, :, None, :])
                kv[l][1].scatter_(2, pos, data[l][2][1][t - 1].to(dev)[:, :, None, :])
            sl += 1
        q_cur.copy_(q_all[t])
        if t % w.stride != 0:
            assert driver.step(t, q_cur) == "partial"
        elif t == 0:
            assert stack.step(0, q_cur) == "full"
        else:
            if full_graph is None:
                torch.cuda.synchronize()
                full_graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(full_graph):
                    stack.step(t, q_cur)
            full_graph.replay()
        torch.cuda.synchronize()
        outs.append(driver.out.clone())
        idxs.append(driver.idx.clone())
    assert full_graph is not None
    for l in range(n_layers):
        got = dict(outs=np.stack([gen.bf16_bits(o[l]) for o in outs]), idx=[i[l].cpu().numpy() for i in idxs],
                   K=gen.bf16_bits(kv[l][0]), V=gen.bf16_bits(kv[l][1]), lens=sl.cpu().numpy())
        (K, V), q, (nk, nv) = data[l]
        compare_with_oracle(w, l, got, K, V, q, nk, nv, lens0)


def test_loop_cfg1_every_step(rk):
    w = gen.WORKLOADS["cfg1_llama_2k"]
    say("loop", w.name)
    got, ref, n_diff = check_loop(rk, w)
    assert got["kinds"] == ["full" if f else "partial" for f in ref["full"][:, 0]]
    assert sum(k == "full" for k in got["kinds"]) == 9          # t = 0 and 8 strided refreshes
    say("cfg1: index entries differing within the gap tolerance:", n_diff)


def test_loop_cfg1_fixed_size_small_cache(rk):
    w = gen.shrink(gen.WORKLOADS["cfg1_llama_2k"], context=1024, k_small=128, n_steps=12, stride=6)
    say("loop evict-lowest", w.name)
    check_loop(rk, w, evict_lowest=True)


def test_loop_dynamic_trigger_fixed_size_small_cache(rk):
    """Dynamic schedule with the paper's fixed-size small cache: r differs per layer and sequence."""
    w = gen.shrink(gen.WORKLOADS["cfg3_qwen_64k_dynamic"], context=3000, k_small=256, n_steps=30, batch=2)
    say("loop dynamic, evict lowest", w.name)
    got, ref, _ = check_loop(rk, w, evict_lowest=True)
    assert ref["full"][1:].any() and not ref["full"][1:].all()


def test_loop_dynamic_trigger_qwen_small(rk):
    w = gen.shrink(gen.WORKLOADS["cfg3_qwen_64k_dynamic"], context=3000, k_small=256, n_steps=40)
    say("loop dynamic", w.name)
    got, ref, _ = check_loop(rk, w)
    fired = int(ref["full"][1:, 0].sum())
    tested = w.n_steps // w.stride
    assert 0 < fired < tested, "want a mix of fired and not fired tests (fired %d of %d)" % (fired, tested)


def test_loop_batched_ragged_small(rk):
    w = gen.shrink(gen.WORKLOADS["cfg4_llama_batch16_ragged"], batch=5, context=1500, ragged=(300, 1500),
                   k_small=128, n_steps=17, stride=8)
    say("loop batched ragged", w.name, gen.seq_lens(w).tolist())
    check_loop(rk, w)


def test_loop_clustered_keys_small(rk):
    w = gen.shrink(gen.WORKLOADS["cfg5_llama_128k"], context=6000, k_small=384, n_steps=9, stride=4)
    say("loop clustered", w.name)
    check_loop(rk, w)


# ----------------------------------------------------------------------------- full sizes
FULL_SIZE = ["cfg2_llama_32k", "cfg3_qwen_64k_dynamic", "cfg5_llama_128k"]


@pytest.mark.parametrize("name", FULL_SIZE)
def test_full_size_one_layer_refresh_and_partial(rk, name):
    """One layer at the workload's real shape through the per-layer calls (rk_full_attn_select, gather,
    rk_partial_attn): full step + selection + gather + partial steps up to 3 tokens later, all against
    the oracle.  (The driver bench.py times, with the refresh batched over the layers, is covered at these
    shapes by test_full_size_whole_stride_through_the_timed_driver.)"""
    w = gen.shrink(gen.WORKLOADS[name], n_layers=1, n_steps=3, stride=100, dynamic=False)
    say("full size", w.name, "L", w.context, "K", w.k_small)
    K, V = gen.make_kv(w, 0, device="cuda")
    q = gen.make_queries(w, 0)
    nk, nv = gen.make_new_rows(w, 0)
    lens0 = gen.seq_lens(w)
    Kc, Vc = K.cpu(), V.cpu()
    got = run_gpu_loop(rk, w, 0, K, V, q, nk, nv, lens0)
    say("  gpu done; running oracle")
    ref = oracle.decode_loop(gen.bf16_bits(q), gen.bf16_bits(Kc), gen.bf16_bits(Vc), gen.bf16_bits(nk),
                             gen.bf16_bits(nv), lens0.numpy(), w.scale, w.k_small, w.stride, pool_w=w.pool_w)
    for t in range(w.n_steps + 1):
        assert_out_close(got["outs"][t], ref["outs"][t], "%s t=%d" % (name, t))
    wts = oracle.full_attn(gen.bf16_bits(q[0]), gen.bf16_bits(Kc), gen.bf16_bits(Vc), lens0.numpy(), w.scale)[1]
    wts = wts.astype(np.float32)
    G = w.group
    n_diff = 0
    for g in range(w.n_kv_heads):
        P = oracle.pooled_group_scores(wts[0, g * G:(g + 1) * G], w.pool_w)
        n_diff += assert_idx_equivalent(got["idx"][0][0, g], ref["idx"][0][0, g], P, w.context, w.k_small, "g=%d" % g)
    say("  index entries differing within the gap tolerance:", n_diff, "of", w.n_kv_heads * w.k_small)


def test_full_size_model_batched_refresh(rk):
    """Workload 2 at its real shape through rk_decode_step_batched, the driver bench.py times: 8 layers, so
    that the batched selection has the 64 rows from which it takes one workgroup per row, as it does with
    all 32 layers; full, partial, full, partial step, every layer against the oracle."""
    w = gen.shrink(gen.WORKLOADS["cfg2_llama_32k"], n_steps=3, stride=2)
    say("full size, batched driver", w.name, "context", w.context, "K", w.k_small)
    kinds, n_full, _ = check_model_loop(rk, w, 8, overlap="batched")
    assert kinds == ["full", "partial", "full", "partial"] and (n_full == 2).all()


WHOLE_STRIDE = [
    # workload, layers, steps: one whole stride period and the refresh that ends it (+ one partial step after)
    ("cfg2_llama_32k", 8, 11),                 # full at t = 0 and 10 (at 32778 rows); partial steps with 1..9 recent rows
    ("cfg5_llama_128k", 8, 17),                # full at t = 0 and 16; 64 rows of 128k in the batched selection
    ("cfg4_llama_batch16_ragged", 4, 9),       # full at t = 0 and 8; 16 ragged sequences
    ("cfg3_qwen_64k_dynamic", 3, 16),          # trigger tested at t = 5, 10, 15: fires for some layers, not for others
]


@pytest.mark.parametrize("case", WHOLE_STRIDE, ids=[c[0] for c in WHOLE_STRIDE])
def test_full_size_whole_stride_through_the_timed_driver(rk, case):
    """Every workload bench.py can time, at its real shape, through the driver it times
    (rk_decode_step_batched: rk_full_attn_deferred per layer, then pooling, selection and gather of all
    layers in one launch each; on the trigger's test steps both branches under the device predicate):
    every step's output and every snapshot of the selection against the oracle's decode loop."""
    name, n_layers, n_steps = case
    w = gen.shrink(gen.WORKLOADS[name], n_steps=n_steps)
    say("whole stride at full size:", name, "layers", n_layers, "steps", n_steps, "context", w.context, "K", w.k_small)
    kinds, n_full, refs = check_model_loop(rk, w, n_layers, overlap="batched", gen_device="cuda")
    S = w.stride
    if w.dynamic:
        assert kinds == ["full"] + ["both" if t % S == 0 else "partial" for t in range(1, n_steps + 1)]
        fired = np.stack([r["full"][S::S, 0] for r in refs])            # [layer, test step]
        say("  trigger decisions per layer at the test steps:", fired.astype(int).tolist())
        assert fired.any() and not fired.all(), "the case must hold a test step that refreshes and one that does not"
        # a partial step that follows a fired refresh of its layer, and one that follows a declined one, both ran
        assert any(fired[l, i] and (i + 1) * S < n_steps for l in range(n_layers) for i in range(fired.shape[1]))
    else:
        assert kinds == ["full" if t % S == 0 else "partial" for t in range(n_steps + 1)]
        assert (n_full == 1 + n_steps // S).all()


def test_batched_refresh_large_k(rk):
    """K large enough for the selection's histogram-driven bucket layout (more than 8192 candidate slots),
    through the batched driver: 2 layers (a row's selection spread over workgroups) and 8 layers (64 rows
    in the launch: one workgroup per row)."""
    w = gen.shrink(gen.WORKLOADS["cfg2_llama_32k"], context=12000, k_small=5000, n_steps=2, stride=2)
    for n_layers in (2, 8):
        say("batched refresh, K =", w.k_small, "layers =", n_layers)
        kinds, n_full, _ = check_model_loop(rk, w, n_layers, overlap="batched")
        assert kinds == ["full", "partial", "full"] and (n_full == 2).all()
    # rows longer than one workgroup holds in registers (32768 positions), one workgroup per row all the same:
    # the rest of the row is read again from memory
    w = gen.shrink(gen.WORKLOADS["cfg2_llama_32k"], context=40000, k_small=5000, n_steps=1, stride=2)
    say("batched refresh, K =", w.k_small, "context", w.context, "layers = 8")
    kinds, n_full, _ = check_model_loop(rk, w, 8, overlap="batched")
    assert kinds == ["full", "partial"] and (n_full == 1).all()


def test_full_size_batched_ragged(rk):
    """Workload 4 at its real shape (16 ragged sequences, one layer): a full step, the refresh and a
    partial step two tokens later against the oracle, per sequence."""
    w = gen.shrink(gen.WORKLOADS["cfg4_llama_batch16_ragged"], n_layers=1, n_steps=2, stride=100)
    lens0 = gen.seq_lens(w)
    say("full size", w.name, "lens", lens0.tolist(), "K", w.k_small)
    K, V = gen.make_kv(w, 0, device="cuda")
    q = gen.make_queries(w, 0)
    nk, nv = gen.make_new_rows(w, 0)
    Kc, Vc = K.cpu(), V.cpu()
    got = run_gpu_loop(rk, w, 0, K, V, q, nk, nv, lens0)
    say("  gpu done; running oracle")
    ref = oracle.decode_loop(gen.bf16_bits(q), gen.bf16_bits(Kc), gen.bf16_bits(Vc), gen.bf16_bits(nk),
                             gen.bf16_bits(nv), lens0.numpy(), w.scale, w.k_small, w.stride, pool_w=w.pool_w)
    for t in range(w.n_steps + 1):
        assert_out_close(got["outs"][t], ref["outs"][t], "%s t=%d" % (w.name, t))
    wts = oracle.full_attn(gen.bf16_bits(q[0]), gen.bf16_bits(Kc), gen.bf16_bits(Vc), lens0.numpy(), w.scale)[1]
    wts = wts.astype(np.float32)
    G, n_diff = w.group, 0
    for b in range(w.batch):
        n = int(lens0[b])
        for g in range(w.n_kv_heads):
            P = oracle.pooled_group_scores(wts[b, g * G:(g + 1) * G, :n], w.pool_w)
            n_diff += assert_idx_equivalent(got["idx"][0][b, g], ref["idx"][0][b, g], P, n, w.k_small, "b=%d g=%d" % (b, g))
    say("  index entries differing within the gap tolerance:", n_diff, "of", w.batch * w.n_kv_heads * w.k_small)


# ----------------------------------------------------------------------------- H2O comparison policy
H2O_CASES = [
    # name, B, Hq, Hkv, budget, recent, n0, T, agg
    ("llama_small", 2, 8, 2, 300, 150, [290, 120], 40, "max"),
    ("qwen_g7", 1, 14, 2, 64, 32, [64], 30, "max"),
    ("mean_recent0", 1, 4, 1, 40, 0, [33], 25, "mean"),
    ("k2048", 1, 32, 8, 2048, 1024, [2048], 4, "max"),
]


@pytest.mark.parametrize("case", H2O_CASES, ids=[c[0] for c in H2O_CASES])
def test_h2o_policy_matches_oracle(rk, case):
    """Section 3 "Comparison systems" / Appendix A.1: the H2O baseline (cumulative scores, K/2 recent,
    greedy drop) on the library's attention step, against the oracle's statement of the policy."""
    name, B, Hq, Hkv, budget, recent, n0, T, agg = case
    say("h2o case", name)
    rng = np.random.default_rng(len(name) * 7 + budget)
    g = torch.Generator().manual_seed(budget + T)
    D, cap = 128, budget + 1
    nmax = max(n0)
    k0 = torch.randn(B, Hkv, nmax, D, generator=g).to(torch.bfloat16)
    v0 = torch.randn(B, Hkv, nmax, D, generator=g).to(torch.bfloat16)
    q = torch.randn(T, B, Hq, D, generator=g).to(torch.bfloat16)
    nk = torch.randn(T, B, Hkv, D, generator=g).to(torch.bfloat16)
    nv = torch.randn(T, B, Hkv, D, generator=g).to(torch.bfloat16)
    k0[:, :, ::13] *= 2.0
    pos0 = np.zeros((B, Hkv, nmax), dtype=np.int64)
    for b in range(B):
        for h in range(Hkv):             # what a prefill-side selection leaves: a subset of the prompt, in any order
            pos0[b, h, :n0[b]] = rng.permutation(np.sort(rng.choice(3 * nmax, size=n0[b], replace=False)))
        pos0[b, :, 0] = 3 * nmax         # the same newest position for every head of a sequence
    tot0 = (rng.random((B, Hkv, nmax)) * 0.05).astype(np.float32)
    scale = float(np.float32(1 / np.sqrt(128)))
    ref = oracle.h2o_decode_loop(gen.bf16_bits(q), gen.bf16_bits(k0), gen.bf16_bits(v0), tot0, pos0, n0,
                                 gen.bf16_bits(nk), gen.bf16_bits(nv), scale, budget, recent, agg)

    geom = rk.Geom(B, Hq, Hkv, D, scale)
    cK = torch.zeros(B, Hkv, cap, D, dtype=torch.bfloat16, device="cuda"); cV = torch.zeros_like(cK)
    cK[:, :, :nmax] = k0.cuda(); cV[:, :, :nmax] = v0.cuda()
    total = torch.zeros(B, Hkv, cap, dtype=torch.float32, device="cuda"); total[:, :, :nmax] = torch.from_numpy(tot0).cuda()
    pos = torch.full((B, Hkv, cap), -1, dtype=torch.int32, device="cuda"); pos[:, :, :nmax] = torch.from_numpy(pos0).int().cuda()
    n_rows = torch.tensor(n0, dtype=torch.int32, device="cuda")
    n_attend = torch.zeros(B, dtype=torch.int32, device="cuda")
    st = rk.h2o_state(geom, cK, cV, total, pos, n_rows, n_attend)
    ws = rk.Workspace(geom, cap, 16)
    out = torch.zeros(B, Hq, D, dtype=torch.bfloat16, device="cuda")
    dropped = torch.zeros(B, Hkv, dtype=torch.int32, device="cuda")
    seq_lens = torch.full((B,), 3 * nmax + 1, dtype=torch.int32, device="cuda")
    code = {"max": rk.RK_AGG_MAX, "mean": rk.RK_AGG_MEAN, "first": rk.RK_AGG_FIRST}[agg]
    alive = np.ones((B, Hkv), dtype=bool)            # (b, g) still on the oracle's path
    qd, nkd, nvd = q.cuda(), nk.cuda(), nv.cuda()
    n_drops = 0
    for t in range(T):
        seq_lens += 1
        rk.rk_h2o_step(geom, st, qd[t], nkd[t], nvd[t], seq_lens, budget, recent, out, agg=code, dropped=dropped, workspace=ws)
        torch.cuda.synchronize()
        got_drop, got_out = dropped.cpu().numpy(), gen.bf16_bits(out)
        for b in range(B):
            for h in range(Hkv):
                if not alive[b, h]:
                    continue
                G = Hq // Hkv
                assert_out_close(got_out[b:b + 1, h * G:(h + 1) * G], ref["outs"][t, b:b + 1, h * G:(h + 1) * G])
                if got_drop[b, h] != ref["dropped"][t, b, h]:
                    assert ref["margin"][t, b, h] < 1e-5, (name, t, b, h, got_drop[b, h], ref["dropped"][t, b, h])
                    alive[b, h] = False              # a near-tie went the other way: the paths part here
                n_drops += int(got_drop[b, h] >= 0)
    assert alive.mean() > 0.7 and n_drops > 0
    nr = n_rows.cpu().numpy()
    tot_n, pos_n = total.cpu().numpy(), pos.cpu().numpy()
    for b in range(B):
        assert nr[b] == min(n0[b] + T, budget)
        for h in range(Hkv):
            if not alive[b, h]:
                continue
            want = ref["final"][b][h]
            got = {int(pos_n[b, h, j]): float(tot_n[b, h, j]) for j in range(nr[b])}
            assert sorted(got) == sorted(want)
            for x in want:
                assert abs(got[x] - float(want[x])) <= 1e-5 * max(abs(float(want[x])), 1e-3)
