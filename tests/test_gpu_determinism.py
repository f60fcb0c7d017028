"""Repeatability of the kernels whose workgroups hand partial results to one another inside a launch.

The partial step, full attention without weights (short rows: merged inside the launch) and the
selection over long rows (candidates listed by several workgroups) pass data between workgroups
with coherent stores and loads ordered by tickets and, in the partial step, by tags carried in the
data.  Nothing in that is allowed to depend on timing: the same inputs must give the same bits on
every call, whichever workgroup arrives last.  Each case runs many back-to-back calls on one
workspace, requires every call's output to equal the first call's bit for bit and the first call's
to match the oracle, and then runs another input on the same workspace to show that the calls left
it clean.  A mismatch here is a finding to be reasoned out from the code.
"""
import sys

import numpy as np
import pytest
import torch

import gen
import oracle
from helpers import assert_out_close

pytestmark = pytest.mark.gpu
N_CALLS = 2000


@pytest.fixture(scope="module")
def rk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_05787_amd as lib     # raises if the HIP library is not built
    return lib


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def first_mismatch(all_calls: torch.Tensor):
    """Index of the first call whose output differs from call 0 (None: all equal), computed on the GPU."""
    same = (all_calls == all_calls[:1]).flatten(1).all(dim=1)
    bad = (~same).nonzero()
    return None if bad.numel() == 0 else int(bad[0])


def partial_inputs(rk, seed, B, Hq, Hkv, k, lens, recent):
    cap = max(lens) + 8
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Hq, 128, generator=g).to(torch.bfloat16)
    K = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16)
    tail = [l - r for l, r in zip(lens, recent)]
    idx = torch.full((B, Hkv, k), -1, dtype=torch.int32)
    for b in range(B):
        kk = min(k, tail[b])
        for h in range(Hkv):
            idx[b, h, :kk] = torch.randperm(tail[b], generator=g)[:kk].to(torch.int32)
    return q, K, V, tail, idx, cap


@pytest.mark.parametrize("shape", [("llama_k2048", 1, 32, 8, 2048, [32768 + 7], [7]),
                                   ("qwen_k4096", 1, 28, 4, 4096, [20000], [3]),
                                   ("batch4_k1024", 4, 32, 8, 1024, [9000, 5000, 7000, 4100], [5, 1, 0, 8])],
                         ids=lambda s: s[0])
def test_partial_attn_repeats_bit_for_bit(rk, shape):
    name, B, Hq, Hkv, k, lens, recent = shape
    say("determinism: rk_partial_attn", name, N_CALLS, "calls")
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    q, K, V, tail, idx, cap = partial_inputs(rk, 91, B, Hq, Hkv, k, lens, recent)
    Kd, Vd, qd = K.cuda(), V.cuda(), q.cuda()
    sK = torch.zeros(B, Hkv, k, 128, dtype=torch.bfloat16, device="cuda"); sV = torch.zeros_like(sK)
    rk.rk_gather_small_kv(geom, Kd, Vd, idx.cuda(), k, sK, sV)
    ws = rk.Workspace(geom, cap, k)
    tail_d = torch.tensor(tail, dtype=torch.int32, device="cuda")
    lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
    outs = torch.zeros(N_CALLS, B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    for i in range(N_CALLS):
        rk.rk_partial_attn(geom, qd, sK, sV, k, Kd, Vd, tail_d, lens_d, max(max(recent), 1), outs[i], workspace=ws)
    torch.cuda.synchronize()
    bad = first_mismatch(outs.view(torch.int16))
    assert bad is None, "call %d differs from call 0" % bad
    rK = np.zeros((B, Hkv, k, 128), dtype=np.uint16); rV = rK.copy()
    oracle.gather_small_kv(gen.bf16_bits(K), gen.bf16_bits(V), idx.numpy(), rK, rV)
    o_ref = oracle.partial_attn(gen.bf16_bits(q), rK, rV, k, gen.bf16_bits(K), gen.bf16_bits(V), tail, lens, scale)
    assert_out_close(gen.bf16_bits(outs[0]), o_ref, name)
    # the lazy form of the same step, then another query, on the same workspace: left clean
    sK2 = torch.zeros_like(sK); sV2 = torch.zeros_like(sV)
    out2 = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    rk.rk_partial_attn_lazy(geom, qd, sK2, sV2, idx.cuda(), k, Kd, Vd, tail_d, lens_d, max(max(recent), 1), out2, workspace=ws)
    torch.cuda.synchronize()
    assert_out_close(gen.bf16_bits(out2), o_ref, name + " lazy")
    q3 = torch.randn(B, Hq, 128, generator=torch.Generator().manual_seed(5)).to(torch.bfloat16)
    out3 = torch.zeros_like(out2)
    rk.rk_partial_attn(geom, q3.cuda(), sK, sV, k, Kd, Vd, tail_d, lens_d, max(max(recent), 1), out3, workspace=ws)
    torch.cuda.synchronize()
    o3 = oracle.partial_attn(gen.bf16_bits(q3), rK, rV, k, gen.bf16_bits(K), gen.bf16_bits(V), tail, lens, scale)
    assert_out_close(gen.bf16_bits(out3), o3, name + " other query, same workspace")


@pytest.mark.parametrize("rows", [9001, 20000])
def test_full_attn_without_weights_repeats_bit_for_bit(rk, rows):
    """9001 rows: merged by the last workgroup of the launch; 20000: the wide split + the merge launch."""
    say("determinism: rk_full_attn(weights=NULL)", rows, "rows", N_CALLS, "calls")
    B, Hq, Hkv = 1, 32, 8
    cap = rows + 23
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    g = torch.Generator().manual_seed(rows)
    q = torch.randn(B, Hq, 128, generator=g).to(torch.bfloat16)
    K = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16)
    Kd, Vd, qd = K.cuda(), V.cuda(), q.cuda()
    sl = torch.tensor([rows], dtype=torch.int32, device="cuda")
    ws = rk.Workspace(geom, cap, 16)
    outs = torch.zeros(N_CALLS, B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    lses = torch.zeros(N_CALLS, B, Hq, dtype=torch.float32, device="cuda")
    for i in range(N_CALLS):
        rk.rk_full_attn(geom, qd, Kd, Vd, sl, rows, outs[i], lse=lses[i], workspace=ws)
    torch.cuda.synchronize()
    bad = first_mismatch(outs.view(torch.int16))
    assert bad is None, "out of call %d differs from call 0" % bad
    bad = first_mismatch(lses.view(torch.int32))
    assert bad is None, "lse of call %d differs from call 0" % bad
    o_ref, _, lse_ref = oracle.full_attn(gen.bf16_bits(q), gen.bf16_bits(K), gen.bf16_bits(V), [rows], scale)
    assert_out_close(gen.bf16_bits(outs[0]), o_ref, "rows=%d" % rows)
    assert np.abs(lses[0].cpu().numpy() - lse_ref).max() < 1e-5
    # a call that returns the weights (ordinary stores into the same regions), then the first form again
    w = torch.zeros(B, Hq, cap, dtype=torch.float32, device="cuda")
    out_w = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    rk.rk_full_attn(geom, qd, Kd, Vd, sl, rows, out_w, weights=w, workspace=ws)
    out_again = torch.zeros_like(out_w)
    rk.rk_full_attn(geom, qd, Kd, Vd, sl, rows, out_again, workspace=ws)
    torch.cuda.synchronize()
    assert_out_close(gen.bf16_bits(out_w), o_ref, "with weights")
    assert torch.equal(out_again, outs[0]), "the call after a weights-returning call differs"


def test_partial_and_full_alternate_on_one_workspace(rk):
    """A weights-returning full step (ordinary stores into the partial-result regions) and a partial step
    (tagged or ticketed hand-over in its own regions) take turns on one workspace; every partial step
    must repeat the first one bit for bit."""
    say("determinism: full step with weights and partial step alternating")
    B, Hq, Hkv, k, lens, recent = 1, 32, 8, 2048, [12000], [6]
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    q, K, V, tail, idx, cap = partial_inputs(rk, 17, B, Hq, Hkv, k, lens, recent)
    Kd, Vd, qd = K.cuda(), V.cuda(), q.cuda()
    sK = torch.zeros(B, Hkv, k, 128, dtype=torch.bfloat16, device="cuda"); sV = torch.zeros_like(sK)
    rk.rk_gather_small_kv(geom, Kd, Vd, idx.cuda(), k, sK, sV)
    ws = rk.Workspace(geom, cap, k)
    tail_d = torch.tensor(tail, dtype=torch.int32, device="cuda")
    lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
    n = 300
    outs = torch.zeros(n, B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    full_outs = torch.zeros(n, B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(B, Hq, cap, dtype=torch.float32, device="cuda")
    for i in range(n):
        rk.rk_full_attn(geom, qd, Kd, Vd, lens_d, lens[0], full_outs[i], weights=w, workspace=ws)
        rk.rk_partial_attn(geom, qd, sK, sV, k, Kd, Vd, tail_d, lens_d, recent[0], outs[i], workspace=ws)
    torch.cuda.synchronize()
    assert first_mismatch(outs.view(torch.int16)) is None
    assert first_mismatch(full_outs.view(torch.int16)) is None
    rK = np.zeros((B, Hkv, k, 128), dtype=np.uint16); rV = rK.copy()
    oracle.gather_small_kv(gen.bf16_bits(K), gen.bf16_bits(V), idx.numpy(), rK, rV)
    o_ref = oracle.partial_attn(gen.bf16_bits(q), rK, rV, k, gen.bf16_bits(K), gen.bf16_bits(V), tail, lens, scale)
    assert_out_close(gen.bf16_bits(outs[0]), o_ref, "partial step between full steps")


def test_topk_select_long_rows_repeats_bit_for_bit(rk):
    """40000 positions: the candidates are listed by ten workgroups and ranked by the one that arrives last."""
    say("determinism: rk_topk_select over 40000 positions", N_CALLS, "calls")
    B, Hq, Hkv, n, k = 1, 8, 2, 40000, 2048
    w = gen.make_weights(B, Hq, n, seed=4, kind="lognormal")
    geom = rk.Geom(B, Hq, Hkv, 128, 1.0)
    ws = rk.Workspace(geom, n, k)
    sl = torch.tensor([n], dtype=torch.int32, device="cuda")
    wd = w.cuda()
    idxs = torch.full((N_CALLS, B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    for i in range(N_CALLS):
        rk.rk_topk_select(geom, wd, sl, n, k, 7, idxs[i], workspace=ws)
    torch.cuda.synchronize()
    bad = first_mismatch(idxs)
    assert bad is None, "idx of call %d differs from call 0" % bad
    i_ref, _ = oracle.topk_select(w.numpy(), [n], Hkv, k, 7)
    assert (idxs[0].cpu().numpy() == i_ref).all()
    # another input (ties everywhere) on the same workspace
    w2 = gen.make_weights(B, Hq, n, seed=5, kind="ties")
    idx2 = torch.full((B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    rk.rk_topk_select(geom, w2.cuda(), sl, n, k, 7, idx2, workspace=ws)
    torch.cuda.synchronize()
    i_ref2, _ = oracle.topk_select(w2.numpy(), [n], Hkv, k, 7)
    assert (idx2.cpu().numpy() == i_ref2).all()


def test_partial_attn_triggered_repeats_bit_for_bit(rk):
    """The partial step with the query-similarity test inside: sequences that ask for a full step and
    sequences that do not in one batch; every call gives the same output, similarity, decision and
    reference, and leaves the test's ticket clean for the next one."""
    say("determinism: rk_partial_attn_triggered", N_CALLS, "calls")
    B, Hq, Hkv, k = 4, 32, 8, 1024
    lens, recent = [9000, 5000, 7000, 4100], [5, 1, 0, 8]
    scale = float(np.float32(1 / np.sqrt(128)))
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    q, K, V, tail, idx, cap = partial_inputs(rk, 92, B, Hq, Hkv, k, lens, recent)
    Kd, Vd, qd = K.cuda(), V.cuda(), q.cuda()
    sK = torch.zeros(B, Hkv, k, 128, dtype=torch.bfloat16, device="cuda"); sV = torch.zeros_like(sK)
    rk.rk_gather_small_kv(geom, Kd, Vd, idx.cuda(), k, sK, sV)
    ws = rk.Workspace(geom, cap, k)
    tail_d = torch.tensor(tail, dtype=torch.int32, device="cuda")
    lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
    ref = torch.randn(B, 128, generator=torch.Generator().manual_seed(3))
    ref[0] = q[0].float().mean(0); ref[2] = q[2].float().mean(0) * 0.5          # sequences 0 and 2: no full step
    s_ref, n_ref, r_ref = oracle.query_sim(gen.bf16_bits(q), ref.double().numpy(), 0.5, False)
    assert n_ref.tolist() == [False, True, False, True]
    outs = torch.full((N_CALLS, B, Hq, 128), 3.0, dtype=torch.bfloat16, device="cuda")
    refs = ref.cuda().repeat(N_CALLS, 1, 1).contiguous()
    sims = torch.zeros(N_CALLS, B, device="cuda")
    needs = torch.full((N_CALLS, B), -1, dtype=torch.int32, device="cuda")
    for i in range(N_CALLS):
        rk.rk_partial_attn_triggered(geom, qd, sK, sV, k, Kd, Vd, tail_d, lens_d, 8, outs[i], refs[i], 0.5, sims[i], needs[i],
                                     workspace=ws)
    torch.cuda.synchronize()
    for what, t in (("out", outs.view(torch.int16)), ("q_ref", refs.view(torch.int32)), ("sim", sims.view(torch.int32)),
                    ("need_full", needs)):
        bad = first_mismatch(t)
        assert bad is None, "%s of call %d differs from call 0" % (what, bad)
    assert (needs[0].cpu().numpy().astype(bool) == n_ref).all()
    assert np.abs(refs[0].cpu().numpy() - r_ref).max() < 1e-6
    rK = np.zeros((B, Hkv, k, 128), dtype=np.uint16); rV = rK.copy()
    oracle.gather_small_kv(gen.bf16_bits(K), gen.bf16_bits(V), idx.numpy(), rK, rV)
    o_ref = oracle.partial_attn(gen.bf16_bits(q), rK, rV, k, gen.bf16_bits(K), gen.bf16_bits(V), tail, lens, scale)
    got = gen.bf16_bits(outs[0])
    assert_out_close(got[~n_ref], o_ref[~n_ref], "sequences without a full step")
    assert (got[n_ref] == gen.bf16_bits(torch.tensor(3.0, dtype=torch.bfloat16))).all()


def test_topk_select_128k_runs_repeat_bit_for_bit(rk):
    """131072 positions, K = 8192: 32 workgroups list runs of equal pooled scores, the last one ranks them."""
    n_calls = 500
    say("determinism: rk_topk_select over 131072 positions", n_calls, "calls")
    B, Hq, Hkv, n, k = 1, 8, 2, 131072, 8192
    w = gen.make_weights(B, Hq, n, seed=14, kind="lognormal")
    geom = rk.Geom(B, Hq, Hkv, 128, 1.0)
    ws = rk.Workspace(geom, n, k)
    sl = torch.tensor([n], dtype=torch.int32, device="cuda")
    wd = w.cuda()
    idxs = torch.full((n_calls, B, Hkv, k), -5, dtype=torch.int32, device="cuda")
    for i in range(n_calls):
        rk.rk_topk_select(geom, wd, sl, n, k, 7, idxs[i], workspace=ws)
    torch.cuda.synchronize()
    bad = first_mismatch(idxs)
    assert bad is None, "idx of call %d differs from call 0" % bad
    i_ref, _ = oracle.topk_select(w.numpy(), [n], Hkv, k, 7)
    assert (idxs[0].cpu().numpy() == i_ref).all()
