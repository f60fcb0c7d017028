"""rk_partial_attn_static (the entry point that allocates nothing) through the raw C ABI.

Its scratch is a device array built into the library, so consecutive calls share memory whatever
their shapes: two calls in a row, the second with a smaller input, each compared with
rk_partial_attn on a caller's workspace (same kernels, another hand-over between the workgroups:
equal to within the bar the outputs are held to) and with the oracle.
"""
import ctypes as C
import sys

import numpy as np
import pytest
import torch

import gen
import oracle
from helpers import assert_out_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_05787_amd as lib     # raises if the HIP library is not built
    return lib


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def one_case(rk, seed, B, Hq, Hkv, lens, recent, k, n_sel):
    """Inputs on the GPU, the oracle's output, and the raw C arguments shared by both entry points."""
    from paper_2411_05787_amd.binding import _Geom, _Kv
    cap = max(lens) + 8
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Hq, 128, generator=g).to(torch.bfloat16)
    K = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, cap, 128, generator=g).to(torch.bfloat16)
    scale = float(np.float32(1 / np.sqrt(128)))
    tail = [l - r for l, r in zip(lens, recent)]
    idx = torch.full((B, Hkv, k), -1, dtype=torch.int32)
    for b in range(B):
        kk = min(k, tail[b])
        for h in range(Hkv):
            idx[b, h, :kk] = torch.randperm(tail[b], generator=g)[:kk].to(torch.int32)
    geom = rk.Geom(B, Hq, Hkv, 128, scale)
    Kd, Vd, qd = K.cuda(), V.cuda(), q.cuda()
    sK = torch.zeros(B, Hkv, k, 128, dtype=torch.bfloat16, device="cuda")
    sV = torch.zeros_like(sK)
    rk.rk_gather_small_kv(geom, Kd, Vd, idx.cuda(), k, sK, sV)
    rK = np.zeros((B, Hkv, k, 128), dtype=np.uint16); rV = rK.copy()
    oracle.gather_small_kv(gen.bf16_bits(K), gen.bf16_bits(V), idx.numpy(), rK, rV)
    o_ref = oracle.partial_attn(gen.bf16_bits(q), rK, rV, n_sel, gen.bf16_bits(K), gen.bf16_bits(V), tail, lens, scale)
    tail_d = torch.tensor(tail, dtype=torch.int32, device="cuda")
    lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
    cg = _Geom(B, Hq, Hkv, 128, scale)
    small = _Kv(sK.data_ptr(), sV.data_ptr(), sK.stride(0), sK.stride(1), k)
    full = _Kv(Kd.data_ptr(), Vd.data_ptr(), Kd.stride(0), Kd.stride(1), cap)
    keep = (Kd, Vd, qd, sK, sV, tail_d, lens_d)
    return dict(geom=geom, cg=cg, q=qd, small=small, full=full, tail=tail_d, lens=lens_d, n_sel=n_sel,
                max_recent=max(max(recent), 1), o_ref=o_ref, cap=cap, k=k, B=B, Hq=Hq, keep=keep)


def run_both(rk, c, what):
    lib = rk.lib
    stream = torch.cuda.current_stream().cuda_stream
    ws = rk.Workspace(c["geom"], c["cap"], c["k"])
    out_ws = torch.zeros(c["B"], c["Hq"], 128, dtype=torch.bfloat16, device="cuda")
    out_st = torch.full((c["B"], c["Hq"], 128), 3.0, dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()          # every allocation of this case is done before the static call
    say("no-alloc case", what, "static scratch bytes",
        lib.rk_partial_attn_static_bytes(C.byref(c["cg"]), c["n_sel"], c["max_recent"]))
    rc = lib.rk_partial_attn_static(C.byref(c["cg"]), c["q"].data_ptr(), c["small"], c["n_sel"], c["full"],
                                    c["tail"].data_ptr(), c["lens"].data_ptr(), c["max_recent"], out_st.data_ptr(),
                                    None, 0, stream)
    assert rc == 0, rk.status_string(rc)
    rc = lib.rk_partial_attn(C.byref(c["cg"]), c["q"].data_ptr(), c["small"], c["n_sel"], c["full"],
                             c["tail"].data_ptr(), c["lens"].data_ptr(), c["max_recent"], out_ws.data_ptr(),
                             None, 0, ws.ptr, ws.nbytes, stream)
    assert rc == 0, rk.status_string(rc)
    torch.cuda.synchronize()
    assert_out_close(gen.bf16_bits(out_st), gen.bf16_bits(out_ws), what + ": static scratch against workspace")
    assert_out_close(gen.bf16_bits(out_st), c["o_ref"], what + ": static scratch against the oracle")
    assert_out_close(gen.bf16_bits(out_ws), c["o_ref"], what + ": workspace against the oracle")


def test_static_entry_two_calls_second_smaller(rk):
    big = one_case(rk, 11, 2, 32, 8, [5000, 3100], [10, 3], 2048, 2048)
    small = one_case(rk, 12, 1, 28, 4, [700], [17], 100, 100)
    run_both(rk, big, "first call: 2 x 8 heads, 2048 + 10 rows")
    run_both(rk, small, "second call, smaller: 1 x 4 heads (groups of 7), 100 + 17 rows")
    run_both(rk, big, "the first shape again")


def test_static_entry_predicate_and_limits(rk):
    lib = rk.lib
    c = one_case(rk, 13, 2, 8, 2, [600, 300], [5, 9], 64, 64)
    stream = torch.cuda.current_stream().cuda_stream
    out = torch.full((2, 8, 128), 3.0, dtype=torch.bfloat16, device="cuda")
    pred = torch.tensor([1, 0], dtype=torch.int32, device="cuda")
    rc = lib.rk_partial_attn_static(C.byref(c["cg"]), c["q"].data_ptr(), c["small"], c["n_sel"], c["full"],
                                    c["tail"].data_ptr(), c["lens"].data_ptr(), c["max_recent"], out.data_ptr(),
                                    pred.data_ptr(), 1, stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert (out[1] == 3.0).all()                       # switched off: untouched
    assert_out_close(gen.bf16_bits(out[:1]), c["o_ref"][:1], "predicated static call")
    # beyond the array: refused on the host, nothing enqueued
    from paper_2411_05787_amd.binding import _Geom
    too_many = _Geom(512, 64, 8, 128, 1.0)
    assert lib.rk_partial_attn_static_bytes(C.byref(too_many), 64, 9) > rk.binding.STATIC_SCRATCH_BYTES
    assert lib.rk_partial_attn_static(C.byref(too_many), c["q"].data_ptr(), c["small"], 64, c["full"], c["tail"].data_ptr(),
                                      c["lens"].data_ptr(), 9, out.data_ptr(), None, 0, stream) == -5
