"""The C-ABI library loads, exports what include/refreshkv.h declares, and rejects bad
arguments on the host before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def rk():
    import paper_2411_05787_amd as lib      # raises when the library is not built
    return lib


def declared_functions():
    text = open(os.path.join(ROOT, "include", "refreshkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rk_[a-z_0-9]+)\s*\(", text)))


def test_header_and_binding_agree(rk):
    names = declared_functions()
    assert "rk_full_attn" in names and "rk_topk_select" in names and "rk_gather_small_kv" in names
    assert "rk_partial_attn" in names and "rk_query_sim" in names
    assert sorted(rk.EXPORTS) == names


def test_every_declared_symbol_is_exported(rk):
    lib = C.CDLL(rk.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_version_and_status_strings(rk):
    assert rk.version() >= 100
    assert rk.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert rk.status_string(code) not in ("ok", "unknown status")
    assert rk.status_string(-99) == "unknown status"


def test_workspace_bytes_grows_and_rejects(rk):
    g = rk.Geom(1, 32, 8, 128, 0.0884)
    a, b = rk.workspace_bytes(g, 2048, 256), rk.workspace_bytes(g, 32768, 2048)
    assert 0 < a < b and a % 256 == 0 and b % 256 == 0
    for bad in (rk.Geom(1, 32, 8, 64, 1.0), rk.Geom(1, 30, 8, 128, 1.0), rk.Geom(0, 32, 8, 128, 1.0),
                rk.Geom(1, 32, 2, 128, 1.0)):
        with pytest.raises(rk.RkError):
            rk.workspace_bytes(bad, 1024, 64)


def test_host_side_argument_checks_return_before_any_launch(rk):
    """Raw ctypes calls with pointers that are never dereferenced: every one must be refused."""
    from paper_2411_05787_amd.binding import _Geom, _Kv
    lib = rk.lib
    g = _Geom(1, 32, 8, 128, 0.0884)
    fake = 0x10000                                # aligned, non-null, never touched
    kv = _Kv(fake, fake, 8 * 4096 * 128, 4096 * 128, 4096)
    ws_bytes = rk.workspace_bytes(rk.Geom(1, 32, 8, 128, 0.0884), 4096, 256)
    full = lambda **kw: lib.rk_full_attn(C.byref(kw.get("g", g)), kw.get("q", fake), kw.get("kv", kv),
                                         kw.get("sl", fake), kw.get("max_len", 4096), fake, kw.get("w", None),
                                         kw.get("ws_stride", 0), None, None, 0, kw.get("ws", fake + 0x100000 - 0x10000),
                                         kw.get("wsb", ws_bytes), None)
    assert full(g=_Geom(1, 32, 8, 64, 1.0)) == -2                       # head_dim
    assert full(g=_Geom(1, 72, 8, 128, 1.0)) == -2                      # group of 9
    assert full(g=_Geom(1, 33, 8, 128, 1.0)) == -1                      # heads do not divide
    assert full(q=None) == -1
    assert full(sl=None) == -1
    assert full(max_len=0) == -1
    assert full(kv=_Kv(fake + 2, fake, 0, 0, 4096)) == -1                     # misaligned K
    assert full(kv=_Kv(fake, fake, 12, 128, 4096)) == -1                      # stride not a multiple of 8
    assert full(kv=_Kv(fake, fake, 0, 0, 0)) == -1                      # no rows allocated
    assert full(kv=_Kv(fake, fake, 0, 2 ** 31, 4096)) == -2             # head stride beyond 32 bits
    assert full(w=fake, ws_stride=100) == -1                            # weights rows shorter than max_len
    assert full(ws=None) == -3
    assert full(ws=fake + 4) == -3                                      # misaligned workspace
    assert full(wsb=1024) == -3                                         # too small
    topk = lambda **kw: lib.rk_topk_select(C.byref(g), fake, 4096, fake, 4096, kw.get("k", 256), kw.get("pool", 7),
                                           kw.get("agg", 0), fake, None, None, 0, 0x100000, ws_bytes, None)
    assert topk(k=0) == -1
    assert topk(k=16385) == -2
    assert topk(pool=4) == -1
    assert topk(pool=65) == -2
    assert topk(agg=3) == -2 and topk(agg=-1) == -2
    # a row beyond RK_MAX_SELECT_LEN positions (28 bits of a ranked item hold the position)
    assert lib.rk_topk_select(C.byref(g), fake, 2 ** 28 + 8, fake, 2 ** 28 + 1, 256, 7, 0, fake, None, None, 0,
                              0x100000, ws_bytes, None) == -2
    fused = lambda **kw: lib.rk_full_attn_select(C.byref(g), kw.get("q", fake), kv, fake, 4096, kw.get("out", fake), None, 0,
                                                 None, kw.get("k", 256), kw.get("pool", 7), 0, kw.get("idx", fake), None,
                                                 None, 0, kw.get("ws", 0x100000), ws_bytes, None)
    assert fused(q=None) == -1
    assert fused(out=None) == -1
    assert fused(idx=None) == -1
    assert fused(k=0) == -1
    assert fused(k=16385) == -2
    assert fused(pool=2) == -1
    assert fused(ws=None) == -3
    kv_k_only = _Kv(fake, None, 8 * 4096 * 128, 4096 * 128, 4096)
    score = lambda **kw: lib.rk_score_select(C.byref(g), kw.get("q", fake), kw.get("kv", kv_k_only), fake, 4096, None, 0, None,
                                             kw.get("k", 256), 7, 0, kw.get("idx", fake), None, None, 0,
                                             kw.get("ws", 0x100000), ws_bytes, None)
    assert score(q=None) == -1
    assert score(kv=_Kv(None, fake, 0, 0, 4096)) == -1                   # keys are required, values are not
    assert score(idx=None) == -1
    assert score(k=0) == -1
    assert score(ws=None) == -3
    assert full(kv=kv_k_only) == -1                                      # a full step needs the values
    window = lambda **kw: lib.rk_window_select(C.byref(g), kw.get("q", fake), kw.get("w", 8), kv_k_only, fake, 4096, None, 0,
                                               kw.get("k", 256), 7, 0, kw.get("idx", fake), None, None, 0,
                                               kw.get("ws", 0x100000), ws_bytes, None)
    assert window(q=None) == -1
    assert window(w=0) == -1
    assert window(w=33) == -2                                            # beyond RK_MAX_WINDOW
    assert window(idx=None) == -1
    assert window(k=0) == -1
    assert window(ws=None) == -3
    assert lib.rk_gather_small_kv(C.byref(g), kv, None, 16, kv, None, None, None, 0, None) == -1
    assert lib.rk_gather_small_kv(C.byref(g), kv, fake, 0, kv, None, None, None, 0, None) == -1
    assert lib.rk_gather_small_kv(C.byref(g), kv, fake, 16, kv, None, fake, None, 0, None) == -1   # tail_start without seq_lens
    assert lib.rk_partial_attn(C.byref(g), fake, kv, -1, kv, fake, fake, 4, fake, None, 0, 0x100000, ws_bytes, None) == -1
    assert lib.rk_partial_attn(C.byref(g), fake, kv, 0, kv, fake, fake, 0, fake, None, 0, 0x100000, ws_bytes, None) == -1
    assert lib.rk_partial_attn(C.byref(g), fake, kv, 16, kv, None, fake, 4, fake, None, 0, 0x100000, ws_bytes, None) == -1
    static = lambda **kw: lib.rk_partial_attn_static(C.byref(kw.get("g", g)), kw.get("q", fake), kv, kw.get("n_sel", 16), kv,
                                                     kw.get("tail", fake), fake, kw.get("recent", 4), fake, None, 0, None)
    assert static(q=None) == -1
    assert static(n_sel=-1) == -1
    assert static(tail=None) == -1
    assert static(n_sel=0, recent=0) == -1
    assert static(g=_Geom(4097, 8, 8, 128, 1.0)) == -5                  # more (sequence, KV head) pairs than counters
    assert static(g=_Geom(512, 64, 8, 128, 1.0)) == -5                  # statistics of 4096 pairs x 8 heads: beyond the array
    assert lib.rk_partial_attn_static_bytes(C.byref(g), 2048, 16) <= 8 << 20
    assert lib.rk_partial_attn_static_bytes(C.byref(_Geom(32, 64, 8, 128, 1.0)), 16384, 64) <= 8 << 20     # 256 pairs, G = 8
    assert lib.rk_partial_attn_static_bytes(C.byref(_Geom(512, 64, 8, 128, 1.0)), 2048, 16) > 8 << 20
    assert lib.rk_partial_attn_static_bytes(C.byref(g), 0, 0) == 0
    assert lib.rk_query_sim(C.byref(g), fake, None, 0.5, 0, fake, fake, None) == -1
    from paper_2411_05787_amd.binding import _H2oState
    h2o = lambda cap=257, total=fake: _H2oState(_Kv(fake, fake, 8 * cap * 128, cap * 128, cap), total, fake, fake, fake)
    assert lib.rk_h2o_append(C.byref(g), h2o(), None, fake, fake, 256, None) == -1
    assert lib.rk_h2o_append(C.byref(g), h2o(cap=256), fake, fake, fake, 256, None) == -1        # no room for budget + 1 rows
    assert lib.rk_h2o_update(C.byref(g), h2o(), fake, 300, 256, 256, 0, None, None) == -1         # recent must stay below the budget
    assert lib.rk_h2o_update(C.byref(g), h2o(), fake, 200, 256, 128, 0, None, None) == -1         # weight rows too short
    assert lib.rk_h2o_update(C.byref(g), h2o(total=None), fake, 300, 256, 128, 0, None, None) == -1
    assert lib.rk_h2o_update(C.byref(g), h2o(), fake, 300, 256, 128, 5, None, None) == -2         # unknown aggregation
    assert lib.rk_h2o_step(C.byref(g), h2o(), fake, fake, fake, fake, 256, 128, 0, None, None, 0x100000, ws_bytes, None) == -1
    assert lib.rk_h2o_step(C.byref(g), h2o(), fake, fake, fake, fake, 256, 128, 0, fake, None, None, ws_bytes, None) == -3
    deferred = lambda **kw: lib.rk_full_attn_deferred(C.byref(g), kw.get("q", fake), kw.get("kv", kv), kw.get("sl", fake), 4096,
                                                      kw.get("out", fake), None, None, 0, kw.get("ws", 0x100000),
                                                      kw.get("wsb", ws_bytes), None)
    assert deferred(q=None) == -1
    assert deferred(out=None) == -1
    assert deferred(sl=None) == -1
    assert deferred(kv=kv_k_only) == -1
    assert deferred(ws=None) == -3
    assert deferred(wsb=1024) == -3
    from paper_2411_05787_amd.binding import _LayerState
    small = _Kv(fake, fake, 8 * 256 * 128, 256 * 128, 256)
    state = lambda **kw: _LayerState(kw.get("full", kv), kw.get("small", small), kw.get("idx", fake), kw.get("tail", fake),
                                     None, None, kw.get("need", None), None)
    wsp = (C.c_void_p * 2)(0x100000, 0x900000)
    batched = lambda layers, **kw: lib.rk_refresh_batched(C.byref(g), len(layers), (_LayerState * len(layers))(*layers),
                                                          kw.get("wsp", wsp), kw.get("wsb", ws_bytes), kw.get("sl", fake), 4096,
                                                          kw.get("k", 256), kw.get("pool", 7), kw.get("agg", 0),
                                                          kw.get("by_need", 0), None)
    assert batched([state(), state()], sl=None) == -1
    assert batched([state(), state()], k=0) == -1
    assert batched([state(), state()], k=16385) == -2
    assert batched([state(), state()], pool=4) == -1                       # even pooling width
    assert batched([state(), state()], agg=7) == -2
    assert batched([state(), state(idx=None)]) == -1
    assert batched([state(), state()], by_need=1) == -1                    # no need_full to go by
    assert batched([state(), state()], wsb=1024) == -3
    assert batched([state(), state(small=_Kv(fake, fake, 8 * 128 * 128, 128 * 128, 128))]) == -1       # fewer than k rows
    assert batched([state(), state(full=_Kv(fake, fake, 8 * 8192 * 128, 8192 * 128, 8192))]) == -2     # strides differ
    trig = lambda **kw: lib.rk_partial_attn_triggered(C.byref(g), kw.get("q", fake), kv, 256, 0, kv, fake, fake, 16, fake,
                                                     kw.get("q_ref", fake), 0.5, kw.get("sim", fake), kw.get("need", fake),
                                                     kw.get("ws", 0x100000), ws_bytes, None)
    assert trig(q_ref=None) == -1 and trig(sim=None) == -1 and trig(need=None) == -1
    assert trig(q=None) == -1
    assert trig(ws=None) == -3
    assert lib.rk_mark_refresh(C.byref(g), None, fake, None, 0, None) == -1
    assert lib.rk_workspace_init(C.byref(g), None, 4096, None) == -3
    assert lib.rk_workspace_init(C.byref(g), 0x100000, 16, None) == -3


def test_binding_refuses_cpu_tensors(rk):
    import torch
    g = rk.Geom(1, 4, 2, 128, 1.0)
    q = torch.zeros(1, 4, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        rk.rk_query_sim(g, q, torch.zeros(1, 128), 0.5, False, torch.zeros(1), torch.zeros(1, dtype=torch.int32))


def test_chunk_policy_host_logic():
    """The split policy (host logic in the binding's library) keeps partial counts bounded:
    checked through rk_workspace_bytes, which sizes the partial-result area from it."""
    import paper_2411_05787_amd as rk
    g = rk.Geom(1, 32, 8, 128, 1.0)
    small, big = rk.workspace_bytes(g, 64 * 512, 16), rk.workspace_bytes(g, 64 * 512 * 4, 16)
    # beyond 256 chunks of 128 rows the partial area stops growing; only the pooled scores (one
    # row per KV head) and the raw scores (one row per query head) grow
    assert big - small == (8 + 32) * (64 * 512 * 3) * 4
