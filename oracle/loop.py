"""The RefreshKV decode schedule around the five steps (TEST INFRASTRUCTURE ONLY).

One attention layer, every sequence of the batch independent.  Follows Section 2.2:
prefill-equivalent initialisation, then alternate partial and full steps, either on a
fixed stride or on the query-similarity trigger tested every S-th step.
"""
from typing import Dict, List

import numpy as np

from .steps import full_attn, attn_scores, topk_select, gather_small_kv, partial_attn, query_sim


def is_full_step(t: int, stride: int) -> bool:
    """Fixed schedule: decode steps are numbered from 1 and every S-th one is full.

    Figure 1 (L=5, K=3, S=3, four generated tokens): t = 1, 2, 4 use the partial cache,
    t = 3 the full one.  t = 0 stands for the prefill, which always attends to everything.
    """
    return t == 0 or (stride > 0 and t % stride == 0)


def decode_loop(q_steps_bits, k_bits, v_bits, new_k_bits, new_v_bits, seq_lens0, scale: float,
                k_small: int, stride: int, pool_w: int = 7, dynamic: bool = False,
                threshold: float = 0.0, evict_lowest: bool = False,
                weights_dtype=np.float32, scores_only_refresh: bool = False) -> Dict[str, object]:
    """Run T decode steps of one layer.

    q_steps_bits [T+1,B,Hq,D] (index 0: the query of the last prompt token, which
    initialises the small cache: Section 2.2 "Prefilling stage"); k_bits/v_bits
    [B,Hkv,cap,D] full cache holding ``seq_lens0[b]`` rows (copied, then grown by one row
    per step: the row is written to the full cache at once, which gives the same
    attention inputs as the paper's deferred flush); new_*_bits [T,B,Hkv,D].

    stride <= 0 means "never refresh after the initialisation".  ``dynamic``: on every
    S-th step the trigger decides per sequence; otherwise every S-th step is full.
    ``evict_lowest``: partial steps read K - r selected rows (r = rows appended since the
    refresh), the paper's fixed-size C_p; otherwise all K selected rows plus the r new ones.
    The attention scores are cast to ``weights_dtype`` (the boundary's fp32) before ranking.
    ``scores_only_refresh``: the "w/o full attention" setting of Section 4.3: a refresh step
    computes the scores over the whole cache, rebuilds the small cache from them and then
    attends to the rebuilt small cache alone (its K rows; nothing has been decoded since).

    Returns outs (bf16 bits [T+1,B,Hq,D]), full (bool [T+1,B]), sims ([T+1,B], nan where
    not tested), idx (list over t of int32 [B,Hkv,K] snapshots taken after each step),
    rows (int64 [T+1,B]: KV rows attended per KV head at that step).
    """
    T = new_k_bits.shape[0]
    B, Hq, D = q_steps_bits.shape[1:]
    Hkv = k_bits.shape[1]
    kf = np.array(k_bits, copy=True)
    vf = np.array(v_bits, copy=True)
    lens = np.array(seq_lens0, dtype=np.int64).copy()
    small_k = np.zeros((B, Hkv, k_small, D), dtype=np.uint16)
    small_v = np.zeros((B, Hkv, k_small, D), dtype=np.uint16)
    idx = np.full((B, Hkv, k_small), -1, dtype=np.int32)
    tail_start = lens.copy()
    q_ref = np.zeros((B, D), dtype=np.float64)

    outs = np.zeros((T + 1, B, Hq, D), dtype=np.uint16)
    full = np.zeros((T + 1, B), dtype=bool)
    sims = np.full((T + 1, B), np.nan)
    rows = np.zeros((T + 1, B), dtype=np.int64)
    idx_hist: List[np.ndarray] = []

    for t in range(T + 1):
        if t >= 1:
            for b in range(B):
                kf[b, :, lens[b], :] = new_k_bits[t - 1, b]
                vf[b, :, lens[b], :] = new_v_bits[t - 1, b]
            lens += 1
        q = q_steps_bits[t]
        scheduled = is_full_step(t, stride)
        for b in range(B):
            sl = slice(b, b + 1)
            if t == 0 or (scheduled and not dynamic):
                _, _, q_ref[sl] = query_sim(q[sl], q_ref[sl], threshold, force_full=True)
                do_full = True
            elif scheduled and dynamic:
                s, need, q_ref[sl] = query_sim(q[sl], q_ref[sl], threshold, force_full=False)
                sims[t, b] = s[0]
                do_full = bool(need[0])
            else:
                do_full = False
            full[t, b] = do_full
            if do_full:
                if scores_only_refresh:
                    w, _ = attn_scores(q[sl], kf[sl], lens[sl], scale)
                else:
                    o, w, _ = full_attn(q[sl], kf[sl], vf[sl], lens[sl], scale)
                i_b, _ = topk_select(w.astype(weights_dtype), lens[sl], Hkv, k_small, pool_w)
                idx[sl] = i_b
                gather_small_kv(kf[sl], vf[sl], idx[sl], small_k[sl], small_v[sl])
                tail_start[b] = lens[b]
                rows[t, b] = lens[b]
                if scores_only_refresh:
                    o = partial_attn(q[sl], small_k[sl], small_v[sl], k_small, kf[sl], vf[sl],
                                     tail_start[sl], lens[sl], scale)
                    rows[t, b] = min(k_small, int(lens[b]))
            else:
                r = int(lens[b] - tail_start[b])
                n_sel = max(k_small - r, 0) if evict_lowest else k_small
                o = partial_attn(q[sl], small_k[sl], small_v[sl], n_sel, kf[sl], vf[sl],
                                 tail_start[sl], lens[sl], scale)
                rows[t, b] = min(n_sel, int(tail_start[b])) + r
            outs[t, b] = o[0]
        idx_hist.append(idx.copy())
    return {"outs": outs, "full": full, "sims": sims, "idx": idx_hist, "rows": rows,
            "k": kf, "v": vf, "lens": lens}
