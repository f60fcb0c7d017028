"""The five steps of the RefreshKV decode-attention path, as plain fp64 numpy.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Each function states one
step the way the paper does, with no blocking, fusion or reordering.
"""
from typing import Optional, Tuple

import numpy as np

from .bf16 import bf16_bits_to_f64, f64_to_bf16_bits

_EPS_NORM = 1e-8   # clamp on each norm in the cosine (the paper does not say; see query_sim)


def _softmax_attention(qh: np.ndarray, keys: np.ndarray, values: np.ndarray, scale: float):
    """Scaled dot-product attention of ONE query vector over a list of rows.

    qh [D], keys [n, D], values [n, D], all fp64.  Returns (o [D], a [n], lse).
    s_j = scale * <q, k_j>;  a = softmax(s);  o = sum_j a_j v_j;  lse = log sum_j exp(s_j).
    The paper takes this as background (Section 2.1: "the model attends to tokens in
    the KV cache"); it is the textbook definition.
    """
    n = keys.shape[0]
    if n == 0:
        return np.zeros_like(qh), np.zeros(0, dtype=np.float64), -np.inf
    s = scale * (keys @ qh)
    m = s.max()
    e = np.exp(s - m)
    z = e.sum()
    a = e / z
    o = a @ values
    return o, a, m + np.log(z)


def full_attn(q_bits, k_bits, v_bits, seq_lens, scale: float
              ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Full-attention decode step (Section 2.2, "Decoding with full cache").

    Every query head attends over all ``seq_lens[b]`` rows of its KV head in the full
    cache C_f and the attention scores a_L of the current token are returned as well
    (the paper recomputes them in an extra step because its attention kernel does not
    return them: Appendix A.1, "Compatibility with Flash Attention").  "Attention
    scores" are read as the post-softmax probabilities.

    Returns (out bf16 bits [B,Hq,D], weights fp64 [B,Hq,max(seq_lens)] zero beyond each
    length, lse fp64 [B,Hq]).
    """
    q = bf16_bits_to_f64(q_bits)
    B, Hq, D = q.shape
    Hkv = k_bits.shape[1]
    G = Hq // Hkv
    lens = np.asarray(seq_lens, dtype=np.int64)
    width = int(lens.max()) if B else 0
    out = np.zeros((B, Hq, D), dtype=np.float64)
    weights = np.zeros((B, Hq, width), dtype=np.float64)
    lse = np.full((B, Hq), -np.inf, dtype=np.float64)
    for b in range(B):
        n = int(lens[b])
        for g in range(Hkv):
            keys = bf16_bits_to_f64(k_bits[b, g, :n])
            vals = bf16_bits_to_f64(v_bits[b, g, :n])
            for h in range(g * G, (g + 1) * G):
                o, a, l = _softmax_attention(q[b, h], keys, vals, scale)
                out[b, h] = o
                weights[b, h, :n] = a
                lse[b, h] = l
    return f64_to_bf16_bits(out), weights, lse


def attn_scores(q_bits, k_bits, seq_lens, scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Attention scores of the current token over the entire full cache, keys only
    (Section 4.3 "Impact of full attention steps", the setting "w/o full attention":
    the scores over the entire KV cache are calculated and the partial cache is updated
    from them, but the step then attends to the updated partial cache, so the values of
    the full cache are never read).

    a[b,h,j] = exp(s_j) / sum_i exp(s_i) with s_j = scale * <q[b,h], K[b,g(h),j]>, j < seq_lens[b].
    Returns (weights fp64 [B,Hq,max(seq_lens)] zero beyond each length, lse fp64 [B,Hq]).
    """
    q = bf16_bits_to_f64(q_bits)
    B, Hq, D = q.shape
    Hkv = k_bits.shape[1]
    G = Hq // Hkv
    lens = np.asarray(seq_lens, dtype=np.int64)
    width = int(lens.max()) if B else 0
    weights = np.zeros((B, Hq, width), dtype=np.float64)
    lse = np.full((B, Hq), -np.inf, dtype=np.float64)
    for b in range(B):
        n = int(lens[b])
        if n == 0:
            continue
        for h in range(Hq):
            keys = bf16_bits_to_f64(k_bits[b, h // G, :n])
            s = scale * (keys @ q[b, h])
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            weights[b, h, :n] = e / z
            lse[b, h] = m + np.log(z)
    return weights, lse


def window_votes(q_win_bits, k_bits, seq_lens, scale: float) -> np.ndarray:
    """Votes of an observation window of prompt tokens for the rows of the full cache.

    Section 2.2 "Prefilling stage" initialises the small cache from the attention scores
    of the last prompt token; Section 3 describes the SnapKV baseline as built from the
    scores of the last few tokens of the prompt, and Appendix A.1 "Baseline Settings"
    names the number of those tokens the observation window size (1 in all of the paper's
    runs).  For a window of W tokens the rule of the cited work is followed: every query
    head sums, over the W queries, the post-softmax scores each of them gives to a row.

    q_win bf16 bits [B, W, Hq, D]: entry i is the query of the token at position
    p_i = seq_lens[b] - W + i (the last entry is the last prompt token); entries with
    p_i < 0 do not exist and are ignored.  Attention is causal: query i sees rows
    0..p_i, its own row included.

        votes[b,h,j] = sum over i with p_i >= j of  exp(s_ij) / sum_{j' <= p_i} exp(s_ij'),
        s_ij = scale * <q_win[b,i,h], K[b,g(h),j]>

    W = 1 gives the scores a_L of the last token (``attn_scores``).  Returns fp64
    [B, Hq, max(seq_lens)], zero beyond each length.
    """
    qw = bf16_bits_to_f64(q_win_bits)
    B, W, Hq, D = qw.shape
    Hkv = k_bits.shape[1]
    G = Hq // Hkv
    lens = np.asarray(seq_lens, dtype=np.int64)
    width = int(lens.max()) if B else 0
    votes = np.zeros((B, Hq, width), dtype=np.float64)
    for b in range(B):
        n = int(lens[b])
        for i in range(W):
            pos = n - W + i
            if pos < 0:
                continue
            for h in range(Hq):
                keys = bf16_bits_to_f64(k_bits[b, h // G, :pos + 1])
                s = scale * (keys @ qw[b, i, h])
                e = np.exp(s - s.max())
                votes[b, h, :pos + 1] += e / e.sum()
    return votes


def pooled_group_scores(weights_row_group: np.ndarray, pool_w: int, agg: str = "max") -> np.ndarray:
    """Scores that rank the tokens of one (sequence, KV head).

    weights_row_group [G, n]: the attention scores of the G query heads of the group.
    1. Aggregate across the group by max (Section 2.2 footnote on GQA).  Appendix A.3 also
       tries the mean over the group and the score of the group's first head: ``agg`` =
       "max" | "mean" | "first".  The mean is taken in the dtype given (fp32 at the
       boundary), heads added in order, then divided by G: the decision is taken in the
       kernel's precision.
    2. Max-pool over neighbouring tokens, window ``pool_w`` centred on each token,
       stride 1, window clipped at both ends (Section 2.2 "Prefilling stage"; kernel
       size 7 in Appendix A.1 "Baseline Settings").  pool_w = 1 leaves step 1 as is.
    """
    if pool_w < 1 or pool_w % 2 == 0:
        raise ValueError("pool_w must be odd and >= 1")
    if agg == "max":
        A = weights_row_group.max(axis=0)
    elif agg == "first":
        A = weights_row_group[0].copy()
    elif agg == "mean":
        acc = weights_row_group[0].copy()
        for h in range(1, weights_row_group.shape[0]):
            acc = acc + weights_row_group[h]
        A = acc / weights_row_group.dtype.type(weights_row_group.shape[0])
    else:
        raise ValueError("agg must be max, mean or first")
    half = (pool_w - 1) // 2
    if half == 0 or A.shape[0] == 0:
        return A.copy()
    # clipping the window at the ends == padding with -inf, which never wins a max
    padded = np.pad(A, half, mode="constant", constant_values=-np.inf)
    windows = np.lib.stride_tricks.sliding_window_view(padded, pool_w)   # [n, pool_w]
    return windows.max(axis=1)


def topk_select(weights, seq_lens, n_kv_heads: int, k: int, pool_w: int = 7, agg: str = "max"
                ) -> Tuple[np.ndarray, np.ndarray]:
    """Pick the K tokens of each (sequence, KV head) that refresh the small cache.

    Section 2.2: the partial cache C_p is rebuilt from the top-K tokens by (pooled,
    group-aggregated) attention score of the last full step.  Order of the result:
    score descending, equal scores by ascending position (the paper is silent on ties;
    pooling makes them common).  Comparisons are done on the values as given, in the
    dtype given: no arithmetic is applied to them (except the mean of ``agg`` = "mean").

    weights [B, Hq, >=max len]; returns (idx int32 [B,Hkv,k], scores [B,Hkv,k] of
    weights' dtype); slots beyond min(k, seq_lens[b]) hold -1 / 0.
    """
    w = np.asarray(weights)
    B, Hq = w.shape[0], w.shape[1]
    G = Hq // n_kv_heads
    idx = np.full((B, n_kv_heads, k), -1, dtype=np.int32)
    sel = np.zeros((B, n_kv_heads, k), dtype=w.dtype)
    for b in range(B):
        n = int(seq_lens[b])
        kk = min(k, n)
        for g in range(n_kv_heads):
            P = pooled_group_scores(w[b, g * G:(g + 1) * G, :n], pool_w, agg)
            # stable sort on the negated score: descending score, ascending position on ties
            order = np.argsort(-P, kind="stable")
            idx[b, g, :kk] = order[:kk]
            sel[b, g, :kk] = P[order[:kk]]
    return idx, sel


def gather_small_kv(k_bits, v_bits, idx, small_k_bits, small_v_bits) -> None:
    """Rebuild the small cache C_p from rows of the full cache C_f (Section 2.2).

    small[b, g, i, :] = full[b, g, idx[b, g, i], :] for every idx >= 0 (bit copy, in place);
    slots whose idx is -1 are left as they were.
    """
    B, Hkv, k = idx.shape
    for b in range(B):
        for g in range(Hkv):
            for i in range(k):
                j = int(idx[b, g, i])
                if j >= 0:
                    small_k_bits[b, g, i, :] = k_bits[b, g, j, :]
                    small_v_bits[b, g, i, :] = v_bits[b, g, j, :]


def partial_attn(q_bits, small_k_bits, small_v_bits, n_sel: int, k_bits, v_bits,
                 tail_start, seq_lens, scale: float) -> np.ndarray:
    """Partial-attention decode step (Section 2.2, "Decoding with partial cache").

    Each query head attends over the first ``min(n_sel, tail_start[b])`` rows of the small
    cache followed by the rows of the full cache written since the last refresh,
    positions ``tail_start[b] .. seq_lens[b]-1`` (the tokens decoded with C_p, the current
    one included; the paper appends them to C_p, which is the same row list).
    With n_sel = K - (number of such rows) this is the paper's fixed-size C_p that drops
    the lowest-scored selected token per appended one, because the small cache is kept in
    descending score order.  Returns out bf16 bits [B,Hq,D].
    """
    q = bf16_bits_to_f64(q_bits)
    B, Hq, D = q.shape
    Hkv = k_bits.shape[1]
    G = Hq // Hkv
    out = np.zeros((B, Hq, D), dtype=np.float64)
    for b in range(B):
        t0, n = int(tail_start[b]), int(seq_lens[b])
        ns = max(0, min(int(n_sel), t0))
        for g in range(Hkv):
            keys = np.concatenate([bf16_bits_to_f64(small_k_bits[b, g, :ns]),
                                   bf16_bits_to_f64(k_bits[b, g, t0:n])], axis=0)
            vals = np.concatenate([bf16_bits_to_f64(small_v_bits[b, g, :ns]),
                                   bf16_bits_to_f64(v_bits[b, g, t0:n])], axis=0)
            for h in range(g * G, (g + 1) * G):
                out[b, h], _, _ = _softmax_attention(q[b, h], keys, vals, scale)
    return f64_to_bf16_bits(out)


def query_sim(q_bits, q_ref, threshold: float, force_full: bool = False,
              ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Query-similarity trigger (Section 2.2, "Deciding when to decode with full cache").

    The query vectors of the current token are averaged over all query heads of the layer
    and compared, by cosine similarity, with the averaged query of the most recent full
    step.  Similarity higher than the threshold: decode with the partial cache; otherwise
    (equal included) a full step is needed.  ``force_full`` marks a step that is full by
    schedule (fixed stride, or the t = 0 initialisation): need_full is then true whatever
    the similarity.  When a full step is taken the stored reference becomes the current
    average.

    q bf16 bits [B,Hq,D]; q_ref fp64 [B,D].  Returns (sim [B], need_full bool [B],
    new q_ref [B,D]).  Each norm is clamped below by 1e-8 (never reached by real inputs).
    """
    q = bf16_bits_to_f64(q_bits)
    q_ref = np.asarray(q_ref, dtype=np.float64)
    qbar = q.mean(axis=1)
    dot = (qbar * q_ref).sum(axis=1)
    n1 = np.maximum(np.sqrt((qbar * qbar).sum(axis=1)), _EPS_NORM)
    n2 = np.maximum(np.sqrt((q_ref * q_ref).sum(axis=1)), _EPS_NORM)
    sim = dot / (n1 * n2)
    need_full = ~(sim > threshold) | bool(force_full)
    new_ref = np.where(need_full[:, None], qbar, q_ref)
    return sim, need_full, new_ref
