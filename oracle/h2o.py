"""The H2O comparison policy on the same attention step (TEST INFRASTRUCTURE ONLY).

Section 3 "Comparison systems": H2O keeps the recent tokens and dynamically updated "heavy
hitters", the tokens with high cumulative attention scores.  Appendix A.1 "Baseline
Settings": the heavy-hitter part and the recent part are K/2 each, and for GQA models the
scores are aggregated over the query heads of a group by max, as for the paper's own method.
Section 4.1 notes why it is slow: it needs the attention scores at every decoding step.

The greedy rule of the cited work, per (sequence, KV head), at every decoding step:
  1. the new token's (k, v) joins the cache;
  2. the step attends over the whole cache; every cached token adds the score it received
     (aggregated over the group) to its running total;
  3. if the cache now holds more than `budget` tokens, the token with the lowest total among
     those that are not among the `recent` most recent ones is dropped, for good.
The totals are kept in fp32 and the scores are cast to fp32 before they are added (the
precision the boundary carries them in), so that the drop decision is taken on the same
numbers by every implementation; equal totals drop the older token.
"""
from typing import Dict, List

import numpy as np

from .bf16 import bf16_bits_to_f64, f64_to_bf16_bits


def h2o_decode_loop(q_steps_bits, k0_bits, v0_bits, total0, pos0, n0, new_k_bits, new_v_bits,
                    scale: float, budget: int, recent: int, agg: str = "max") -> Dict[str, object]:
    """Run T decoding steps of one layer under the H2O policy.

    State before the first step, per sequence b and KV head g: ``n0[b]`` cached tokens with
    rows k0/v0 [B,Hkv,>=max n0,D] (bf16 bits), positions pos0 [B,Hkv,>=max n0] and running
    totals total0 (fp32) - what the prefill left (the prefill's own accumulation over the
    prompt is outside this path).  Step t decodes the token at position max(pos0[b]) + 1 + t
    with query q_steps_bits[t,b] and new rows new_k_bits[t,b], new_v_bits[t,b] ([T,B,Hkv,D]).

    Returns outs (bf16 bits [T,B,Hq,D]), dropped (int64 [T,B,Hkv]: position dropped at that
    step, -1 if none), margin ([T,B,Hkv]: by how much, relative, the runner-up's total exceeded
    the dropped token's; inf where nothing or the only candidate was dropped) and the final
    caches as lists over (b, g) of dicts position -> total.
    """
    if agg not in ("max", "mean", "first"):
        raise ValueError("agg must be max, mean or first")
    if not 0 <= recent < budget:
        raise ValueError("the recent part must be smaller than the budget")
    T, B, Hq, D = q_steps_bits.shape
    Hkv = k0_bits.shape[1]
    G = Hq // Hkv
    cache: List[List[List[dict]]] = []
    for b in range(B):
        per_head = []
        for g in range(Hkv):
            per_head.append([{"pos": int(pos0[b, g, j]), "k": bf16_bits_to_f64(k0_bits[b, g, j]),
                              "v": bf16_bits_to_f64(v0_bits[b, g, j]), "total": np.float32(total0[b, g, j])}
                             for j in range(int(n0[b]))])
        cache.append(per_head)
    outs = np.zeros((T, B, Hq, D), dtype=np.float64)
    dropped = np.full((T, B, Hkv), -1, dtype=np.int64)
    margin = np.full((T, B, Hkv), np.inf)
    for b in range(B):
        first_pos = max([e["pos"] for e in cache[b][0]], default=-1) + 1
        for t in range(T):
            p = first_pos + t
            for g in range(Hkv):
                c = cache[b][g]
                c.append({"pos": p, "k": bf16_bits_to_f64(new_k_bits[t, b, g]),
                          "v": bf16_bits_to_f64(new_v_bits[t, b, g]), "total": np.float32(0.0)})
                keys = np.stack([e["k"] for e in c])
                vals = np.stack([e["v"] for e in c])
                a_heads = []
                for h in range(g * G, (g + 1) * G):
                    s = scale * (keys @ bf16_bits_to_f64(q_steps_bits[t, b, h]))
                    e = np.exp(s - s.max())
                    a = e / e.sum()
                    outs[t, b, h] = a @ vals
                    a_heads.append(a.astype(np.float32))
                if agg == "max":
                    a_g = np.max(np.stack(a_heads), axis=0)
                elif agg == "first":
                    a_g = a_heads[0]
                else:
                    acc = a_heads[0].copy()
                    for a in a_heads[1:]:
                        acc = acc + a
                    a_g = acc / np.float32(G)
                for j, e in enumerate(c):
                    e["total"] = np.float32(e["total"] + a_g[j])
                if len(c) > budget:
                    old = [e for e in c if e["pos"] <= p - recent]
                    victim = min(old, key=lambda e: (e["total"], e["pos"]))
                    dropped[t, b, g] = victim["pos"]
                    others = [float(e["total"]) for e in old if e is not victim]
                    if others:
                        margin[t, b, g] = (min(others) - float(victim["total"])) / max(min(others), 1e-30)
                    c.pop(next(i for i, e in enumerate(c) if e is victim))
    final = [[{e["pos"]: e["total"] for e in cache[b][g]} for g in range(Hkv)] for b in range(B)]
    return {"outs": f64_to_bf16_bits(outs), "dropped": dropped, "margin": margin, "final": final}
