"""Shared helpers of the GPU parity tests: tolerances and comparisons (no method arithmetic)."""
import numpy as np
import torch

import gen

OUT_MAX_ABS = 2e-2          # bf16 outputs, fp32 accumulation: bound stated for this path
IDX_REL_GAP = 1e-6          # index differences are legal only between scores this close


def bf16_val(bits: np.ndarray) -> np.ndarray:
    return gen.bits_to_bf16(bits).to(torch.float64).numpy()


def assert_out_close(gpu_bits: np.ndarray, ref_bits: np.ndarray, what: str = "out") -> float:
    """Outputs agree within 2e-2 absolute and within one bf16 step of the larger magnitude.

    Both sides round an (almost) equal real number to bf16, so they may differ by one unit in
    the last place (2^-8 relative to the binade, 2^-7 at worst) when it lies near a tie.  On top
    of that comes an absolute term: an output element is sum_j p_j v_j with sum_j p_j = 1 and
    |v_j| = O(1), the kernel carries p_j to 2^-17 (two bf16 operands) and accumulates in fp32, so
    its error is a few 1e-6 whatever the element's own size (an element of 9e-5 was seen 2.4e-6
    off); 4e-6 covers that and is 5000 times below the 2e-2 the path is held to.
    """
    a, b = bf16_val(gpu_bits), bf16_val(ref_bits)
    assert np.isfinite(a).all(), what + ": non-finite GPU output"
    d = np.abs(a - b)
    assert d.max(initial=0.0) <= OUT_MAX_ABS, "%s: max abs diff %.3g" % (what, d.max())
    ulp = np.maximum(np.abs(a), np.abs(b)) * 2.0 ** -7 + 4e-6
    worst = np.unravel_index(np.argmax(d / ulp), d.shape)
    assert (d <= ulp).all(), "%s: differs by more than one bf16 step (max %.3g at %s: gpu %.6g, oracle %.6g)" % (
        what, (d / ulp).max(), worst, a[worst], b[worst])
    return float(d.max(initial=0.0))


def assert_idx_equivalent(gpu_idx: np.ndarray, ref_idx: np.ndarray, ref_scores_all: np.ndarray, n: int,
                          k: int, what: str = "idx") -> int:
    """Selection of one (sequence, KV head): exact wherever the reference scores are apart.

    ref_scores_all[j] is the reference pooled score of position j.  Entry by entry the two lists
    must name the same position, or two positions whose reference scores differ by at most
    IDX_REL_GAP relative; a position selected by only one side must be that close to the K-th
    score.  Returns the number of entries that differ.
    """
    kk = min(k, n)
    assert (gpu_idx[kk:] == -1).all(), what + ": slots beyond min(k, len) must be -1"
    gi, ri = gpu_idx[:kk].astype(np.int64), ref_idx[:kk].astype(np.int64)
    assert ((gi >= 0) & (gi < n)).all(), what + ": index out of range"
    assert len(set(gi.tolist())) == kk, what + ": duplicate index"
    P = np.asarray(ref_scores_all, dtype=np.float64)
    diff = gi != ri
    if diff.any():
        sg, sr = P[gi[diff]], P[ri[diff]]
        assert (np.abs(sg - sr) <= IDX_REL_GAP * np.maximum(sg, sr)).all(), \
            "%s: %d entries differ across a score gap > %g" % (what, int(diff.sum()), IDX_REL_GAP)
        kth = P[ri[kk - 1]]
        for j in set(gi.tolist()) ^ set(ri.tolist()):
            assert abs(P[j] - kth) <= IDX_REL_GAP * max(P[j], kth), what + ": membership differs across a gap"
    return int(diff.sum())
