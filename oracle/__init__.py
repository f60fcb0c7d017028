"""CPU oracle for the RefreshKV decode-attention path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what each step of the path computes,
written from the paper (Section 2.2 "Methodology and Implementation",
Appendix A.1 "Implementation details", Appendix A.3 "Attention score
aggregation for models with GQA").  It shares no code with the HIP library and
must never be imported by it: only ``tests/``, ``__graft_entry__.smoke()`` and
the ``cpu_baseline`` leg of ``bench.py`` may use this package.

Conventions
-----------
* bf16 tensors travel as numpy ``uint16`` arrays of bit patterns and are widened
  exactly to fp64 before any arithmetic; outputs are rounded once, from fp64 to
  bf16, round-to-nearest-even.
* Shapes: q ``[B, Hq, D]``; K, V ``[B, Hkv, cap, D]``; query head h reads KV head
  ``h // G`` with ``G = Hq // Hkv`` (the heads of one GQA group are contiguous).
* ``seq_lens[b]`` is the number of valid rows of sequence b in the full cache,
  the current token included.

Pins: every function here is pinned by ``tests/test_oracle_*.py`` against closed
forms, brute-force pure-Python loops on tiny inputs, the worked schedule of the
paper's Figure 1, and the invariants the paper states (never refreshed ==
SnapKV-style fixed set; stride 1 == vanilla attention; partial cache as large as
the context == full attention).  The quality numbers of the paper (perplexity,
ROUGE, F1) need model weights and datasets and are not reproduced: for those,
parity unpinned.
"""
from .bf16 import bf16_bits_to_f64, f64_to_bf16_bits
from .steps import (full_attn, attn_scores, window_votes, topk_select, gather_small_kv, partial_attn, query_sim,
                    pooled_group_scores)
from .loop import decode_loop, is_full_step
from .h2o import h2o_decode_loop

__all__ = ["bf16_bits_to_f64", "f64_to_bf16_bits", "full_attn", "attn_scores", "window_votes",
           "topk_select",
           "gather_small_kv", "partial_attn", "query_sim", "pooled_group_scores",
           "decode_loop", "is_full_step", "h2o_decode_loop"]
