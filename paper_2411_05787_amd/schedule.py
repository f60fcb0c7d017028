"""Host-side schedule of one RefreshKV attention layer (Section 2.2 of the paper).

Only sequencing lives here: which of the library's calls are enqueued at step t.  Nothing is
read back from the GPU; with the dynamic trigger both branches are enqueued and the device
predicate written by ``rk_query_sim`` switches one of them off per sequence.

State of a layer (all caller-visible tensors, so a run can be checkpointed and resumed):
full cache K/V, seq_lens, small cache, idx, q_ref, tail_start, need_full.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as rk


class RefreshKVLayer:
    def __init__(self, geom: rk.Geom, K: torch.Tensor, V: torch.Tensor, seq_lens: torch.Tensor,
                 max_len: int, k_small: int, stride: int, pool_w: int = 7, dynamic: bool = False,
                 threshold: float = 0.0, evict_lowest: bool = False,
                 workspace: Optional[rk.Workspace] = None, weights: Optional[torch.Tensor] = None,
                 scores_only_refresh: bool = False):
        """K, V: bf16 [B, Hkv, capacity, D] holding seq_lens[b] rows; seq_lens int32 [B] on the
        GPU; max_len: host upper bound of seq_lens now (kept up to date by :meth:`advance`).
        scores_only_refresh: refresh steps compute the scores over the full cache, rebuild the
        small cache and attend to the rebuilt small cache alone (Section 4.3, "w/o full
        attention"); the values of the full cache are then read only by the gather."""
        dev = K.device
        B, Hq, Hkv, D = geom.batch, geom.n_q_heads, geom.n_kv_heads, geom.head_dim
        self.geom, self.K, self.V, self.seq_lens = geom, K, V, seq_lens
        self.capacity = K.shape[2]
        self.max_len = int(max_len)
        self.k_small, self.stride, self.pool_w = int(k_small), int(stride), int(pool_w)
        self.dynamic, self.threshold, self.evict_lowest = bool(dynamic), float(threshold), bool(evict_lowest)
        self.scores_only_refresh = bool(scores_only_refresh)
        self.ws = workspace if workspace is not None else rk.Workspace(geom, self.capacity, k_small, device=dev)
        self.weights = weights        # optional fp32 [B, Hq, capacity]: the weights of the last full step, if wanted
        self.small_K = torch.zeros(B, Hkv, k_small, D, dtype=torch.bfloat16, device=dev)
        self.small_V = torch.zeros(B, Hkv, k_small, D, dtype=torch.bfloat16, device=dev)
        self.idx = torch.full((B, Hkv, k_small), -1, dtype=torch.int32, device=dev)
        self.q_ref = torch.zeros(B, D, dtype=torch.float32, device=dev)
        self.sim = torch.zeros(B, dtype=torch.float32, device=dev)
        self.need_full = torch.zeros(B, dtype=torch.int32, device=dev)
        self.tail_start = seq_lens.clone()
        self.out = torch.empty(B, Hq, D, dtype=torch.bfloat16, device=dev)
        self.recent_bound = 0          # host bound of seq_lens - tail_start
        self._static = False

    def use_static_bounds(self, max_len: int, max_recent: int) -> None:
        """Freeze the host-side bounds (grid sizes) so that a step can be captured in a HIP graph
        and replayed at later steps: max_len bounds seq_lens for the whole run, max_recent bounds
        the rows decoded between two refreshes.  The kernels read the true lengths on the GPU."""
        if max_len > self.capacity:
            raise ValueError("max_len exceeds the cache capacity")
        self.max_len, self.recent_bound, self._static = int(max_len), int(max_recent), True

    # -- cache growth is the caller's copy; this keeps the host bounds in step with it
    def append(self, k_row: torch.Tensor, v_row: torch.Tensor, shared_lens: bool = False) -> None:
        """Write the new token's (k, v) rows [B, Hkv, D] at position seq_lens[b] and grow.

        shared_lens: seq_lens is shared with other layers and is incremented elsewhere."""
        if self.max_len + 1 > self.capacity:
            raise ValueError("KV cache capacity exceeded")
        B, Hkv = self.geom.batch, self.geom.n_kv_heads
        pos = self.seq_lens.to(torch.int64)[:, None, None, None].expand(B, Hkv, 1, self.geom.head_dim)
        self.K.scatter_(2, pos, k_row[:, :, None, :])
        self.V.scatter_(2, pos, v_row[:, :, None, :])
        if not shared_lens:
            self.seq_lens += 1
        self.advance()

    def advance(self) -> None:
        if not self._static:
            self.max_len += 1
            self.recent_bound += 1

    def tighten_recent_bound(self) -> int:
        """Re-reads the host bound of the rows decoded since the refresh from the GPU (max over the
        sequences of seq_lens - tail_start).  Under the trigger's schedule the host never learns of a
        refresh, so the bound only grows; results do not depend on it, launch shapes do.  Synchronises
        with the stream: for an occasional step."""
        if not self._static:
            self.recent_bound = max(int((self.seq_lens - self.tail_start).max().item()), 0)
        return self.recent_bound

    def _full(self, q, out, pred=None, stream=None) -> None:
        g = self.geom
        if self.scores_only_refresh:
            rk.rk_score_select(g, q, self.K, self.seq_lens, self.max_len, self.k_small, self.pool_w, self.idx,
                               weights=self.weights, pred=pred, pred_val=1, workspace=self.ws, stream=stream)
        else:
            rk.rk_full_attn_select(g, q, self.K, self.V, self.seq_lens, self.max_len, out, self.k_small, self.pool_w,
                                   self.idx, weights=self.weights, pred=pred, pred_val=1, workspace=self.ws,
                                   stream=stream)
        rk.rk_gather_small_kv(g, self.K, self.V, self.idx, self.k_small, self.small_K, self.small_V,
                              seq_lens=self.seq_lens, tail_start=self.tail_start,
                              pred=pred, pred_val=1, stream=stream)
        if self.scores_only_refresh:      # tail_start == seq_lens now: the K selected rows and nothing else
            rk.rk_partial_attn(g, q, self.small_K, self.small_V, self.k_small, self.K, self.V, self.tail_start,
                               self.seq_lens, 1, out, pred=pred, pred_val=1, workspace=self.ws, stream=stream)

    def prefill_init(self, q_win: torch.Tensor, stream=None) -> None:
        """Start the small cache right after the prefill (Section 2.2, "Prefilling stage"): q_win
        bf16 [B, W, Hq, D] holds the queries of the last W prompt tokens (W = 1 in the paper), whose
        rows are already in the full cache.  Selection from their votes, gather, tail_start <-
        seq_lens; with the dynamic trigger the last prompt token's query becomes the reference.
        Produces no attention output: that is the prefill's."""
        g = self.geom
        if self.dynamic:
            rk.rk_query_sim(g, q_win[:, -1].contiguous(), self.q_ref, self.threshold, True, self.sim, self.need_full,
                            stream=stream)
        rk.rk_window_select(g, q_win, self.K, self.seq_lens, self.max_len, self.k_small, self.pool_w, self.idx,
                            workspace=self.ws, stream=stream)
        rk.rk_gather_small_kv(g, self.K, self.V, self.idx, self.k_small, self.small_K, self.small_V,
                              seq_lens=self.seq_lens, tail_start=self.tail_start, stream=stream)
        if not self._static:
            self.recent_bound = 0

    def _partial(self, q, out, pred=None, stream=None) -> None:
        fn = rk.rk_partial_attn_fixed if self.evict_lowest else rk.rk_partial_attn
        fn(self.geom, q, self.small_K, self.small_V, self.k_small, self.K, self.V, self.tail_start,
           self.seq_lens, max(self.recent_bound, 1), out, pred=pred, pred_val=0, workspace=self.ws, stream=stream)

    def step(self, t: int, q: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None) -> str:
        """Attention of decode step t (t = 0: the prefill-equivalent initialisation).

        Returns which calls were enqueued: "full", "partial", or "both" (dynamic test step)."""
        out = self.out if out is None else out
        scheduled = t == 0 or (self.stride > 0 and t % self.stride == 0)
        if t == 0 or (scheduled and not self.dynamic):
            if self.dynamic:        # the trigger's reference follows every full step; a fixed stride never reads it
                rk.rk_query_sim(self.geom, q, self.q_ref, self.threshold, True, self.sim, self.need_full, stream=stream)
            self._full(q, out, stream=stream)
            if not self._static:
                self.recent_bound = 0
            return "full"
        if scheduled and self.dynamic:
            rk.rk_query_sim(self.geom, q, self.q_ref, self.threshold, False, self.sim, self.need_full, stream=stream)
            self._partial(q, out, pred=self.need_full, stream=stream)
            self._full(q, out, pred=self.need_full, stream=stream)
            return "both"
        self._partial(q, out, stream=stream)
        return "partial"


class RefreshKVModel:
    """All attention layers of a model stepped by one library call (``rk_decode_step``).

    Same schedule and state as :class:`RefreshKVLayer`, per layer; the per-layer pointers are
    packed once, so a decode step costs one foreign call whatever the number of layers.
    ``n_full[l]`` counts the refreshes of every sequence in layer l on the GPU (effective stride
    of a layer = steps / refreshes).
    """

    def __init__(self, geom: rk.Geom, kv, seq_lens: torch.Tensor, max_len: int, k_small: int, stride: int,
                 pool_w: int = 7, dynamic: bool = False, threshold: float = 0.0, evict_lowest: bool = False,
                 scores_only_refresh: bool = False, workspace: Optional[rk.Workspace] = None):
        """kv: list of (K, V) per layer, bf16 [B, Hkv, capacity, D]; seq_lens int32 [B] on the GPU,
        shared by the layers (every layer holds the same tokens)."""
        import ctypes as C
        from .binding import _Schedule, _LayerState, layer_state
        dev = kv[0][0].device
        B, Hq, Hkv, D = geom.batch, geom.n_q_heads, geom.n_kv_heads, geom.head_dim
        n = len(kv)
        self.geom, self.kv, self.seq_lens, self.n_layers = geom, kv, seq_lens, n
        self.capacity = kv[0][0].shape[2]
        self.max_len, self.k_small, self.stride = int(max_len), int(k_small), int(stride)
        self.ws = workspace if workspace is not None else rk.Workspace(geom, self.capacity, k_small, device=dev)
        self.sched = _Schedule(int(k_small), int(pool_w), int(stride), int(bool(dynamic)), float(threshold),
                               int(bool(evict_lowest)), int(bool(scores_only_refresh)))
        self.small_K = torch.zeros(n, B, Hkv, k_small, D, dtype=torch.bfloat16, device=dev)
        self.small_V = torch.zeros(n, B, Hkv, k_small, D, dtype=torch.bfloat16, device=dev)
        self.idx = torch.full((n, B, Hkv, k_small), -1, dtype=torch.int32, device=dev)
        self.q_ref = torch.zeros(n, B, D, dtype=torch.float32, device=dev)
        self.sim = torch.zeros(n, B, dtype=torch.float32, device=dev)
        self.need_full = torch.zeros(n, B, dtype=torch.int32, device=dev)
        self.tail_start = seq_lens.clone().unsqueeze(0).repeat(n, 1).contiguous()
        self.n_full = torch.zeros(n, B, dtype=torch.int32, device=dev)
        self.out = torch.empty(n, B, Hq, D, dtype=torch.bfloat16, device=dev)
        self._layers = (_LayerState * n)(*[
            layer_state(geom, kv[l][0], kv[l][1], self.small_K[l], self.small_V[l], self.idx[l], self.tail_start[l],
                        self.q_ref[l], self.sim[l], self.need_full[l], self.n_full[l], k=k_small) for l in range(n)])
        self._out_ptrs = (C.c_void_p * n)(*[self.out[l].data_ptr() for l in range(n)])
        self._q_ptrs = (C.c_void_p * n)()
        self.recent_bound = 0
        self._static = False
        self._overlap = None

    def overlap_refresh(self, n_workspaces: int = 3) -> None:
        """From now on full steps run their selections and gathers on a second stream, beside the
        following layers' full attention (``rk_decode_step_overlapped``)."""
        import ctypes as C
        from .binding import _Overlap
        n = self.n_layers
        dev = self.out.device
        self._side = torch.cuda.Stream(device=dev)
        self._wss = [self.ws] + [rk.Workspace(self.geom, self.capacity, self.k_small, device=dev)
                                 for _ in range(max(int(n_workspaces), 2) - 1)]
        self._events = [torch.cuda.Event() for _ in range(2 * n + 1)]
        for e in self._events:          # an event gets its handle when it is first recorded
            e.record()
        torch.cuda.synchronize(dev)
        handles = [e.cuda_event for e in self._events]
        self._ready = (C.c_void_p * n)(*handles[:n])
        self._done = (C.c_void_p * n)(*handles[n:2 * n])
        self._ws_ptrs = (C.c_void_p * len(self._wss))(*[w_.ptr for w_ in self._wss])
        self._overlap = _Overlap(self._side.cuda_stream, self._ready, self._done, handles[2 * n], self._ws_ptrs,
                                 len(self._wss), min(w_.nbytes for w_ in self._wss))

    def batched_refresh(self) -> None:
        """From now on full steps run every layer's attention first (one workspace per layer) and then all
        selections and all gathers in one launch each (``rk_decode_step_batched``)."""
        import ctypes as C
        dev = self.out.device
        self._wss = [self.ws] + [rk.Workspace(self.geom, self.capacity, self.k_small, device=dev)
                                 for _ in range(self.n_layers - 1)]
        self._batched_ptrs = (C.c_void_p * self.n_layers)(*[w_.ptr for w_ in self._wss])
        self._batched_bytes = min(w_.nbytes for w_ in self._wss)
        self._overlap = None

    def use_static_bounds(self, max_len: int, max_recent: int) -> None:
        if max_len > self.capacity:
            raise ValueError("max_len exceeds the cache capacity")
        self.max_len, self.recent_bound, self._static = int(max_len), int(max_recent), True

    def advance(self) -> None:
        """The caller has appended one token to every layer's full cache and to seq_lens."""
        if not self._static:
            if self.max_len + 1 > self.capacity:
                raise ValueError("KV cache capacity exceeded")
            self.max_len += 1
            self.recent_bound += 1

    def tighten_recent_bound(self) -> int:
        """Re-reads the host bound of the rows decoded since a refresh from the GPU: max over layers and
        sequences of seq_lens - tail_start.  With the trigger's schedule the host never learns of a
        refresh (the decision stays on the GPU), so its bound grows by one per step; the results do not
        depend on it (the kernels clamp on the device-side lengths) but launch shapes do.  This call
        synchronises with the stream: meant for an occasional step, not for every one."""
        if not self._static:
            r = int((self.seq_lens.unsqueeze(0) - self.tail_start).max().item())
            self.recent_bound = max(r, 0)
        return self.recent_bound

    def step(self, t: int, q: torch.Tensor, stream=None) -> str:
        """q: bf16 [n_layers, B, Hq, D] on the GPU (the query of the current token in every layer).
        Outputs land in ``self.out[l]``."""
        n, g = self.n_layers, self.geom
        if not q.is_cuda or q.dtype != torch.bfloat16 or not q.is_contiguous() or \
                tuple(q.shape) != (n, g.batch, g.n_q_heads, g.head_dim):
            raise ValueError("q must be a contiguous bf16 GPU tensor [n_layers, batch, n_q_heads, head_dim]")
        base, step_bytes = q.data_ptr(), q.stride(0) * 2
        for l in range(n):
            self._q_ptrs[l] = base + l * step_bytes
        if getattr(self, "_batched_ptrs", None) is not None:
            kind = rk.rk_decode_step_batched(g, self.sched, t, self._layers, self._q_ptrs, self._out_ptrs, self.seq_lens,
                                             self.max_len, max(self.recent_bound, 1), self._batched_ptrs,
                                             self._batched_bytes, stream=stream)
        elif self._overlap is not None:
            kind = rk.rk_decode_step_overlapped(g, self.sched, t, self._layers, self._q_ptrs, self._out_ptrs,
                                                self.seq_lens, self.max_len, max(self.recent_bound, 1), self._overlap,
                                                stream=stream)
        else:
            kind = rk.rk_decode_step(g, self.sched, t, self._layers, self._q_ptrs, self._out_ptrs, self.seq_lens,
                                     self.max_len, max(self.recent_bound, 1), workspace=self.ws, stream=stream)
        if kind == "full" and not self._static:
            self.recent_bound = 0
        return kind


class RefreshKVStack:
    """The layers of a model stepped in order, full steps with the refresh off the critical path.

    The output of a full step is complete once ``rk_full_attn_pool`` has run; the selection and
    the gather only prepare the layer's NEXT partial step.  Here they go to a second stream, where
    they run beside the full attention of the following layers (in a model: beside the rest of
    the layer), and the streams join at the end of the step.  A layer's pooled scores must survive
    until its selection has read them: ``n_workspaces`` workspaces are used in turn, and the main
    stream waits for the selection that last used a workspace before it reuses it.  Three measured
    best at 32 layers of 32k tokens (full step 46.8 us per layer; two: 50.0, four: 48.2, one per
    layer: 57, where the second stream falls behind and its kernels crowd later layers).  Partial
    steps and the trigger's test steps are issued as :class:`RefreshKVLayer` issues them.

    Submission: a full step issued (or its graph replayed) while many earlier steps are still
    pending leaves the second stream's queue blocked behind all of them, and on this hardware a
    blocked queue slows every dispatch of the first one (measured: +0.9 us per layer on each partial
    step in between).  A driver loop should therefore submit a full step late, when at most one
    earlier step is still pending (wait on the event that ended the step before the last).
    """

    def __init__(self, layers, n_workspaces: int = 3, batched: bool = False, deferred: bool = True):
        """batched: no second stream; a full step runs ``rk_full_attn_deferred`` (``rk_full_attn_pool``
        with deferred=False, or where a layer wants the weights of the step) for every layer (one
        workspace per layer) and then ``rk_refresh_batched``: (all poolings,) all selections and all
        gathers, each in one launch, after the last layer's attention."""
        if not layers:
            raise ValueError("no layers")
        l0 = layers[0]
        if l0.scores_only_refresh:
            raise ValueError("the scores-only refresh is not split over two streams")
        self.layers = layers
        dev = l0.K.device
        self.batched = bool(batched)
        self.deferred = bool(deferred) and all(lay.weights is None for lay in layers)
        if self.batched:
            import ctypes as C
            from .binding import _LayerState, layer_state
            n = len(layers)
            self.wss = [l0.ws] + [rk.Workspace(l0.geom, l0.capacity, l0.k_small, device=dev) for _ in range(n - 1)]
            self._states = (_LayerState * n)(*[layer_state(l0.geom, lay.K, lay.V, lay.small_K, lay.small_V, lay.idx,
                                                           lay.tail_start, k=lay.k_small) for lay in layers])
            self._ws_ptrs = (C.c_void_p * n)(*[w_.ptr for w_ in self.wss])
            self._ws_bytes = min(w_.nbytes for w_ in self.wss)
            return
        n_ws = len(layers) if n_workspaces <= 0 else max(2, min(int(n_workspaces), len(layers)))
        self.wss = [l0.ws] + [rk.Workspace(l0.geom, l0.capacity, l0.k_small, device=dev) for _ in range(n_ws - 1)]
        self.side = torch.cuda.Stream(device=dev)
        self.ready = [torch.cuda.Event() for _ in layers]
        self.done = [torch.cuda.Event() for _ in layers]

    def step(self, t: int, q_layers) -> str:
        """q_layers[l]: bf16 [B, Hq, D], the query of the current token in layer l."""
        l0 = self.layers[0]
        scheduled = t == 0 or (l0.stride > 0 and t % l0.stride == 0)
        if not (t == 0 or (scheduled and not l0.dynamic)):
            kind = None
            for l, lay in enumerate(self.layers):
                kind = lay.step(t, q_layers[l])
            return kind
        main = torch.cuda.current_stream()
        if self.batched:
            for l, lay in enumerate(self.layers):
                if lay.dynamic:
                    rk.rk_query_sim(lay.geom, q_layers[l], lay.q_ref, lay.threshold, True, lay.sim, lay.need_full, stream=main)
                if self.deferred:
                    rk.rk_full_attn_deferred(lay.geom, q_layers[l], lay.K, lay.V, lay.seq_lens, lay.max_len, lay.out,
                                             workspace=self.wss[l], stream=main)
                else:
                    rk.rk_full_attn_pool(lay.geom, q_layers[l], lay.K, lay.V, lay.seq_lens, lay.max_len, lay.out,
                                         lay.pool_w, weights=lay.weights, workspace=self.wss[l], stream=main)
                if not lay._static:
                    lay.recent_bound = 0
            rk.rk_refresh_batched(l0.geom, self._states, self._ws_ptrs, self._ws_bytes, l0.seq_lens, l0.max_len,
                                  l0.k_small, pool_w=l0.pool_w if self.deferred else 0, stream=main)
            return "full"
        for l, lay in enumerate(self.layers):
            n_ws = len(self.wss)
            ws = self.wss[l % n_ws]
            if l >= n_ws:                   # the selection of layer l - n_ws must be done with this workspace
                main.wait_event(self.done[l - n_ws])
            q, g = q_layers[l], lay.geom
            if lay.dynamic:
                rk.rk_query_sim(g, q, lay.q_ref, lay.threshold, True, lay.sim, lay.need_full, stream=main)
            rk.rk_full_attn_pool(g, q, lay.K, lay.V, lay.seq_lens, lay.max_len, lay.out, lay.pool_w,
                                 weights=lay.weights, workspace=ws, stream=main, beside_other_work=True)
            self.ready[l].record(main)
            self.side.wait_event(self.ready[l])
            rk.rk_select_pooled(g, lay.seq_lens, lay.max_len, lay.k_small, lay.idx, workspace=ws, stream=self.side)
            rk.rk_gather_small_kv(g, lay.K, lay.V, lay.idx, lay.k_small, lay.small_K, lay.small_V,
                                  seq_lens=lay.seq_lens, tail_start=lay.tail_start, stream=self.side)
            self.done[l].record(self.side)
            if not lay._static:
                lay.recent_bound = 0
        main.wait_stream(self.side)         # the next step reads the small caches
        return "full"
