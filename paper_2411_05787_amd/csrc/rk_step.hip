// rk_decode_step: the attention-side work of one decode step for all layers of a model, enqueued
// by one call (host code only: it sequences the library's own entry points).
//
// Section 2.2: every layer keeps its own small cache and takes its own decision.  Step 0 is the
// prefill-equivalent initialisation (full step, selection, gather, reference query).  On a fixed
// stride every S-th step is a full step for all layers.  With the query-similarity trigger every
// S-th step tests, per layer and sequence, the head-averaged query against the one of the last
// full step; both branches are enqueued and the device predicate written by the test switches
// one of them off per sequence, so nothing is read back to the host.
#include "rk_internal.h"

using namespace rk;

extern "C" int rk_decode_step(const rk_geom* geom, const rk_schedule* sched, int32_t t, int32_t n_layers,
                              const rk_layer_state* layers, const void* const* q, void* const* out,
                              const int32_t* seq_lens, int32_t max_len, int32_t max_recent,
                              void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!sched || !layers || !q || !out || !seq_lens || t < 0 || n_layers <= 0) return RK_ERR_INVALID_ARG;
    if (sched->k <= 0 || max_len <= 0 || max_recent < 0) return RK_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        const rk_layer_state& L = layers[l];
        if (!q[l] || !out[l] || !L.idx || !L.tail_start) return RK_ERR_INVALID_ARG;
        if (sched->dynamic && (!L.q_ref || !L.sim || !L.need_full)) return RK_ERR_INVALID_ARG;
    }
    const bool scheduled = t == 0 || (sched->stride > 0 && t % sched->stride == 0);
    const bool all_full = t == 0 || (scheduled && !sched->dynamic);
    const bool both = scheduled && !all_full;                // dynamic test step
    const int recent = max_recent > 0 ? max_recent : 1;

    auto partial = [&](const rk_layer_state& L, int l, const int32_t* pred, int pred_val) -> int {
        auto fn = sched->fixed_size ? rk_partial_attn_fixed : rk_partial_attn;
        return fn(geom, q[l], L.small, sched->k, L.full, L.tail_start, seq_lens, recent, out[l], pred, pred_val,
                  workspace, workspace_bytes, stream);
    };
    auto full = [&](const rk_layer_state& L, int l, const int32_t* pred) -> int {
        int r;
        if (sched->scores_only)
            r = rk_score_select(geom, q[l], L.full, seq_lens, max_len, nullptr, 0, nullptr, sched->k, sched->pool_w,
                                RK_AGG_MAX, L.idx, nullptr, pred, 1, workspace, workspace_bytes, stream);
        else
            r = rk_full_attn_select(geom, q[l], L.full, seq_lens, max_len, out[l], nullptr, 0, nullptr, sched->k,
                                    sched->pool_w, RK_AGG_MAX, L.idx, nullptr, pred, 1, workspace, workspace_bytes,
                                    stream);
        if (r != RK_OK) return r;
        r = gather_stage(geom, L.full, L.idx, sched->k, L.small, seq_lens, L.tail_start, L.n_full, pred, 1,
                         (hipStream_t)stream);
        if (r != RK_OK || !sched->scores_only) return r;
        // scores-only refresh: the output comes from the rebuilt small cache (nothing decoded since)
        return rk_partial_attn(geom, q[l], L.small, sched->k, L.full, L.tail_start, seq_lens, 1, out[l], pred, 1,
                               workspace, workspace_bytes, stream);
    };

    for (int l = 0; l < n_layers; ++l) {
        const rk_layer_state& L = layers[l];
        if (all_full) {
            if (sched->dynamic) {     // the trigger's reference follows every full step
                rc = rk_query_sim(geom, q[l], L.q_ref, sched->threshold, 1, L.sim, L.need_full, stream);
                if (rc != RK_OK) return rc;
            }
            rc = full(L, l, nullptr);
        } else if (both) {
            // the test rides on the partial step; the full step follows under the predicate it leaves
            rc = rk_partial_attn_triggered(geom, q[l], L.small, sched->k, sched->fixed_size, L.full, L.tail_start,
                                           seq_lens, recent, out[l], L.q_ref, sched->threshold, L.sim, L.need_full,
                                           workspace, workspace_bytes, stream);
            if (rc != RK_OK) return rc;
            rc = full(L, l, L.need_full);
        } else {
            rc = partial(L, l, nullptr, 0);
        }
        if (rc != RK_OK) return rc;
    }
    return all_full ? RK_STEP_FULL : both ? RK_STEP_BOTH : RK_STEP_PARTIAL;
}

// The same step with the refresh of a full step off the critical path.  The output of a full
// step is complete after rk_full_attn_pool; the selection and the gather only prepare the layer's
// next partial step, so they are enqueued on a second stream, where they run beside the full
// attention of the following layers; the streams are joined before the call returns its last
// work to `stream`.  The workspaces are used in turn: before one is reused the main stream waits
// for the selection that used it last.  Steps that are not full steps of all layers go through
// rk_decode_step unchanged (on the first workspace).
extern "C" int rk_decode_step_overlapped(const rk_geom* geom, const rk_schedule* sched, int32_t t, int32_t n_layers,
                                         const rk_layer_state* layers, const void* const* q, void* const* out,
                                         const int32_t* seq_lens, int32_t max_len, int32_t max_recent,
                                         const rk_overlap* ov, void* stream) {
    if (!ov || !ov->workspaces || ov->n_workspaces < 1 || !ov->workspaces[0]) return RK_ERR_WORKSPACE;
    if (!sched) return RK_ERR_INVALID_ARG;
    const bool scheduled = t == 0 || (sched->stride > 0 && t % sched->stride == 0);
    const bool all_full = t == 0 || (scheduled && !sched->dynamic);
    if (!all_full || sched->scores_only || ov->n_workspaces < 2)
        return rk_decode_step(geom, sched, t, n_layers, layers, q, out, seq_lens, max_len, max_recent,
                              ov->workspaces[0], ov->workspace_bytes, stream);
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!layers || !q || !out || !seq_lens || t < 0 || n_layers <= 0 || sched->k <= 0 || max_len <= 0)
        return RK_ERR_INVALID_ARG;
    if (!ov->side_stream || !ov->ready || !ov->done || !ov->join) return RK_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        const rk_layer_state& L = layers[l];
        if (!q[l] || !out[l] || !L.idx || !L.tail_start || !ov->ready[l] || !ov->done[l]) return RK_ERR_INVALID_ARG;
        if (sched->dynamic && (!L.q_ref || !L.sim || !L.need_full)) return RK_ERR_INVALID_ARG;
    }
    for (int i = 0; i < ov->n_workspaces; ++i)
        if (!ov->workspaces[i]) return RK_ERR_WORKSPACE;
    hipStream_t main = (hipStream_t)stream, side = (hipStream_t)ov->side_stream;
    auto hip_ok = [](hipError_t e) { return e == hipSuccess ? RK_OK : RK_ERR_HIP; };
    const int nw = ov->n_workspaces;
    for (int l = 0; l < n_layers; ++l) {
        const rk_layer_state& L = layers[l];
        void* ws = ov->workspaces[l % nw];
        if (l >= nw && (rc = hip_ok(hipStreamWaitEvent(main, (hipEvent_t)ov->done[l - nw], 0))) != RK_OK) return rc;
        if (sched->dynamic) {
            rc = rk_query_sim(geom, q[l], L.q_ref, sched->threshold, 1, L.sim, L.need_full, main);
            if (rc != RK_OK) return rc;
        }
        rc = rk_full_attn_pool(geom, q[l], L.full, seq_lens, max_len, out[l], nullptr, 0, nullptr, sched->pool_w,
                               RK_AGG_MAX, 1, nullptr, 0, ws, ov->workspace_bytes, main);
        if (rc != RK_OK) return rc;
        if ((rc = hip_ok(hipEventRecord((hipEvent_t)ov->ready[l], main))) != RK_OK) return rc;
        if ((rc = hip_ok(hipStreamWaitEvent(side, (hipEvent_t)ov->ready[l], 0))) != RK_OK) return rc;
        rc = rk_select_pooled(geom, seq_lens, max_len, sched->k, L.idx, nullptr, nullptr, 0, ws, ov->workspace_bytes, side);
        if (rc != RK_OK) return rc;
        rc = gather_stage(geom, L.full, L.idx, sched->k, L.small, seq_lens, L.tail_start, L.n_full, nullptr, 0, side);
        if (rc != RK_OK) return rc;
        if ((rc = hip_ok(hipEventRecord((hipEvent_t)ov->done[l], side))) != RK_OK) return rc;
    }
    if ((rc = hip_ok(hipEventRecord((hipEvent_t)ov->join, side))) != RK_OK) return rc;
    if ((rc = hip_ok(hipStreamWaitEvent(main, (hipEvent_t)ov->join, 0))) != RK_OK) return rc;
    return RK_STEP_FULL;
}

// The refreshes of all layers after their rk_full_attn_pool calls, in two launches per
// kBatchLayers layers: every selection, then every gather (+ tail_start <- seq_lens, refresh
// counters).  Nothing of it is needed before the layers' next partial step, so it can wait until
// the last layer's attention is done; batched, the selections of all layers share the chip instead
// of one layer's 8 workgroups at a time, and the gathers run at memory speed.
extern "C" int rk_refresh_batched(const rk_geom* geom, int32_t n_layers, const rk_layer_state* layers,
                                  void* const* workspaces, size_t workspace_bytes,
                                  const int32_t* seq_lens, int32_t max_len, int32_t k, int32_t pool_w, int32_t agg,
                                  int32_t by_need_full, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!layers || !workspaces || !seq_lens || n_layers <= 0 || k <= 0 || max_len <= 0) return RK_ERR_INVALID_ARG;
    if (k > RK_MAX_K) return RK_ERR_UNSUPPORTED;
    if (pool_w != 0 && (rc = rk::check_select_args(k, pool_w, agg, max_len)) != RK_OK) return rc;
    if ((int64_t)rk::kBatchLayers * geom->batch > 65535) return RK_ERR_UNSUPPORTED;
    // every argument is checked before the first launch
    for (int l = 0; l < n_layers; ++l) {
        const rk_layer_state& L = layers[l];
        rk::Workspace w;
        if (!L.idx || !L.tail_start || (by_need_full && !L.need_full)) return RK_ERR_INVALID_ARG;
        if ((rc = rk::check_workspace(geom, max_len, k, workspaces[l], workspace_bytes, &w)) != RK_OK) return rc;
        if ((rc = rk::check_kv(L.full)) != RK_OK || (rc = rk::check_kv(L.small)) != RK_OK) return rc;
        if (L.small.capacity < k) return RK_ERR_INVALID_ARG;
        if (L.full.stride_b != layers[0].full.stride_b || L.full.stride_h != layers[0].full.stride_h ||
            L.full.capacity != layers[0].full.capacity || L.small.stride_b != layers[0].small.stride_b ||
            L.small.stride_h != layers[0].small.stride_h) return RK_ERR_UNSUPPORTED;
    }
    hipStream_t st = (hipStream_t)stream;
    for (int pass = pool_w != 0 ? -1 : 0; pass < 2; ++pass) {     // (all poolings,) all selections, then all gathers
        for (int l0 = 0; l0 < n_layers; l0 += rk::kBatchLayers) {
            const int n = n_layers - l0 < rk::kBatchLayers ? n_layers - l0 : rk::kBatchLayers;
            rk::Workspace wss[rk::kBatchLayers];
            rk_kv full[rk::kBatchLayers], small[rk::kBatchLayers];
            int32_t* idx[rk::kBatchLayers]; int32_t* tail[rk::kBatchLayers]; int32_t* nref[rk::kBatchLayers];
            const int32_t* pred[rk::kBatchLayers];
            for (int l = 0; l < n; ++l) {
                const rk_layer_state& L = layers[l0 + l];
                wss[l] = rk::carve(geom, max_len, k, workspaces[l0 + l]);
                full[l] = L.full; small[l] = L.small; idx[l] = L.idx; tail[l] = L.tail_start; nref[l] = L.n_full;
                pred[l] = by_need_full ? L.need_full : nullptr;
            }
            rc = pass < 0  ? rk::pool_batched_stage(geom, n, wss, seq_lens, max_len, layers[0].full.capacity,
                                                    (pool_w - 1) / 2, agg, pred, 1, st)
               : pass == 0 ? rk::select_batched_stage(geom, n, wss, idx, seq_lens, max_len, k, pred, 1, st)
                           : rk::gather_batched_stage(geom, n, full, small, idx, k, seq_lens, tail, nref, pred, 1, st);
            if (rc != RK_OK) return rc;
        }
    }
    return RK_OK;
}

// rk_decode_step with the refreshes of a full step batched over the layers: every layer's
// rk_full_attn_deferred (workspace l), then rk_refresh_batched (pooling, selection, gather).  Steps that are not full steps of all
// layers, and the scores-only refresh, go through rk_decode_step with the first workspace.
extern "C" int rk_decode_step_batched(const rk_geom* geom, const rk_schedule* sched, int32_t t, int32_t n_layers,
                                      const rk_layer_state* layers, const void* const* q, void* const* out,
                                      const int32_t* seq_lens, int32_t max_len, int32_t max_recent,
                                      void* const* workspaces, size_t workspace_bytes, void* stream) {
    if (!workspaces || !workspaces[0]) return RK_ERR_WORKSPACE;
    if (!sched) return RK_ERR_INVALID_ARG;
    const bool scheduled = t == 0 || (sched->stride > 0 && t % sched->stride == 0);
    const bool all_full = t == 0 || (scheduled && !sched->dynamic);
    if (!scheduled || sched->scores_only)
        return rk_decode_step(geom, sched, t, n_layers, layers, q, out, seq_lens, max_len, max_recent,
                              workspaces[0], workspace_bytes, stream);
    const bool both = !all_full;                             // the trigger's test step: both branches, predicated
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!layers || !q || !out || !seq_lens || t < 0 || n_layers <= 0 || sched->k <= 0 || max_len <= 0 || max_recent < 0)
        return RK_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        const rk_layer_state& L = layers[l];
        if (!q[l] || !out[l] || !L.idx || !L.tail_start || !workspaces[l]) return RK_ERR_INVALID_ARG;
        if (sched->dynamic && (!L.q_ref || !L.sim || !L.need_full)) return RK_ERR_INVALID_ARG;
    }
    const int recent = max_recent > 0 ? max_recent : 1;
    for (int l = 0; l < n_layers; ++l) {
        const rk_layer_state& L = layers[l];
        if (both) {       // the test rides on the partial step; the full step follows under the predicate it leaves
            rc = rk_partial_attn_triggered(geom, q[l], L.small, sched->k, sched->fixed_size, L.full, L.tail_start,
                                           seq_lens, recent, out[l], L.q_ref, sched->threshold, L.sim, L.need_full,
                                           workspaces[l], workspace_bytes, stream);
            if (rc != RK_OK) return rc;
        } else if (sched->dynamic) {      // the trigger's reference follows every full step
            rc = rk_query_sim(geom, q[l], L.q_ref, sched->threshold, 1, L.sim, L.need_full, stream);
            if (rc != RK_OK) return rc;
        }
        rc = rk_full_attn_deferred(geom, q[l], L.full, seq_lens, max_len, out[l], nullptr,
                                   both ? L.need_full : nullptr, 1, workspaces[l], workspace_bytes, stream);
        if (rc != RK_OK) return rc;
    }
    rc = rk_refresh_batched(geom, n_layers, layers, workspaces, workspace_bytes, seq_lens, max_len, sched->k,
                            sched->pool_w, RK_AGG_MAX, both ? 1 : 0, stream);
    return rc != RK_OK ? rc : (both ? RK_STEP_BOTH : RK_STEP_FULL);
}
