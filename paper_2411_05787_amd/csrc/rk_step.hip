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
            rc = rk_query_sim(geom, q[l], L.q_ref, sched->threshold, 0, L.sim, L.need_full, stream);
            if (rc != RK_OK) return rc;
            rc = partial(L, l, L.need_full, 0);
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
                               RK_AGG_MAX, nullptr, 0, ws, ov->workspace_bytes, main);
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
