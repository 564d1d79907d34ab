// Ragged batches, host side (see ragged_plan.h): checks, the count of the chains of every length
// (launch planning: none of the method's arithmetic) and the workspace layout.
#include <algorithm>

#include "ragged_plan.h"

namespace ckpt {

int ragged_make_plan(const int64_t *off, int64_t batch, int max_layers, RaggedPlan &p)
{
    if (batch < 0 || batch > INT32_MAX) return CKPT_ERR_SHAPE;
    if (batch == 0) return CKPT_OK;
    if (!off) return CKPT_ERR_NULL;
    if (off[0] < 0) return CKPT_ERR_SHAPE;
    // one pass: every length checked and counted
    std::vector<int64_t> count((size_t)max_layers + 2, 0);
    for (int64_t c = 0; c < batch; ++c) {
        if (off[c + 1] < off[c]) return CKPT_ERR_SHAPE;
        const int64_t len = off[c + 1] - off[c];  // (both are non-negative here: no wrap)
        if (len < 2 || len - 1 > max_layers) return CKPT_ERR_SHAPE;
        ++count[(size_t)(len - 1)];
    }
    if (off[batch] > INT64_MAX / 32) return CKPT_ERR_SHAPE;
    int64_t first = 0;
    for (int n = 1; n <= max_layers; ++n)
        if (count[(size_t)n] > 0) {
            p.groups.push_back(RaggedGroup{n, first, count[(size_t)n]});
            first += count[(size_t)n];
        }
    return CKPT_OK;
}

RaggedWorkspace ragged_layout(int which, const RaggedPlan &p, int64_t batch)
{
    size_t d = 0, mask = 0, wide = 0, vec = 0, inner = 0;
    for (const RaggedGroup &g : p.groups) {
        const size_t pitch = (size_t)ragged_pitch(g.count), rows = (size_t)g.n + 1;
        d = std::max(d, rows * pitch * 8);
        mask = std::max(mask, rows * pitch);
        vec = std::max(vec, pitch * 8);
        if (which == CKPT_CALL_EVAL_TIMELINE) wide = std::max(wide, 2 * rows * pitch * 8);
        if (which == CKPT_CALL_SOLVE_LINEAR) inner = std::max(inner, linear_workspace_bytes(g.count, g.n));
        if (which == CKPT_CALL_SOLVE_CUBIC) inner = std::max(inner, cubic_workspace_bytes(g.count, g.n));
    }
    RaggedWorkspace w;
    size_t at = 0;
    auto take = [&at](size_t bytes) { const size_t here = at; at += align_up(bytes); return here; };
    w.off = take((size_t)(batch + 1) * 8);
    w.perm = take((size_t)batch * 4);
    w.groups = take(p.groups.size() * sizeof(RaggedGroupDev));
    w.cursor = take(p.groups.size() * 4);
    w.d = take(d);
    w.mask = take(mask);
    w.wide = take(wide);
    w.peak = take(vec);
    w.budget = take(vec);
    w.status = take(vec);
    w.inner = take(inner);
    w.total = at;
    return w;
}

size_t ragged_workspace_bytes(int which, const int64_t *offsets_host, int64_t batch)
{
    RaggedPlan p;
    const int max_layers = which == CKPT_CALL_SOLVE_CUBIC ? CKPT_CUBIC_MAX_LAYERS : CKPT_MAX_LAYERS;
    if (ragged_make_plan(offsets_host, batch, max_layers, p) != CKPT_OK || batch == 0) return 0;
    return ragged_layout(which, p, batch).total;
}

int launch_ragged(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host,
                  const int64_t *offsets_dev, int64_t batch,
                  int objective, uint8_t *mask_out, int64_t *peak_out, int64_t *budget_out, int64_t *timeline_out,
                  int32_t *status_out, void *ws, size_t ws_bytes, hipStream_t stream)
{
    RaggedPlan p;
    const int max_layers = which == CKPT_CALL_SOLVE_CUBIC ? CKPT_CUBIC_MAX_LAYERS : CKPT_MAX_LAYERS;
    const int rc = ragged_make_plan(offsets_host, batch, max_layers, p);
    if (rc != CKPT_OK) return rc;
    if (batch == 0) return CKPT_OK;
    const bool eval = which == CKPT_CALL_EVAL_PEAK || which == CKPT_CALL_EVAL_TIMELINE;
    if (!d || !ws || (eval && !mask_in) || (!eval && !mask_out)) return CKPT_ERR_NULL;
    if (which == CKPT_CALL_EVAL_TIMELINE ? !timeline_out : !peak_out) return CKPT_ERR_NULL;
    const RaggedWorkspace w = ragged_layout(which, p, batch);
    if (((uintptr_t)ws & 255u) != 0 || ws_bytes < w.total) return CKPT_ERR_WORKSPACE;
    return ragged_run(which, d, mask_in, offsets_host, offsets_dev, batch, objective, mask_out, peak_out, budget_out, timeline_out,
                      status_out, p, w, ws, stream);
}

}  // namespace ckpt
