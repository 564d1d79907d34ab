// Ragged batches, host side (see ragged_plan.h): checks, the count of the chains of every length
// and where each length's group is staged (launch planning: none of the method's arithmetic), and
// the workspace layout.
#include <algorithm>

#include "ragged_plan.h"

namespace ckpt {

int ragged_layer_limit(int which) { return which == CKPT_CALL_SOLVE_CUBIC ? CKPT_CUBIC_MAX_LAYERS : CKPT_MAX_LAYERS; }

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
    if (off[batch] > INT64_MAX / 64) return CKPT_ERR_SHAPE;
    for (int n = 1; n <= max_layers; ++n) {
        const int64_t many = count[(size_t)n];
        if (many == 0) continue;
        int64_t first2;
        p.groups.push_back(ragged_next_group(p.t, n, many, &first2));
        p.tile_first2.push_back(first2);
    }
    return ragged_check_totals(p.t, batch);
}

int ragged_check_totals(const RaggedTotals &t, int64_t batch)
{
    // a padded staging is at most 8 times the sizes themselves (one chain to a group everywhere);
    // launches are 32-bit
    if (t.chains != batch || t.staged > INT64_MAX / 64 || t.tiles2 > 0x7fffffffLL || t.waves > 0x7fffffffLL)
        return CKPT_ERR_SHAPE;
    return CKPT_OK;
}

RaggedWorkspace ragged_layout(int which, const RaggedPlan &p, int64_t batch)
{
    // (eval_peak may be asked for both objectives: two peaks per chain)
    size_t inner = 0;
    if (which == CKPT_CALL_SOLVE_LINEAR) inner = linear_workspace_bytes(batch, p.t.max_layers);
    if (which == CKPT_CALL_SOLVE_CUBIC)
        for (const RaggedGroupDev &g : p.groups) inner = std::max(inner, cubic_workspace_bytes(g.count, g.n));
    const size_t limit = (size_t)ragged_layer_limit(which);
    const size_t room = std::min((size_t)batch, limit);  // groups at most
    RaggedWorkspace w;
    size_t at = 0;
    auto take = [&at](size_t bytes) { const size_t here = at; at += align_up(bytes); return here; };
    w.off = take((size_t)(batch + 1) * 8);
    w.perm = take((size_t)batch * 4);
    w.totals = take(sizeof(RaggedTotals));
    w.hist = take((limit + 1) * 4);  // directly behind the totals: one fill clears both
    w.groups = take(room * sizeof(RaggedGroupDev));
    w.tiles2 = take(room * 8);
    w.cursor = take(room * 4);
    w.d = take((size_t)p.t.staged * 8);
    w.mask = take((size_t)p.t.staged);
    w.wide = take(which == CKPT_CALL_EVAL_TIMELINE ? (size_t)p.t.staged * 16 : 0);
    w.peak = take((size_t)batch * (which == CKPT_CALL_EVAL_PEAK ? 16 : 8));
    w.budget = take(which == CKPT_CALL_SOLVE_CUBIC ? (size_t)batch * 8 : 0);
    w.status = take((size_t)batch * 4);
    w.inner = take(inner);
    w.total = at;
    return w;
}

size_t ragged_workspace_bytes(int which, const int64_t *offsets_host, int64_t batch)
{
    RaggedPlan p;
    if (ragged_make_plan(offsets_host, batch, ragged_layer_limit(which), p) != CKPT_OK || batch == 0) return 0;
    return ragged_layout(which, p, batch).total;
}

int launch_ragged(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host,
                  const int64_t *offsets_dev, int64_t batch,
                  int objective, uint8_t *mask_out, int64_t *peak_out, int64_t *budget_out, int64_t *timeline_out,
                  int32_t *status_out, void *ws, size_t ws_bytes, hipStream_t stream)
{
    const bool eval = which == CKPT_CALL_EVAL_PEAK || which == CKPT_CALL_EVAL_TIMELINE;
    // With the offsets on the device the lengths are counted there (a pass over the host's copy is
    // the longest step of a call on a large batch otherwise); the cubic solver is launched group
    // by group and needs the table on the host.
    const bool on_device = offsets_dev && which != CKPT_CALL_SOLVE_CUBIC;
    RaggedPlan p;
    if (!on_device) {
        const int rc = ragged_make_plan(offsets_host, batch, ragged_layer_limit(which), p);
        if (rc != CKPT_OK) return rc;
    } else if (batch < 0 || batch > INT32_MAX) {
        return CKPT_ERR_SHAPE;
    }
    if (batch == 0) return CKPT_OK;
    if (!d || !ws || (eval && !mask_in) || (!eval && !mask_out)) return CKPT_ERR_NULL;
    if (which == CKPT_CALL_EVAL_TIMELINE ? !timeline_out : !peak_out) return CKPT_ERR_NULL;
    if (((uintptr_t)ws & 255u) != 0) return CKPT_ERR_WORKSPACE;
    if (on_device) {
        const RaggedWorkspace tables = ragged_layout(which, p, batch);  // nothing staged yet: the tables only
        if (ws_bytes < tables.d) return CKPT_ERR_WORKSPACE;
        const int rc = ragged_plan_on_device(offsets_dev, batch, ragged_layer_limit(which), tables, ws, stream, p);
        if (rc != CKPT_OK) return rc;
    }
    const RaggedWorkspace w = ragged_layout(which, p, batch);
    if (ws_bytes < w.total) return CKPT_ERR_WORKSPACE;
    return ragged_run(which, d, mask_in, offsets_host, offsets_dev, batch, objective, mask_out, peak_out, budget_out, timeline_out,
                      status_out, p, w, ws, stream);
}

}  // namespace ckpt
