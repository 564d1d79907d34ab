// Ragged batches, host side: the grouping of the chains by length and the layout of the workspace.
// Plain host code (no kernels): it is also built on its own, under sanitizers, by the tests.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "ckpt_internal.h"

namespace ckpt {

struct RaggedPlan {
    // The sums over all groups: chains, waves of 64 chains, transposition tiles for arrays of n+1
    // rows per chain (tiles) and of 2n+2 rows (tiles2, the timelines), elements of staging for an
    // array of n+1 rows per chain, the longest chain.
    RaggedTotals t = {};
    // Ascending length; what each entry says is described at RaggedGroupDev (ckpt_internal.h).
    // Empty when the device made the plan (the tables are then in the workspace already).
    std::vector<RaggedGroupDev> groups;
    std::vector<int64_t> tile_first2;  // group g's first tile among those of the 2n+2-row arrays
};

// Byte offsets of the parts of a ragged call's workspace.  Everything before `d` has a size that
// the lengths do not change (the tables have room for a group per chain or per possible length,
// whichever is fewer), so the device can count the lengths into it before the rest is laid out.
struct RaggedWorkspace {
    size_t off = 0, perm = 0, totals = 0, hist = 0, groups = 0, tiles2 = 0, cursor = 0, d = 0, mask = 0, wide = 0,
           peak = 0, budget = 0, status = 0, inner = 0, total = 0;
};

// The most layers a chain of this call may have.
int ragged_layer_limit(int which);
// Validates the offsets and groups the chains by length.  Returns a ckpt_status.
int ragged_make_plan(const int64_t *offsets_host, int64_t batch, int max_layers, RaggedPlan &plan);
// What a finished plan must still satisfy (sizes that fit the launches).  Returns a ckpt_status.
int ragged_check_totals(const RaggedTotals &t, int64_t batch);
RaggedWorkspace ragged_layout(int which, const RaggedPlan &plan, int64_t batch);

// The device side (ragged.hip).
// The plan made on the device from the caller's device copy of the offsets: counts the lengths,
// lays the groups out into the tables of the workspace (laid out by w up to w.d, which must fit)
// and waits for the totals.  Returns a ckpt_status (CKPT_ERR_SHAPE for an offset out of range).
int ragged_plan_on_device(const int64_t *offsets_dev, int64_t batch, int max_layers, const RaggedWorkspace &w,
                          void *ws, hipStream_t stream, RaggedPlan &plan);
// Copies the group table (unless the device made it) and the offsets (unless the caller has them
// on the device already) into the workspace, waits for the copies, hands out the chains' places,
// gathers all groups into their staging, runs the solvers and scatters the results.  Returns a
// ckpt_status.
int ragged_run(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host,
               const int64_t *offsets_dev, int64_t batch, int objective, uint8_t *mask_out, int64_t *peak_out,
               int64_t *budget_out, int64_t *timeline_out, int32_t *status_out, const RaggedPlan &plan,
               const RaggedWorkspace &w, void *ws, hipStream_t stream);

}  // namespace ckpt
