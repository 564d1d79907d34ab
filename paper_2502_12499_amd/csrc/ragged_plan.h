// Ragged batches, host side: the grouping of the chains by length and the layout of the workspace.
// Plain host code (no kernels): it is also built on its own, under sanitizers, by the tests.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "ckpt_internal.h"

namespace ckpt {

struct RaggedPlan {
    // ascending length; what each entry says is described at RaggedGroupDev (ckpt_internal.h)
    std::vector<RaggedGroupDev> groups;
    int64_t waves = 0;    // waves of 64 chains over all groups
    int64_t tiles = 0;    // transposition tiles over all groups for arrays of n+1 rows per chain ...
    int64_t tiles2 = 0;   // ... and of 2n+2 rows (the timelines); group g's start at tile_first2[g]
    std::vector<int64_t> tile_first2;
    int64_t staged = 0;   // elements of staging for an array of n+1 rows per chain, all groups
    int max_layers = 0;   // the longest chain
};

// Byte offsets of the parts of a ragged call's workspace.
struct RaggedWorkspace {
    size_t off = 0, perm = 0, groups = 0, tiles2 = 0, cursor = 0, d = 0, mask = 0, wide = 0, peak = 0, budget = 0,
           status = 0, inner = 0, total = 0;
};

// Elements from one position to the next in a group's staging: rows start on 256 bytes for groups
// of 32 chains or more, on 64 bytes for smaller ones (a lone long chain is not blown up 32 times).
inline int64_t ragged_pitch(int64_t count) { return count >= 32 ? (count + 31) / 32 * 32 : (count + 7) / 8 * 8; }

// Validates the offsets and groups the chains by length.  Returns a ckpt_status.
int ragged_make_plan(const int64_t *offsets_host, int64_t batch, int max_layers, RaggedPlan &plan);
RaggedWorkspace ragged_layout(int which, const RaggedPlan &plan, int64_t batch);

// The device side (ragged.hip): copies the group table (and the offsets, unless the caller has
// them on the device already) into the workspace, waits for the copies, hands out the chains'
// places, gathers all groups into their staging, runs the solvers and scatters the results.
// Returns a ckpt_status.
int ragged_run(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host,
               const int64_t *offsets_dev, int64_t batch, int objective, uint8_t *mask_out, int64_t *peak_out,
               int64_t *budget_out, int64_t *timeline_out, int32_t *status_out, const RaggedPlan &plan,
               const RaggedWorkspace &w, void *ws, hipStream_t stream);

}  // namespace ckpt
