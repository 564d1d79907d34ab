// Ragged batches, host side: the grouping of the chains by length and the layout of the workspace.
// Plain host code (no kernels): it is also built on its own, under sanitizers, by the tests.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "ckpt_internal.h"

namespace ckpt {

struct RaggedGroup {
    int n;
    int64_t first;  // index into perm of the group's first chain
    int64_t count;
};

struct RaggedPlan {
    std::vector<RaggedGroup> groups;  // ascending length; group g's chains take places first .. first + count - 1
};

// What the device is told about a group (the places themselves are handed out on the device).
struct RaggedGroupDev {
    int32_t n;
    int32_t first;
};

// Byte offsets of the parts of a ragged call's workspace.
struct RaggedWorkspace {
    size_t off = 0, perm = 0, groups = 0, cursor = 0, d = 0, mask = 0, wide = 0, peak = 0, budget = 0, status = 0,
           inner = 0, total = 0;
};

// rows of the staging start on 256 bytes
inline int64_t ragged_pitch(int64_t count) { return (count + 31) / 32 * 32; }

// Validates the offsets and groups the chains by length.  Returns a ckpt_status.
int ragged_make_plan(const int64_t *offsets_host, int64_t batch, int max_layers, RaggedPlan &plan);
// Staging is sized for the group that needs most of each part.
RaggedWorkspace ragged_layout(int which, const RaggedPlan &plan, int64_t batch);

// The device side (ragged.hip): copies the group table (and the offsets, unless the caller has
// them on the device already) into the workspace, waits for the copies, hands out the chains'
// places, and enqueues gather, the equal-length kernels and scatter for every group.  Returns a
// ckpt_status.
int ragged_run(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host,
               const int64_t *offsets_dev, int64_t batch,
               int objective, uint8_t *mask_out, int64_t *peak_out, int64_t *budget_out, int64_t *timeline_out,
               int32_t *status_out, const RaggedPlan &plan, const RaggedWorkspace &w, void *ws, hipStream_t stream);

}  // namespace ckpt
