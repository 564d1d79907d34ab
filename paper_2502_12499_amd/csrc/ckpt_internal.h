// Internal launch interface between the C-ABI entry points (ckpt_api.hip) and
// the kernel translation units.  Host code only validates and launches; every
// step of the path runs in the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/ckpt.h"

namespace ckpt {

constexpr int kWave = 64;

// Chain c, position k of an array laid out by a ckpt_layout.
struct Strides {
    int64_t chain;
    int64_t pos;
};

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Workgroups are handed to the eight XCDs of the chip in turn, and each XCD has its own L2.  A
// one-wave workgroup of a lane-per-chain kernel touches 64 bytes of a mask row, half a 128-byte
// line; its neighbour, which holds the other half, would run on the next XCD and fetch the line
// again.  This maps the workgroup index so that, within every 16 consecutive workgroups, the two
// that one XCD receives take neighbouring groups of chains.  A bijection on [0, grid).
__device__ inline unsigned xcd_paired_block(unsigned b, unsigned grid)
{
    constexpr unsigned kXcds = 8;
    if (b >= grid / (2 * kXcds) * (2 * kXcds)) return b;  // the ragged end keeps its order
    return (b / (2 * kXcds)) * (2 * kXcds) + (b % kXcds) * 2 + (b / kXcds) % 2;
}

// ---- wave reductions on the data-parallel-primitive path (no LDS traffic) --------------------------

constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;

// One step of a wave reduction: every lane whose DPP source exists (and whose
// row is in ROW_MASK) joins its value with the source's; the others keep theirs.
template <int CTRL, int ROW_MASK>
__device__ inline uint64_t dpp_min_step_u64(uint64_t v)
{
    const uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    const uint32_t olo = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, ROW_MASK, 0xf, false);
    const uint32_t ohi = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, ROW_MASK, 0xf, false);
    const uint64_t o = ((uint64_t)ohi << 32) | olo;
    return o < v ? o : v;
}

template <int CTRL, int ROW_MASK>
__device__ inline uint32_t dpp_min_step_u32(uint32_t v)
{
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, ROW_MASK, 0xf, false);
    return o < v ? o : v;
}

// Minimum over the wave, returned to every lane.  Shifts by 1, 2, 4, 8 inside
// each row of 16 lanes leave the row's minimum in its last lane; lane 15 is
// then broadcast into row 1 and lane 47 into row 3, lane 31 into rows 2 and 3,
// and lane 63 holds the minimum of all 64.
__device__ inline uint64_t wave_min_u64(uint64_t v)
{
    v = dpp_min_step_u64<kDppRowShr1, 0xf>(v);
    v = dpp_min_step_u64<kDppRowShr2, 0xf>(v);
    v = dpp_min_step_u64<kDppRowShr4, 0xf>(v);
    v = dpp_min_step_u64<kDppRowShr8, 0xf>(v);
    v = dpp_min_step_u64<kDppRowBcast15, 0xa>(v);
    v = dpp_min_step_u64<kDppRowBcast31, 0xc>(v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, 63);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), 63);
    return ((uint64_t)hi << 32) | lo;
}

__device__ inline uint32_t wave_min_u32(uint32_t v)
{
    v = dpp_min_step_u32<kDppRowShr1, 0xf>(v);
    v = dpp_min_step_u32<kDppRowShr2, 0xf>(v);
    v = dpp_min_step_u32<kDppRowShr4, 0xf>(v);
    v = dpp_min_step_u32<kDppRowShr8, 0xf>(v);
    v = dpp_min_step_u32<kDppRowBcast15, 0xa>(v);
    v = dpp_min_step_u32<kDppRowBcast31, 0xc>(v);
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// ---- eval_peak ---------------------------------------------------------------
hipError_t launch_eval_peak(const int64_t *d, const uint8_t *mask, int64_t batch, int n, Strides st,
                            int objective, int64_t *peak_out, int32_t *status_out, hipStream_t stream);

// ---- eval_timeline, select_baseline ------------------------------------------
hipError_t launch_eval_timeline(const int64_t *d, const uint8_t *mask, int64_t batch, int n, Strides st,
                                int objective, int64_t *out, Strides out_st, int32_t *status_out,
                                hipStream_t stream);
hipError_t launch_select_baseline(int64_t batch, int n, Strides st, int kind, uint8_t *mask_out,
                                  hipStream_t stream);

// ---- solve_linear ------------------------------------------------------------
size_t linear_workspace_bytes(int64_t batch, int n);
hipError_t launch_solve_linear(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                               int64_t *peak_out, int32_t *status_out, void *ws, hipStream_t stream);
// the same launches with the lists in an array of the library's own (batch and n within the
// CKPT_NOALLOC_* limits, checked by the caller); no allocation, no other library call
hipError_t launch_solve_linear_noalloc(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                                       int64_t *peak_out, int32_t *status_out, hipStream_t stream);

// ---- solve_quadratic ---------------------------------------------------------
hipError_t launch_solve_quadratic(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                                  int64_t *peak_out, int64_t *value_out, int32_t *status_out,
                                  hipStream_t stream);

// ---- solve_cubic -------------------------------------------------------------
size_t cubic_workspace_bytes(int64_t batch, int n);
// pruned: budgets that a sample of the budgets shows cannot be optimal are skipped (same results);
// evaluated_out (may be null) receives the number of budgets whose recurrence was run, per chain
// trace_s, trace_cost (may be null): per budget lane, the budget and its cost s + c_s in bytes
hipError_t launch_solve_cubic(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                              int64_t *peak_out, int64_t *budget_out, int32_t *status_out, bool pruned,
                              int64_t *evaluated_out, int64_t *trace_s, int64_t *trace_cost, void *ws,
                              hipStream_t stream);
// entries per chain of the two trace arrays: one per lane of the chain's waves of 64 budgets
int64_t cubic_trace_len(int n);

// ---- ragged batches ----------------------------------------------------------
// What the kernels are told about the chains of one length (a "group") when all groups of a call
// are staged side by side and taken by one launch.  Groups ascend in n; their chains have the
// places first .. first + count - 1, their waves of 64 chains the numbers wave_first .., their
// transposition tiles the numbers tile_first ..; the group's staging (position-major, `pitch`
// elements from one position to the next) starts stage_off elements into the staging arrays.
struct RaggedGroupDev {
    int32_t n;
    int32_t count;
    int32_t first;
    int32_t wave_first;
    int64_t tile_first;
    int64_t stage_off;
    int64_t pitch;
    int32_t tiles_x;  // tiles across the chains: ceil(count / 64)
    int32_t pad;
};

// The sums over the groups laid out so far (all of them at the end); `bad` is set by the device's
// count of the lengths when an offset is out of range.
struct RaggedTotals {
    int32_t n_groups, bad, max_layers, pad;
    int64_t chains, waves, tiles, tiles2, staged;
};

// Elements from one position to the next in a group's staging: rows start on 256 bytes for groups
// of 32 chains or more, on 64 bytes for smaller ones (a lone long chain is not blown up 32 times).
__host__ __device__ inline int64_t ragged_pitch(int64_t count)
{
    return count >= 32 ? (count + 31) / 32 * 32 : (count + 7) / 8 * 8;
}

// The descriptor of the group of `many` chains of n layers that follows the groups summed up in
// t, which it then joins; *tile_first2 receives the number of its first tile among those of the
// arrays with 2n+2 rows per chain.  The host's plan and the device's are both built with this.
__host__ __device__ inline RaggedGroupDev ragged_next_group(RaggedTotals &t, int n, int64_t many, int64_t *tile_first2)
{
    RaggedGroupDev g;
    g.n = n;
    g.count = (int32_t)many;
    g.first = (int32_t)t.chains;
    g.wave_first = (int32_t)t.waves;
    g.tile_first = t.tiles;
    g.stage_off = t.staged;
    g.pitch = ragged_pitch(many);
    g.tiles_x = (int32_t)((many + 63) / 64);
    g.pad = 0;
    *tile_first2 = t.tiles2;
    t.n_groups += 1;
    t.max_layers = n;
    t.chains += many;
    t.waves += (many + 63) / 64;
    t.tiles += (int64_t)g.tiles_x * ((n + 1 + 63) / 64);
    t.tiles2 += (int64_t)g.tiles_x * ((2 * n + 2 + 63) / 64);
    t.staged += ((int64_t)(n + 1) * g.pitch + 31) / 32 * 32;  // the next group starts on 256 bytes
    return g;
}

// The group that holds wave `wave`, place `place` or tile `tile` (each exists).
__device__ inline int ragged_group_of_wave(const RaggedGroupDev *g, int n_groups, int64_t wave)
{
    int lo = 0, hi = n_groups - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)g[mid].wave_first <= wave) lo = mid; else hi = mid - 1;
    }
    return lo;
}
__device__ inline int ragged_group_of_place(const RaggedGroupDev *g, int n_groups, int64_t place)
{
    int lo = 0, hi = n_groups - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)g[mid].first <= place) lo = mid; else hi = mid - 1;
    }
    return lo;
}
__device__ inline int ragged_group_of_tile(const RaggedGroupDev *g, int n_groups, int64_t tile)
{
    int lo = 0, hi = n_groups - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (g[mid].tile_first <= tile) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// All groups of a ragged call in one launch each (the staging arrays hold every group).
// batch: chains in all groups (with CKPT_OBJ_BOTH peak_stage holds 2 * batch values)
hipError_t launch_eval_peak_ragged(const int64_t *d_stage, const uint8_t *mask_stage, const RaggedGroupDev *groups,
                                   int n_groups, int64_t waves, int64_t batch, int objective, int64_t *peak_stage,
                                   int32_t *status_stage, hipStream_t stream);
hipError_t launch_eval_timeline_ragged(const int64_t *d_stage, const uint8_t *mask_stage,
                                       const RaggedGroupDev *groups, int n_groups, int64_t waves, int objective,
                                       int64_t *wide_stage, int32_t *status_stage, hipStream_t stream);
// batch: chains in all groups; max_layers: the longest chain.  ws as for launch_solve_linear(batch, max_layers).
hipError_t launch_solve_linear_ragged(const int64_t *d_stage, const RaggedGroupDev *groups, int n_groups,
                                      int64_t waves, int64_t batch, int max_layers, uint8_t *mask_stage,
                                      int64_t *peak_stage, int32_t *status_stage, void *ws, hipStream_t stream);

// which: a ckpt_call; offsets_host: batch + 1 element offsets in host memory
size_t ragged_workspace_bytes(int which, const int64_t *offsets_host, int64_t batch);
// Returns a ckpt_status.  Copies the group table (and the offsets, if offsets_dev is null) to the
// workspace and waits for the copies; everything else is enqueued on the stream.
int launch_ragged(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host,
                  const int64_t *offsets_dev, int64_t batch,
                  int objective, uint8_t *mask_out, int64_t *peak_out, int64_t *budget_out, int64_t *timeline_out,
                  int32_t *status_out, void *ws, size_t ws_bytes, hipStream_t stream);

}  // namespace ckpt
