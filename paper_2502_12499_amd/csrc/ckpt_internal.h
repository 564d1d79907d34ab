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

// ---- solve_quadratic ---------------------------------------------------------
hipError_t launch_solve_quadratic(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                                  int64_t *peak_out, int64_t *value_out, int32_t *status_out,
                                  hipStream_t stream);

// ---- solve_cubic -------------------------------------------------------------
size_t cubic_workspace_bytes(int64_t batch, int n);
// pruned: budgets that a sample of the budgets shows cannot be optimal are skipped (same results);
// evaluated_out (may be null) receives the number of budgets whose recurrence was run, per chain
hipError_t launch_solve_cubic(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                              int64_t *peak_out, int64_t *budget_out, int32_t *status_out, bool pruned,
                              int64_t *evaluated_out, void *ws, hipStream_t stream);

}  // namespace ckpt
