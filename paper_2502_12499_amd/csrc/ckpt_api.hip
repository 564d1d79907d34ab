// C-ABI entry points (declared in include/ckpt.h): host-side argument checks,
// workspace sizing, and the kernel launches.  Nothing is computed on the host.
#include "ckpt_internal.h"

namespace {

using ckpt::Strides;

int check_layout(const ckpt_layout *L, int max_layers)
{
    if (!L) return CKPT_ERR_NULL;
    if (L->batch < 0 || L->batch > INT32_MAX || L->n_layers < 1 || L->n_layers > max_layers) return CKPT_ERR_SHAPE;
    if (L->chain_stride <= 0 || L->pos_stride <= 0) return CKPT_ERR_SHAPE;
    // the largest element offset must be addressable with 63 bits
    const __int128 last = (__int128)(L->batch > 0 ? L->batch - 1 : 0) * L->chain_stride +
                          (__int128)L->n_layers * L->pos_stride;
    if (last > (__int128)INT64_MAX / 8) return CKPT_ERR_SHAPE;
    return CKPT_OK;
}

int max_layers_of(int which)
{
    return which == CKPT_CALL_SOLVE_CUBIC ? CKPT_CUBIC_MAX_LAYERS : CKPT_MAX_LAYERS;
}

int finish(hipError_t e) { return e == hipSuccess ? CKPT_OK : CKPT_ERR_DEVICE; }

// ckpt_solve_cubic and ckpt_solve_cubic_pruned: the same checks and launches
int solve_cubic(const int64_t *d, const ckpt_layout *L, uint8_t *mask_out, int64_t *peak_out, int64_t *budget_out,
                int32_t *status_out, bool pruned, int64_t *evaluated_out, void *ws, size_t ws_bytes,
                void *hip_stream, int64_t *trace_s = nullptr, int64_t *trace_cost = nullptr)
{
    const int rc = check_layout(L, CKPT_CUBIC_MAX_LAYERS);
    if (rc != CKPT_OK) return rc;
    if (L->batch == 0) return CKPT_OK;
    if (!d || !mask_out || !peak_out || !ws) return CKPT_ERR_NULL;
    if (((uintptr_t)ws & 255u) != 0 || ws_bytes < ckpt::cubic_workspace_bytes(L->batch, L->n_layers))
        return CKPT_ERR_WORKSPACE;
    return finish(ckpt::launch_solve_cubic(d, L->batch, L->n_layers, Strides{L->chain_stride, L->pos_stride},
                                           mask_out, peak_out, budget_out, status_out, pruned, evaluated_out,
                                           trace_s, trace_cost, ws, (hipStream_t)hip_stream));
}

}  // namespace

extern "C" {

size_t ckpt_workspace_bytes(int which, const ckpt_layout *L)
{
    if (which < CKPT_CALL_EVAL_PEAK || which > CKPT_CALL_EVAL_TIMELINE) return 0;
    if (check_layout(L, max_layers_of(which)) != CKPT_OK) return 0;
    switch (which) {
        case CKPT_CALL_EVAL_PEAK:
        case CKPT_CALL_EVAL_TIMELINE: return 256;
        case CKPT_CALL_SOLVE_CUBIC: return ckpt::cubic_workspace_bytes(L->batch, L->n_layers);
        default: return ckpt::linear_workspace_bytes(L->batch, L->n_layers);
    }
}

int ckpt_eval_peak(const int64_t *d, const uint8_t *mask, const ckpt_layout *L, int objective,
                   int64_t *peak_out, int32_t *status_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    (void)ws;
    (void)ws_bytes;  // the evaluation keeps all its state in registers
    const int rc = check_layout(L, CKPT_MAX_LAYERS);
    if (rc != CKPT_OK) return rc;
    if (objective != CKPT_OBJ_STATIC && objective != CKPT_OBJ_DYNAMIC && objective != CKPT_OBJ_BOTH)
        return CKPT_ERR_SHAPE;
    if (L->batch == 0) return CKPT_OK;
    if (!d || !mask || !peak_out) return CKPT_ERR_NULL;
    return finish(ckpt::launch_eval_peak(d, mask, L->batch, L->n_layers, Strides{L->chain_stride, L->pos_stride},
                                         objective, peak_out, status_out, (hipStream_t)hip_stream));
}

int ckpt_eval_timeline(const int64_t *d, const uint8_t *mask, const ckpt_layout *L, int objective,
                       int64_t *timeline_out, int64_t out_chain_stride, int64_t out_phase_stride,
                       int32_t *status_out, void *hip_stream)
{
    const int rc = check_layout(L, CKPT_MAX_LAYERS);
    if (rc != CKPT_OK) return rc;
    if (objective != CKPT_OBJ_STATIC && objective != CKPT_OBJ_DYNAMIC) return CKPT_ERR_SHAPE;
    if (out_chain_stride <= 0 || out_phase_stride <= 0) return CKPT_ERR_SHAPE;
    const __int128 last = (__int128)(L->batch > 0 ? L->batch - 1 : 0) * out_chain_stride +
                          (__int128)(2 * (int64_t)L->n_layers + 1) * out_phase_stride;
    if (last > (__int128)INT64_MAX / 8) return CKPT_ERR_SHAPE;
    if (L->batch == 0) return CKPT_OK;
    if (!d || !mask || !timeline_out) return CKPT_ERR_NULL;
    return finish(ckpt::launch_eval_timeline(d, mask, L->batch, L->n_layers,
                                             Strides{L->chain_stride, L->pos_stride}, objective, timeline_out,
                                             Strides{out_chain_stride, out_phase_stride}, status_out,
                                             (hipStream_t)hip_stream));
}

int ckpt_select_baseline(const ckpt_layout *L, int kind, uint8_t *mask_out, void *hip_stream)
{
    const int rc = check_layout(L, CKPT_MAX_LAYERS);
    if (rc != CKPT_OK) return rc;
    if (kind < CKPT_SELECT_ENDS || kind > CKPT_SELECT_SQRT) return CKPT_ERR_SHAPE;
    if (L->batch == 0) return CKPT_OK;
    if (!mask_out) return CKPT_ERR_NULL;
    return finish(ckpt::launch_select_baseline(L->batch, L->n_layers, Strides{L->chain_stride, L->pos_stride},
                                               kind, mask_out, (hipStream_t)hip_stream));
}

int ckpt_solve_cubic(const int64_t *d, const ckpt_layout *L, uint8_t *mask_out, int64_t *peak_out,
                     int64_t *budget_out, int32_t *status_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    return solve_cubic(d, L, mask_out, peak_out, budget_out, status_out, false, nullptr, ws, ws_bytes, hip_stream);
}

int ckpt_solve_cubic_pruned(const int64_t *d, const ckpt_layout *L, uint8_t *mask_out, int64_t *peak_out,
                            int64_t *budget_out, int64_t *evaluated_out, int32_t *status_out, void *ws,
                            size_t ws_bytes, void *hip_stream)
{
    return solve_cubic(d, L, mask_out, peak_out, budget_out, status_out, true, evaluated_out, ws, ws_bytes,
                       hip_stream);
}

int64_t ckpt_cubic_costs_len(int32_t n_layers)
{
    if (n_layers < 1 || n_layers > CKPT_CUBIC_MAX_LAYERS) return 0;
    return ckpt::cubic_trace_len(n_layers);
}

int ckpt_solve_cubic_costs(const int64_t *d, const ckpt_layout *L, uint8_t *mask_out, int64_t *peak_out,
                           int64_t *budget_out, int64_t *budgets_out, int64_t *costs_out, int32_t *status_out,
                           void *ws, size_t ws_bytes, void *hip_stream)
{
    if (L && L->batch > 0 && (!budgets_out || !costs_out)) return CKPT_ERR_NULL;
    return solve_cubic(d, L, mask_out, peak_out, budget_out, status_out, false, nullptr, ws, ws_bytes, hip_stream,
                       budgets_out, costs_out);
}

int ckpt_solve_linear(const int64_t *d, const ckpt_layout *L, uint8_t *mask_out, int64_t *peak_out,
                      int32_t *status_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc = check_layout(L, CKPT_MAX_LAYERS);
    if (rc != CKPT_OK) return rc;
    if (L->batch == 0) return CKPT_OK;
    if (!d || !mask_out || !peak_out || !ws) return CKPT_ERR_NULL;
    if (((uintptr_t)ws & 255u) != 0 || ws_bytes < ckpt::linear_workspace_bytes(L->batch, L->n_layers))
        return CKPT_ERR_WORKSPACE;
    return finish(ckpt::launch_solve_linear(d, L->batch, L->n_layers, Strides{L->chain_stride, L->pos_stride},
                                            mask_out, peak_out, status_out, ws, (hipStream_t)hip_stream));
}

int ckpt_solve_linear_noalloc(const int64_t *d, const ckpt_layout *L, uint8_t *mask_out, int64_t *peak_out,
                              int32_t *status_out, void *hip_stream)
{
    const int rc = check_layout(L, CKPT_NOALLOC_MAX_LAYERS);
    if (rc != CKPT_OK) return rc;
    if (L->batch > CKPT_NOALLOC_MAX_BATCH) return CKPT_ERR_SHAPE;
    if (L->batch == 0) return CKPT_OK;
    if (!d || !mask_out || !peak_out) return CKPT_ERR_NULL;
    return finish(ckpt::launch_solve_linear_noalloc(d, L->batch, L->n_layers,
                                                    Strides{L->chain_stride, L->pos_stride}, mask_out, peak_out,
                                                    status_out, (hipStream_t)hip_stream));
}

int ckpt_solve_quadratic(const int64_t *d, const ckpt_layout *L, uint8_t *mask_out, int64_t *peak_out,
                         int64_t *value_out, int32_t *status_out, void *hip_stream)
{
    const int rc = check_layout(L, CKPT_QUADRATIC_MAX_LAYERS);
    if (rc != CKPT_OK) return rc;
    if (L->batch == 0) return CKPT_OK;
    if (!d || !mask_out || !peak_out) return CKPT_ERR_NULL;
    return finish(ckpt::launch_solve_quadratic(d, L->batch, L->n_layers, Strides{L->chain_stride, L->pos_stride},
                                               mask_out, peak_out, value_out, status_out,
                                               (hipStream_t)hip_stream));
}

size_t ckpt_ragged_workspace_bytes(int which, const int64_t *offsets_host, int64_t batch)
{
    if (which < CKPT_CALL_EVAL_PEAK || which > CKPT_CALL_EVAL_TIMELINE) return 0;
    return ckpt::ragged_workspace_bytes(which, offsets_host, batch);
}

int ckpt_ragged_eval_peak(const int64_t *d, const uint8_t *mask, const int64_t *offsets_host,
                          const int64_t *offsets_dev, int64_t batch, int objective, int64_t *peak_out, int32_t *status_out, void *ws, size_t ws_bytes,
                          void *hip_stream)
{
    if (objective != CKPT_OBJ_STATIC && objective != CKPT_OBJ_DYNAMIC && objective != CKPT_OBJ_BOTH)
        return CKPT_ERR_SHAPE;
    return ckpt::launch_ragged(CKPT_CALL_EVAL_PEAK, d, mask, offsets_host, offsets_dev, batch, objective, nullptr, peak_out,
                               nullptr, nullptr, status_out, ws, ws_bytes, (hipStream_t)hip_stream);
}

int ckpt_ragged_eval_timeline(const int64_t *d, const uint8_t *mask, const int64_t *offsets_host,
                              const int64_t *offsets_dev, int64_t batch, int objective, int64_t *timeline_out, int32_t *status_out, void *ws, size_t ws_bytes,
                              void *hip_stream)
{
    if (objective != CKPT_OBJ_STATIC && objective != CKPT_OBJ_DYNAMIC) return CKPT_ERR_SHAPE;
    return ckpt::launch_ragged(CKPT_CALL_EVAL_TIMELINE, d, mask, offsets_host, offsets_dev, batch, objective, nullptr, nullptr,
                               nullptr, timeline_out, status_out, ws, ws_bytes, (hipStream_t)hip_stream);
}

int ckpt_ragged_solve_linear(const int64_t *d, const int64_t *offsets_host, const int64_t *offsets_dev,
                             int64_t batch, uint8_t *mask_out,
                             int64_t *peak_out, int32_t *status_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    return ckpt::launch_ragged(CKPT_CALL_SOLVE_LINEAR, d, nullptr, offsets_host, offsets_dev, batch, 0, mask_out, peak_out,
                               nullptr, nullptr, status_out, ws, ws_bytes, (hipStream_t)hip_stream);
}

int ckpt_ragged_solve_cubic(const int64_t *d, const int64_t *offsets_host, const int64_t *offsets_dev,
                            int64_t batch, uint8_t *mask_out,
                            int64_t *peak_out, int64_t *budget_out, int32_t *status_out, void *ws, size_t ws_bytes,
                            void *hip_stream)
{
    return ckpt::launch_ragged(CKPT_CALL_SOLVE_CUBIC, d, nullptr, offsets_host, offsets_dev, batch, 0, mask_out, peak_out,
                               budget_out, nullptr, status_out, ws, ws_bytes, (hipStream_t)hip_stream);
}

int64_t ckpt_cubic_cells(int32_t n_layers)
{
    if (n_layers < 1) return 0;
    const int64_t n = n_layers;
    return (n * (n - 1) / 2 + 1) * n;
}

const char *ckpt_status_string(int status)
{
    switch (status) {
        case CKPT_OK: return "ok";
        case CKPT_ERR_NULL: return "null pointer";
        case CKPT_ERR_SHAPE: return "bad shape, stride, objective or kind, or beyond a call's size limit";
        case CKPT_ERR_SIZE: return "non-positive size";
        case CKPT_ERR_OVERFLOW: return "sum(d)+max(d) overflows int64";
        case CKPT_ERR_MASK: return "mask does not contain both ends";
        case CKPT_ERR_WORKSPACE: return "workspace too small or misaligned";
        case CKPT_ERR_DEVICE: return "HIP launch failed";
        default: return "unknown status";
    }
}

}  // extern "C"
