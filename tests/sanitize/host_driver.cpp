// The host side of the C ABI (csrc/ckpt_api.hip: argument checks, workspace sizes, layout
// arithmetic) built for the CPU alone under AddressSanitizer and UndefinedBehaviorSanitizer by
// tests/test_sanitizers.py.  The kernel launchers are replaced by stubs that only record the
// call, so every path of the shim runs without a GPU: extreme strides and batch sizes must be
// rejected before any 64-bit product can wrap.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "../../include/ckpt.h"

#include "../../paper_2502_12499_amd/csrc/ckpt_internal.h"

namespace ckpt {
static int launches = 0;
hipError_t launch_eval_peak(const int64_t *, const uint8_t *, int64_t, int, Strides, int, int64_t *, int32_t *,
                            hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_eval_timeline(const int64_t *, const uint8_t *, int64_t, int, Strides, int, int64_t *, Strides,
                                int32_t *, hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_select_baseline(int64_t, int, Strides, int, uint8_t *, hipStream_t) { ++launches; return hipSuccess; }
size_t linear_workspace_bytes(int64_t batch, int n) { return 256 + (size_t)batch * 8 + (size_t)n * 64; }
hipError_t launch_solve_linear(const int64_t *, int64_t, int, Strides, uint8_t *, int64_t *, int32_t *, void *,
                               hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_solve_linear_noalloc(const int64_t *, int64_t, int, Strides, uint8_t *, int64_t *, int32_t *,
                                       hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_solve_quadratic(const int64_t *, int64_t, int, Strides, uint8_t *, int64_t *, int64_t *, int32_t *,
                                  hipStream_t) { ++launches; return hipSuccess; }
size_t cubic_workspace_bytes(int64_t batch, int n) { return 4096 + (size_t)batch * (size_t)n * (size_t)n * 4; }
hipError_t launch_solve_cubic(const int64_t *, int64_t, int, Strides, uint8_t *, int64_t *, int64_t *, int32_t *, bool,
                              int64_t *, int64_t *, int64_t *, void *, hipStream_t) { ++launches; return hipSuccess; }
int64_t cubic_trace_len(int n) { return ((int64_t)n * (n - 1) / 2 + 1 + 63) / 64 * 64; }
}  // namespace ckpt

// the device side of the ragged calls (csrc/ragged.hip); the plan and the layout it is handed are
// checked here for what the kernels rely on
#include "../../paper_2502_12499_amd/csrc/ragged_plan.h"
namespace ckpt {
static int ragged_runs = 0;
int ragged_run(int, const int64_t *, const uint8_t *, const int64_t *off, const int64_t *, int64_t batch, int,
               uint8_t *, int64_t *, int64_t *, int64_t *, int32_t *, const RaggedPlan &plan, const RaggedWorkspace &w,
               void *, hipStream_t)
{
    ++ragged_runs;
    // the groups ascend in length, follow each other without gaps (places, waves, tiles, staging)
    // and hold every chain of their length
    int64_t seen = 0, waves = 0, tiles = 0, tiles2 = 0, staged = 0;
    int last_n = 0;
    size_t gi = 0;
    for (const RaggedGroupDev &g : plan.groups) {
        if (g.first != seen || g.count <= 0 || g.n <= last_n) return CKPT_ERR_DEVICE;
        if (g.wave_first != waves || g.tile_first != tiles || plan.tile_first2[gi] != tiles2) return CKPT_ERR_DEVICE;
        if (g.stage_off < staged || g.stage_off % 32 != 0 || g.pitch < g.count || g.tiles_x != (g.count + 63) / 64)
            return CKPT_ERR_DEVICE;
        int64_t have = 0;
        for (int64_t c = 0; c < batch; ++c) have += off[c + 1] - off[c] - 1 == g.n;
        if (have != g.count) return CKPT_ERR_DEVICE;
        seen += g.count;
        waves += (g.count + 63) / 64;
        tiles += (int64_t)g.tiles_x * ((g.n + 1 + 63) / 64);
        tiles2 += (int64_t)g.tiles_x * ((2 * g.n + 2 + 63) / 64);
        staged = g.stage_off + (int64_t)(g.n + 1) * g.pitch;
        last_n = g.n;
        ++gi;
    }
    if (!plan.groups.empty() &&
        (seen != batch || waves != plan.t.waves || tiles != plan.t.tiles || tiles2 != plan.t.tiles2 ||
         staged > plan.t.staged || last_n != plan.t.max_layers || (int)gi != plan.t.n_groups))
        return CKPT_ERR_DEVICE;
    if (plan.t.chains != batch || plan.t.n_groups < 1 || (int64_t)plan.t.n_groups > batch) return CKPT_ERR_DEVICE;
    if (w.total % 256 != 0 || w.inner > w.total || w.totals < w.perm + (size_t)batch * 4 ||
        w.hist != w.totals + 256 || w.cursor + (size_t)plan.t.n_groups * 4 > w.d ||
        w.mask < w.d + (size_t)plan.t.staged * 8)
        return CKPT_ERR_DEVICE;
    return CKPT_OK;
}

// the device's count of the lengths: here the host's, with the tables left out as the device
// leaves them in the workspace
static int device_plans = 0;
int ragged_plan_on_device(const int64_t *offsets_dev, int64_t batch, int max_layers, const RaggedWorkspace &w, void *,
                          hipStream_t, RaggedPlan &plan)
{
    ++device_plans;
    if (w.d != w.mask || w.d % 256 != 0) return CKPT_ERR_DEVICE;  // nothing staged in the layout it is handed
    const int rc = ragged_make_plan(offsets_dev, batch, max_layers, plan);
    plan.groups.clear();
    plan.tile_first2.clear();
    return rc;
}
}  // namespace ckpt

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "host_driver: %s failed at line %d\n", #c, __LINE__); std::exit(1); } } while (0)

int main()
{
    alignas(256) static unsigned char buf[1 << 16];
    int64_t *d = (int64_t *)buf, *out = (int64_t *)(buf + 4096);
    uint8_t *mask = buf + 8192;
    void *ws = buf + 16384;
    const int64_t big = INT64_MAX;
    // layouts that must be refused before anything is multiplied out of range
    const ckpt_layout bad[] = {
        {-1, 8, 1, 4}, {4, 0, 1, 4}, {4, 65536, 1, 4}, {4, 8, 0, 4}, {4, 8, 1, 0}, {4, 8, -3, 4},
        {2147483647, 65535, big / 2, big / 2}, {2147483647, 8, big, 1}, {3, 65535, 1, big / 8},
        {(int64_t)1 << 40, 8, 1, 1},
    };
    for (const ckpt_layout &L : bad) {
        CHECK(ckpt_workspace_bytes(CKPT_CALL_SOLVE_LINEAR, &L) == 0);
        CHECK(ckpt_eval_peak(d, mask, &L, 0, out, nullptr, nullptr, 0, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_solve_linear(d, &L, mask, out, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_solve_cubic(d, &L, mask, out, nullptr, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_eval_timeline(d, mask, &L, 1, out, 1, 4, nullptr, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_select_baseline(&L, 0, mask, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_solve_quadratic(d, &L, mask, out, nullptr, nullptr, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_solve_linear_noalloc(d, &L, mask, out, nullptr, nullptr) == CKPT_ERR_SHAPE);
    }
    CHECK(ckpt::launches == 0);
    const ckpt_layout ok = {4, 8, 1, 4};
    CHECK(ckpt_eval_timeline(d, mask, &ok, 1, out, big / 2, big / 2, nullptr, nullptr) == CKPT_ERR_SHAPE);
    CHECK(ckpt_eval_peak(d, mask, &ok, 7, out, nullptr, nullptr, 0, nullptr) == CKPT_ERR_SHAPE);
    CHECK(ckpt_eval_peak(d, mask, &ok, 3, out, nullptr, nullptr, 0, nullptr) == CKPT_ERR_SHAPE);
    CHECK(ckpt_eval_timeline(d, mask, &ok, CKPT_OBJ_BOTH, out, 1, 4, nullptr, nullptr) == CKPT_ERR_SHAPE);
    CHECK(ckpt_eval_peak(nullptr, mask, &ok, 0, out, nullptr, nullptr, 0, nullptr) == CKPT_ERR_NULL);
    CHECK(ckpt_solve_linear(d, &ok, mask, out, nullptr, ws, 8, nullptr) == CKPT_ERR_WORKSPACE);
    CHECK(ckpt_solve_linear(d, &ok, mask, out, nullptr, (char *)ws + 8, 1 << 15, nullptr) == CKPT_ERR_WORKSPACE);
    CHECK(ckpt_solve_linear_noalloc(d, nullptr, mask, out, nullptr, nullptr) == CKPT_ERR_NULL);
    CHECK(ckpt::launches == 0);
    // and the calls that are in order reach their launcher exactly once each
    CHECK(ckpt_eval_peak(d, mask, &ok, 1, out, nullptr, nullptr, 0, nullptr) == CKPT_OK);
    CHECK(ckpt_eval_peak(d, mask, &ok, CKPT_OBJ_BOTH, out, nullptr, nullptr, 0, nullptr) == CKPT_OK);
    CHECK(ckpt_eval_timeline(d, mask, &ok, 0, out, 1, 4, nullptr, nullptr) == CKPT_OK);
    CHECK(ckpt_select_baseline(&ok, 2, mask, nullptr) == CKPT_OK);
    CHECK(ckpt_solve_linear(d, &ok, mask, out, nullptr, ws, 1 << 15, nullptr) == CKPT_OK);
    CHECK(ckpt_solve_linear_noalloc(d, &ok, mask, out, nullptr, nullptr) == CKPT_OK);
    CHECK(ckpt_solve_quadratic(d, &ok, mask, out, nullptr, nullptr, nullptr) == CKPT_OK);
    CHECK(ckpt_solve_cubic(d, &ok, mask, out, nullptr, nullptr, ws, 1 << 15, nullptr) == CKPT_OK);
    CHECK(ckpt_solve_cubic_pruned(d, &ok, mask, out, nullptr, nullptr, nullptr, ws, 1 << 15, nullptr) == CKPT_OK);
    CHECK(ckpt_solve_cubic_costs(d, &ok, mask, out, nullptr, nullptr, out, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_NULL);
    CHECK(ckpt_solve_cubic_costs(d, &ok, mask, out, nullptr, out, out, nullptr, ws, 1 << 15, nullptr) == CKPT_OK);
    CHECK(ckpt_cubic_costs_len(8) == 64 && ckpt_cubic_costs_len(12) == 128 && ckpt_cubic_costs_len(0) == 0);
    CHECK(ckpt::launches == 10);
    CHECK(ckpt_cubic_cells(8191) == ((int64_t)8191 * 8190 / 2 + 1) * 8191 && ckpt_cubic_cells(0) == 0);
    // ragged batches: the grouping by length and the workspace layout are host code (csrc/ragged.hip);
    // only calls that end before any device work are made here
    {
        const int64_t off[] = {0, 16, 41, 43, 59, 1061};  // n = 15, 24, 1, 15, 1001
        const int calls[] = {CKPT_CALL_EVAL_PEAK, CKPT_CALL_SOLVE_CUBIC, CKPT_CALL_SOLVE_LINEAR, CKPT_CALL_EVAL_TIMELINE};
        for (const int which : calls) {
            const size_t need = ckpt_ragged_workspace_bytes(which, off, 5);
            CHECK(need > 0 && need % 256 == 0);
            CHECK(ckpt_ragged_workspace_bytes(which, off, 0) == 0);
            CHECK(ckpt_ragged_workspace_bytes(which, nullptr, 5) == 0);
        }
        CHECK(ckpt_ragged_workspace_bytes(9, off, 5) == 0);
        const int64_t dec[] = {0, 16, 10}, tiny[] = {0, 1, 17}, neg[] = {-4, 16, 32}, huge[] = {0, big / 16, big / 8};
        const int64_t longc[] = {0, 8193};
        for (const int64_t *bad_off : {dec, tiny, neg, huge}) {
            CHECK(ckpt_ragged_workspace_bytes(CKPT_CALL_SOLVE_LINEAR, bad_off, 2) == 0);
            CHECK(ckpt_ragged_solve_linear(d, bad_off, nullptr, 2, mask, out, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_SHAPE);
            CHECK(ckpt_ragged_eval_peak(d, mask, bad_off, nullptr, 2, 0, out, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_SHAPE);
        }
        CHECK(ckpt_ragged_workspace_bytes(CKPT_CALL_SOLVE_CUBIC, longc, 1) == 0);
        CHECK(ckpt_ragged_workspace_bytes(CKPT_CALL_SOLVE_LINEAR, longc, 1) > 0);
        CHECK(ckpt_ragged_solve_cubic(d, longc, nullptr, 1, mask, out, nullptr, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_ragged_solve_linear(d, off, nullptr, -1, mask, out, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_ragged_solve_linear(d, off, nullptr, 5, nullptr, out, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_NULL);
        CHECK(ckpt_ragged_solve_linear(d, off, nullptr, 5, mask, out, nullptr, ws, 64, nullptr) == CKPT_ERR_WORKSPACE);
        CHECK(ckpt_ragged_eval_timeline(d, mask, off, nullptr, 5, 3, out, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_ragged_eval_timeline(d, mask, off, nullptr, 5, 1, nullptr, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_NULL);
        CHECK(ckpt_ragged_solve_cubic(nullptr, off, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == CKPT_OK);
        CHECK(ckpt::ragged_runs == 0);
        // calls in order reach the device side once each, with a plan that covers every chain once
        CHECK(ckpt_ragged_solve_linear(d, off, nullptr, 5, mask, out, nullptr, ws, 1 << 15, nullptr) == CKPT_ERR_WORKSPACE);
        static unsigned char big_ws[1 << 22] __attribute__((aligned(256)));
        CHECK(ckpt_ragged_solve_linear(d, off, nullptr, 5, mask, out, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_OK);
        CHECK(ckpt_ragged_eval_peak(d, mask, off, nullptr, 5, 1, out, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_OK);
        CHECK(ckpt_ragged_eval_timeline(d, mask, off, nullptr, 5, 0, out, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_OK);
        CHECK(ckpt::ragged_runs == 3);
        // with a device copy of the offsets the plan comes from the device side (not for the cubic solver)
        CHECK(ckpt::device_plans == 0);
        CHECK(ckpt_ragged_solve_linear(d, nullptr, off, 5, mask, out, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_OK);
        CHECK(ckpt_ragged_eval_timeline(d, mask, off, off, 5, 0, out, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_OK);
        CHECK(ckpt_ragged_eval_peak(d, mask, off, off, 5, 1, out, nullptr, ws, 4096, nullptr) == CKPT_ERR_WORKSPACE);
        CHECK(ckpt::device_plans == 2 && ckpt::ragged_runs == 5);
        CHECK(ckpt_ragged_solve_linear(d, off, off, -1, mask, out, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_ERR_SHAPE);
        CHECK(ckpt_ragged_solve_linear(d, off, off, 0, mask, out, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_OK);
        CHECK(ckpt_ragged_solve_linear(nullptr, off, off, 5, mask, out, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_ERR_NULL);
        CHECK(ckpt_ragged_solve_cubic(d, off, off, 5, mask, out, out + 64, nullptr, big_ws, sizeof(big_ws), nullptr) == CKPT_OK);
        CHECK(ckpt::device_plans == 2 && ckpt::ragged_runs == 6);
        // a large batch of mixed lengths: the plan's counting sort and the sizes it adds up
        const int64_t many = 200000;
        int64_t *offs = (int64_t *)std::malloc((size_t)(many + 1) * sizeof(int64_t));
        CHECK(offs != nullptr);
        offs[0] = 0;
        for (int64_t c = 0; c < many; ++c) offs[c + 1] = offs[c] + 2 + (c * 7919) % 300;
        CHECK(ckpt_ragged_workspace_bytes(CKPT_CALL_EVAL_TIMELINE, offs, many) > (size_t)many * 12);
        std::free(offs);
        CHECK(ckpt::launches == 10);
    }
    for (int s = -1; s < 10; ++s) CHECK(ckpt_status_string(s) != nullptr);
    std::printf("host_driver ok\n");
    return 0;
}
