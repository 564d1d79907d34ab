// Ragged batches: chains of different lengths in one call (the networks of Section 5 range from
// n = 15 to n = 1001 layers).  Chain c occupies elements offsets[c] .. offsets[c+1]-1 of one flat
// array.  The host sorts the chain indices by length (a counting sort: launch planning, no
// arithmetic of the method); for each group of equal length a tiled transposition through LDS
// brings the group's chains into the position-major layout, the group runs through the same
// kernels as an equal-length batch, and a second transposition puts the results where the flat
// layout wants them.  Everything is enqueued on the caller's stream.
#include "ragged_plan.h"

namespace ckpt {
namespace {

constexpr int kTile = 64;         // chains and positions per transposition tile
constexpr int kTileThreads = 256; // four waves

// Flat -> position-major for one group.  Element k of chain c is src[mult*off[c] + k], k < rows;
// it goes to stage[k*pitch + j], j the chain's place in the group.  Reads run along a chain,
// writes along the chains: both are contiguous per wave.
template <typename T>
__global__ __launch_bounds__(kTileThreads) void ragged_gather_kernel(const T *__restrict__ src,
                                                                     const int64_t *__restrict__ off,
                                                                     const int32_t *__restrict__ perm, int64_t first,
                                                                     int64_t count, int rows, int mult, int64_t pitch,
                                                                     T *__restrict__ stage)
{
    __shared__ T tile[kTile][kTile + 1];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t j0 = (int64_t)blockIdx.x * kTile;
    const int k0 = (int)blockIdx.y * kTile;
    for (int r = wave; r < kTile; r += kTileThreads / kWave) {
        const int64_t j = j0 + r;
        const int k = k0 + lane;
        if (j < count && k < rows) tile[r][lane] = src[(int64_t)mult * off[perm[first + j]] + k];
    }
    __syncthreads();
    for (int r = wave; r < kTile; r += kTileThreads / kWave) {
        const int k = k0 + r;
        const int64_t j = j0 + lane;
        if (k < rows && j < count) stage[(int64_t)k * pitch + j] = tile[lane][r];
    }
}

// Position-major -> flat: the inverse.
template <typename T>
__global__ __launch_bounds__(kTileThreads) void ragged_scatter_kernel(const T *__restrict__ stage,
                                                                      const int64_t *__restrict__ off,
                                                                      const int32_t *__restrict__ perm, int64_t first,
                                                                      int64_t count, int rows, int mult, int64_t pitch,
                                                                      T *__restrict__ dst)
{
    __shared__ T tile[kTile][kTile + 1];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t j0 = (int64_t)blockIdx.x * kTile;
    const int k0 = (int)blockIdx.y * kTile;
    for (int r = wave; r < kTile; r += kTileThreads / kWave) {
        const int k = k0 + r;
        const int64_t j = j0 + lane;
        if (k < rows && j < count) tile[lane][r] = stage[(int64_t)k * pitch + j];
    }
    __syncthreads();
    for (int r = wave; r < kTile; r += kTileThreads / kWave) {
        const int64_t j = j0 + r;
        const int k = k0 + lane;
        if (j < count && k < rows) dst[(int64_t)mult * off[perm[first + j]] + k] = tile[r][lane];
    }
}

// One value per chain back to the chain's own index.
template <typename T>
__global__ __launch_bounds__(kTileThreads) void ragged_scatter_value_kernel(const T *__restrict__ stage,
                                                                            const int32_t *__restrict__ perm,
                                                                            int64_t first, int64_t count,
                                                                            T *__restrict__ dst)
{
    const int64_t j = (int64_t)blockIdx.x * kTileThreads + threadIdx.x;
    if (j < count) dst[perm[first + j]] = stage[j];
}

struct Device {
    const int64_t *off;
    const int32_t *perm;
    int64_t *d, *wide, *peak, *budget;
    uint8_t *mask;
    int32_t *status;
    void *inner;
};

template <typename T>
void gather(const T *src, const Device &dv, const RaggedGroup &g, int rows, int mult, T *stage, hipStream_t s)
{
    const dim3 grid((unsigned)((g.count + kTile - 1) / kTile), (unsigned)((rows + kTile - 1) / kTile));
    hipLaunchKernelGGL(ragged_gather_kernel<T>, grid, dim3(kTileThreads), 0, s, src, dv.off, dv.perm, g.first, g.count,
                       rows, mult, ragged_pitch(g.count), stage);
}

template <typename T>
void scatter(const T *stage, const Device &dv, const RaggedGroup &g, int rows, int mult, T *dst, hipStream_t s)
{
    const dim3 grid((unsigned)((g.count + kTile - 1) / kTile), (unsigned)((rows + kTile - 1) / kTile));
    hipLaunchKernelGGL(ragged_scatter_kernel<T>, grid, dim3(kTileThreads), 0, s, stage, dv.off, dv.perm, g.first,
                       g.count, rows, mult, ragged_pitch(g.count), dst);
}

template <typename T>
void scatter_value(const T *stage, const Device &dv, const RaggedGroup &g, T *dst, hipStream_t s)
{
    if (!dst) return;
    hipLaunchKernelGGL(ragged_scatter_value_kernel<T>, dim3((unsigned)((g.count + kTileThreads - 1) / kTileThreads)),
                       dim3(kTileThreads), 0, s, stage, dv.perm, g.first, g.count, dst);
}

}  // namespace

int ragged_run(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host, int64_t batch,
               int objective, uint8_t *mask_out, int64_t *peak_out, int64_t *budget_out, int64_t *timeline_out,
               int32_t *status_out, const RaggedPlan &p, const RaggedWorkspace &w, void *ws, hipStream_t stream)
{
    const bool eval = which == CKPT_CALL_EVAL_PEAK || which == CKPT_CALL_EVAL_TIMELINE;
    char *base = (char *)ws;
    Device dv{(const int64_t *)(base + w.off), (const int32_t *)(base + w.perm), (int64_t *)(base + w.d),
              (int64_t *)(base + w.wide),      (int64_t *)(base + w.peak),       (int64_t *)(base + w.budget),
              (uint8_t *)(base + w.mask),      (int32_t *)(base + w.status),     base + w.inner};
    // The plan lives in host memory that ends with this call: wait until the copies have read it.
    if (hipMemcpyAsync(base + w.off, offsets_host, (size_t)(batch + 1) * 8, hipMemcpyHostToDevice, stream) !=
            hipSuccess ||
        hipMemcpyAsync(base + w.perm, p.perm.data(), (size_t)batch * 4, hipMemcpyHostToDevice, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return CKPT_ERR_DEVICE;
    for (const RaggedGroup &g : p.groups) {
        const int rows = g.n + 1;
        const Strides st{1, ragged_pitch(g.count)};
        hipError_t e = hipSuccess;
        gather(d, dv, g, rows, 1, dv.d, stream);
        if (eval) gather(mask_in, dv, g, rows, 1, dv.mask, stream);
        switch (which) {
            case CKPT_CALL_EVAL_PEAK:
                e = launch_eval_peak(dv.d, dv.mask, g.count, g.n, st, objective, dv.peak, dv.status, stream);
                break;
            case CKPT_CALL_EVAL_TIMELINE:
                e = launch_eval_timeline(dv.d, dv.mask, g.count, g.n, st, objective, dv.wide, st, dv.status, stream);
                break;
            case CKPT_CALL_SOLVE_LINEAR:
                e = launch_solve_linear(dv.d, g.count, g.n, st, dv.mask, dv.peak, dv.status, dv.inner, stream);
                break;
            default:
                e = launch_solve_cubic(dv.d, g.count, g.n, st, dv.mask, dv.peak, dv.budget, dv.status, false, nullptr,
                                       nullptr, nullptr, dv.inner, stream);
                break;
        }
        if (e != hipSuccess) return CKPT_ERR_DEVICE;
        if (which == CKPT_CALL_EVAL_TIMELINE) {
            scatter(dv.wide, dv, g, 2 * rows, 2, timeline_out, stream);
        } else {
            if (!eval) scatter(dv.mask, dv, g, rows, 1, mask_out, stream);
            scatter_value(dv.peak, dv, g, peak_out, stream);
            if (which == CKPT_CALL_SOLVE_CUBIC) scatter_value(dv.budget, dv, g, budget_out, stream);
        }
        scatter_value(dv.status, dv, g, status_out, stream);
    }
    return hipGetLastError() == hipSuccess ? CKPT_OK : CKPT_ERR_DEVICE;
}

}  // namespace ckpt
