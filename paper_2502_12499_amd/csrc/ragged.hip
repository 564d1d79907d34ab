// Ragged batches: chains of different lengths in one call (the networks of Section 5 range from
// n = 15 to n = 1001 layers).  Chain c occupies elements offsets[c] .. offsets[c+1]-1 of one flat
// array.  The host counts the chains of every length (launch planning, no arithmetic of the
// method) and a kernel hands every chain a place in its length's group; for each group a tiled
// transposition through LDS
// brings the group's chains into the position-major layout, the group runs through the same
// kernels as an equal-length batch, and a second transposition puts the results where the flat
// layout wants them.  Everything is enqueued on the caller's stream.
#include <vector>

#include "ragged_plan.h"

namespace ckpt {
namespace {

constexpr int kTile = 64;         // chains and positions per transposition tile
constexpr int kTileThreads = 256; // four waves

// Hands every chain a place among the chains of its length: perm[first(group) + k] = chain, k
// taken from a counter per group.  The lanes of a wave that belong to one group take their
// places together; with few groups (at most kPermLdsGroups) the waves of a workgroup first add
// up in LDS, so that a group's counter in memory is touched once per workgroup (a few lengths
// shared by a million chains would otherwise queue up on a handful of addresses).  The order
// inside a group is whatever the waves make it; everything downstream goes through perm, so the
// results do not depend on it.
constexpr int kPermThreads = 1024;
constexpr int kPermLdsGroups = 64;

__global__ __launch_bounds__(kPermThreads) void ragged_perm_kernel(const int64_t *__restrict__ off, int64_t batch,
                                                                   const RaggedGroupDev *__restrict__ groups,
                                                                   int n_groups, int32_t *__restrict__ cursor,
                                                                   int32_t *__restrict__ perm)
{
    __shared__ int32_t block_count[kPermLdsGroups];  // chains of the workgroup per group, then its base
    const bool in_lds = n_groups <= kPermLdsGroups;
    const int64_t c = (int64_t)blockIdx.x * kPermThreads + threadIdx.x;
    const int lane = threadIdx.x % kWave;
    const bool valid = c < batch;
    if (threadIdx.x < kPermLdsGroups) block_count[threadIdx.x] = 0;
    __syncthreads();
    int g = -1;
    if (valid) {
        const int32_t n = (int32_t)(off[c + 1] - off[c] - 1);
        int lo = 0, hi = n_groups - 1;  // the group of length n: it exists, the host counted this chain
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (groups[mid].n < n) lo = mid + 1; else hi = mid;
        }
        g = lo;
    }
    // a place inside the wave's share of its group, and the share's start (in the workgroup's
    // share if in_lds, else in the group)
    int32_t place = 0;
    uint64_t todo = __builtin_amdgcn_ballot_w64(valid);
    while (todo) {
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const int gl = __builtin_amdgcn_readlane(g, leader);
        const uint64_t same = __builtin_amdgcn_ballot_w64(valid && g == gl);
        const int32_t many = (int32_t)__popcll((unsigned long long)same);
        int32_t base = 0;
        if (lane == leader) base = in_lds ? atomicAdd(block_count + gl, many) : atomicAdd(cursor + gl, many);
        base = __builtin_amdgcn_readlane(base, leader);
        if (valid && g == gl) place = base + (int32_t)__popcll((unsigned long long)(same & ((1ull << lane) - 1ull)));
        todo &= ~same;
    }
    if (in_lds) {
        __syncthreads();
        if ((int)threadIdx.x < n_groups) {
            const int32_t many = block_count[threadIdx.x];
            block_count[threadIdx.x] = many > 0 ? atomicAdd(cursor + threadIdx.x, many) : 0;
        }
        __syncthreads();
        if (valid) place += block_count[g];
    }
    if (valid) perm[groups[g].first + place] = (int32_t)c;
}

__global__ void ragged_clear_kernel(int32_t *cursor, int n_groups)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g < n_groups) cursor[g] = 0;
}

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
    // the tile's elements in chain order, as many chains to a wave as fit its 64 lanes when the
    // rows are few (a chain of 16 sizes would otherwise use a quarter of a wave's load)
    const int width = min(kTile, rows - k0);  // positions of this tile
    for (int e = threadIdx.x; e < kTile * width; e += kTileThreads) {
        const int r = e / width, k = e - r * width;
        const int64_t j = j0 + r;
        if (j < count) tile[r][k] = src[(int64_t)mult * off[perm[first + j]] + k0 + k];
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
    const int width = min(kTile, rows - k0);
    for (int e = threadIdx.x; e < kTile * width; e += kTileThreads) {
        const int r = e / width, k = e - r * width;
        const int64_t j = j0 + r;
        if (j < count) dst[(int64_t)mult * off[perm[first + j]] + k0 + k] = tile[r][k];
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

int ragged_run(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host,
               const int64_t *offsets_dev, int64_t batch, int objective, uint8_t *mask_out, int64_t *peak_out, int64_t *budget_out, int64_t *timeline_out,
               int32_t *status_out, const RaggedPlan &p, const RaggedWorkspace &w, void *ws, hipStream_t stream)
{
    const bool eval = which == CKPT_CALL_EVAL_PEAK || which == CKPT_CALL_EVAL_TIMELINE;
    char *base = (char *)ws;
    Device dv{offsets_dev ? offsets_dev : (const int64_t *)(base + w.off),
              (const int32_t *)(base + w.perm), (int64_t *)(base + w.d),
              (int64_t *)(base + w.wide),      (int64_t *)(base + w.peak),       (int64_t *)(base + w.budget),
              (uint8_t *)(base + w.mask),      (int32_t *)(base + w.status),     base + w.inner};
    // The table of lengths lives in host memory that ends with this call (and the caller's offsets
    // may end with it too): wait until the copies have read them.
    std::vector<RaggedGroupDev> table;
    table.reserve(p.groups.size());
    for (const RaggedGroup &g : p.groups) table.push_back(RaggedGroupDev{(int32_t)g.n, (int32_t)g.first});
    const int n_groups = (int)table.size();
    if (hipMemcpyAsync(base + w.groups, table.data(), table.size() * sizeof(RaggedGroupDev), hipMemcpyHostToDevice,
                       stream) != hipSuccess)
        return CKPT_ERR_DEVICE;
    if (!offsets_dev && hipMemcpyAsync(base + w.off, offsets_host, (size_t)(batch + 1) * 8, hipMemcpyHostToDevice,
                                       stream) != hipSuccess)
        return CKPT_ERR_DEVICE;
    if (hipStreamSynchronize(stream) != hipSuccess) return CKPT_ERR_DEVICE;
    int32_t *cursor = (int32_t *)(base + w.cursor);
    hipLaunchKernelGGL(ragged_clear_kernel, dim3((unsigned)((n_groups + 255) / 256)), dim3(256), 0, stream, cursor,
                       n_groups);
    hipLaunchKernelGGL(ragged_perm_kernel, dim3((unsigned)((batch + kPermThreads - 1) / kPermThreads)),
                       dim3(kPermThreads), 0, stream, dv.off, batch, (const RaggedGroupDev *)(base + w.groups), n_groups,
                       cursor, (int32_t *)(base + w.perm));
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
