// Ragged batches: chains of different lengths in one call (the networks of Section 5 range from
// n = 15 to n = 1001 layers).  Chain c occupies elements offsets[c] .. offsets[c+1]-1 of one flat
// array.  The host counts the chains of every length (launch planning, no arithmetic of the
// method) and decides where each length's group is staged; a kernel hands every chain a place in
// its group; a tiled transposition through LDS brings all groups into position-major staging at
// once; eval_peak, eval_timeline and solve_linear then take every group in one launch (a wave looks
// up the group its chains belong to), the cubic solver group by group; a second
// transposition puts the results where the flat layout wants them.  Everything is enqueued on
// the caller's stream.
#include <vector>

#include "ragged_plan.h"

namespace ckpt {
namespace {

constexpr int kTile = 64;         // chains and positions per transposition tile
constexpr int kTileThreads = 256; // four waves

// ---- the plan made on the device ------------------------------------------------------------
// When the caller has the offsets in device memory, the lengths are counted here instead of on the
// host: ragged_count_kernel checks every offset and counts the chains of every length (hist[n]),
// ragged_layout_kernel turns the counts into the table of groups, exactly as the host would
// (ragged_next_group), and the host reads back the totals only: how many waves, tiles and bytes of
// staging the launches that follow need.
constexpr int kCountThreads = 1024;
constexpr int kCountLds = 4096;  // lengths below this are first added up per workgroup in LDS

__global__ __launch_bounds__(kCountThreads) void ragged_count_kernel(const int64_t *__restrict__ off, int64_t batch,
                                                                     int max_layers, uint32_t *__restrict__ hist,
                                                                     RaggedTotals *__restrict__ totals)
{
    __shared__ uint32_t near_count[kCountLds];
    for (int b = threadIdx.x; b < kCountLds; b += kCountThreads) near_count[b] = 0;
    __syncthreads();
    const int64_t c = (int64_t)blockIdx.x * kCountThreads + threadIdx.x;
    const int lane = threadIdx.x % kWave;
    constexpr uint64_t kMaxOffset = (uint64_t)(INT64_MAX / 64);
    bool ok = false;
    uint32_t n = 0;
    if (c < batch) {
        // every offset in 0 .. INT64_MAX / 64 (a negative one reads as huge), so the difference is
        // exact, and a decreasing pair wraps to a huge length
        const uint64_t lo = (uint64_t)off[c], hi = (uint64_t)off[c + 1];
        const uint64_t below = hi - lo - 2;  // n - 1
        ok = below <= (uint64_t)(max_layers - 1) && hi <= kMaxOffset && lo <= kMaxOffset;
        n = (uint32_t)below + 1u;
        if (!ok) totals->bad = 1;  // (every writer writes the same value)
    }
    // the lanes of a wave that hold the same length count together
    uint64_t todo = __builtin_amdgcn_ballot_w64(ok);
    while (todo) {
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const uint32_t nl = (uint32_t)__builtin_amdgcn_readlane((int)n, leader);
        const uint64_t same = __builtin_amdgcn_ballot_w64(ok && n == nl);
        if (lane == leader) {
            const uint32_t many = (uint32_t)__popcll((unsigned long long)same);
            if (nl < (uint32_t)kCountLds) atomicAdd(near_count + nl, many); else atomicAdd(hist + nl, many);
        }
        todo &= ~same;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kCountLds && b <= max_layers; b += kCountThreads) {
        const uint32_t many = near_count[b];
        if (many) atomicAdd(hist + b, many);
    }
}

// Exclusive prefix sum of one value per thread over the workgroup (kCountThreads threads);
// `wave_sum` is LDS for one value per wave.
__device__ inline int64_t block_exclusive_sum(int64_t v, int64_t *wave_sum)
{
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    int64_t incl = v;
#pragma unroll
    for (int s = 1; s < kWave; s <<= 1) {
        const int64_t up = __shfl_up(incl, s, kWave);
        if (lane >= s) incl += up;
    }
    __syncthreads();  // (the previous call's readers are done with wave_sum)
    if (lane == kWave - 1) wave_sum[wave] = incl;
    __syncthreads();
    int64_t before = 0;
    for (int k = 0; k < wave; ++k) before += wave_sum[k];
    return before + incl - v;
}

// One workgroup: thread t takes the lengths t*span+1 .. (t+1)*span, first adds up what its groups
// contribute to the totals, then, knowing the totals of the threads before it, writes their
// descriptors.  The last thread's totals are the call's.
__global__ __launch_bounds__(kCountThreads) void ragged_layout_kernel(const uint32_t *__restrict__ hist, int max_layers,
                                                                      RaggedGroupDev *__restrict__ groups,
                                                                      int64_t *__restrict__ tile_first2,
                                                                      RaggedTotals *__restrict__ totals)
{
    __shared__ int64_t wave_sum[kCountThreads / kWave];
    __shared__ int longest;
    if (threadIdx.x == 0) longest = 0;
    const int span = (max_layers + kCountThreads - 1) / kCountThreads;
    const int n_lo = (int)threadIdx.x * span + 1, n_hi = min(n_lo + span - 1, max_layers);
    RaggedTotals mine = {};
    for (int n = n_lo; n <= n_hi; ++n) {
        const int64_t many = hist[n];
        int64_t unused;
        if (many) (void)ragged_next_group(mine, n, many, &unused);
    }
    RaggedTotals t = {};
    t.n_groups = (int32_t)block_exclusive_sum(mine.n_groups, wave_sum);
    t.chains = block_exclusive_sum(mine.chains, wave_sum);
    t.waves = block_exclusive_sum(mine.waves, wave_sum);
    t.tiles = block_exclusive_sum(mine.tiles, wave_sum);
    t.tiles2 = block_exclusive_sum(mine.tiles2, wave_sum);
    t.staged = block_exclusive_sum(mine.staged, wave_sum);
    for (int n = n_lo; n <= n_hi; ++n) {
        const int64_t many = hist[n];
        if (!many) continue;
        const int at = t.n_groups;
        int64_t first2;
        groups[at] = ragged_next_group(t, n, many, &first2);
        tile_first2[at] = first2;
    }
    if (mine.n_groups) atomicMax(&longest, mine.max_layers);
    __syncthreads();
    if (threadIdx.x == kCountThreads - 1) {
        totals->n_groups = t.n_groups;
        totals->max_layers = longest;
        totals->chains = t.chains;
        totals->waves = t.waves;
        totals->tiles = t.tiles;
        totals->tiles2 = t.tiles2;
        totals->staged = t.staged;
    }
}

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

// Flat -> position-major, every group in one launch.  A workgroup takes one tile of 64 chains x 64
// rows of one group (found from the tile's number).  Element k of chain c is src[mult*off[c] + k],
// k < rows = mult * (n + 1); it goes to stage[mult*stage_off + k*pitch + j], j the chain's place
// in its group.  Reads run along a chain (several short chains to a wave), writes along the
// chains: both are contiguous per wave.
struct TileAt {
    RaggedGroupDev g;
    int64_t j0;  // first chain of the tile within the group
    int k0;      // first row
    int rows;
};

__device__ inline TileAt tile_at(const RaggedGroupDev *groups, const int64_t *tile_first2, int n_groups, int mult)
{
    TileAt t;
    int gi;
    int64_t local;
    if (mult == 1) {
        gi = ragged_group_of_tile(groups, n_groups, blockIdx.x);
        local = (int64_t)blockIdx.x - groups[gi].tile_first;
    } else {  // the tiles of the arrays with 2n+2 rows per chain are numbered on their own
        int lo = 0, hi = n_groups - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (tile_first2[mid] <= (int64_t)blockIdx.x) lo = mid; else hi = mid - 1;
        }
        gi = lo;
        local = (int64_t)blockIdx.x - tile_first2[gi];
    }
    t.g = groups[gi];
    t.rows = mult * (t.g.n + 1);
    t.j0 = (local % t.g.tiles_x) * kTile;
    t.k0 = (int)(local / t.g.tiles_x) * kTile;
    return t;
}

// Where the tile's part of each of its 64 chains starts in the flat array (element index), looked
// up once per tile; the caller synchronises before use.
__device__ inline void tile_chains(const TileAt &t, const int64_t *__restrict__ off, const int32_t *__restrict__ perm,
                                   int mult, int64_t *chain_at)
{
    if (threadIdx.x < kTile) {
        const int64_t j = t.j0 + threadIdx.x;
        chain_at[threadIdx.x] = j < t.g.count ? (int64_t)mult * off[perm[t.g.first + j]] + t.k0 : 0;
    }
}

// The workgroup's threads laid along the chains of a tile `width` rows wide (1..64): a thread keeps
// one row k of the tile and walks the chains; width is rounded up to a power of two so that a
// thread's chain and row are a shift and a mask away.
struct AlongChain {
    int shift, width;
    __device__ explicit AlongChain(int w) : shift(w > 1 ? 32 - __builtin_clz((unsigned)w - 1u) : 0), width(w) {}
    __device__ int k() const { return (int)threadIdx.x & ((1 << shift) - 1); }
    __device__ bool active() const { return k() < width; }
    __device__ int first_chain() const { return (int)threadIdx.x >> shift; }
    __device__ int chains_per_pass() const { return kTileThreads >> shift; }
};

template <typename T>
__global__ __launch_bounds__(kTileThreads) void ragged_gather_kernel(const T *__restrict__ src,
                                                                     const int64_t *__restrict__ off,
                                                                     const int32_t *__restrict__ perm,
                                                                     const RaggedGroupDev *__restrict__ groups,
                                                                     const int64_t *__restrict__ tile_first2,
                                                                     int n_groups, int mult, T *__restrict__ stage)
{
    __shared__ T tile[kTile][kTile + 1];
    __shared__ int64_t chain_at[kTile];
    const TileAt t = tile_at(groups, tile_first2, n_groups, mult);
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t count = t.g.count;
    tile_chains(t, off, perm, mult, chain_at);
    __syncthreads();
    const AlongChain a(min(kTile, t.rows - t.k0));
    for (int r = a.first_chain(); r < kTile; r += a.chains_per_pass())
        if (a.active() && t.j0 + r < count) tile[r][a.k()] = src[chain_at[r] + a.k()];
    __syncthreads();
    T *out = stage + (int64_t)mult * t.g.stage_off;
    for (int r = wave; r < kTile; r += kTileThreads / kWave) {
        const int k = t.k0 + r;
        const int64_t j = t.j0 + lane;
        if (k < t.rows && j < count) out[(int64_t)k * t.g.pitch + j] = tile[lane][r];
    }
}

// Position-major -> flat: the inverse.
template <typename T>
__global__ __launch_bounds__(kTileThreads) void ragged_scatter_kernel(const T *__restrict__ stage,
                                                                      const int64_t *__restrict__ off,
                                                                      const int32_t *__restrict__ perm,
                                                                      const RaggedGroupDev *__restrict__ groups,
                                                                      const int64_t *__restrict__ tile_first2,
                                                                      int n_groups, int mult, T *__restrict__ dst)
{
    __shared__ T tile[kTile][kTile + 1];
    __shared__ int64_t chain_at[kTile];
    const TileAt t = tile_at(groups, tile_first2, n_groups, mult);
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t count = t.g.count;
    tile_chains(t, off, perm, mult, chain_at);
    const T *in = stage + (int64_t)mult * t.g.stage_off;
    for (int r = wave; r < kTile; r += kTileThreads / kWave) {
        const int k = t.k0 + r;
        const int64_t j = t.j0 + lane;
        if (k < t.rows && j < count) tile[lane][r] = in[(int64_t)k * t.g.pitch + j];
    }
    __syncthreads();
    const AlongChain a(min(kTile, t.rows - t.k0));
    for (int r = a.first_chain(); r < kTile; r += a.chains_per_pass())
        if (a.active() && t.j0 + r < count) dst[chain_at[r] + a.k()] = tile[r][a.k()];
}

// One value per chain from its place back to the chain's own index, all groups at once.
template <typename T>
__global__ __launch_bounds__(kTileThreads) void ragged_scatter_value_kernel(const T *__restrict__ stage,
                                                                            const int32_t *__restrict__ perm,
                                                                            int64_t batch, T *__restrict__ dst)
{
    const int64_t p = (int64_t)blockIdx.x * kTileThreads + threadIdx.x;
    if (p < batch) dst[perm[p]] = stage[p];
}

template <typename T>
void scatter_value(const T *stage, const int32_t *perm, int64_t batch, T *dst, hipStream_t s)
{
    if (!dst) return;
    hipLaunchKernelGGL(ragged_scatter_value_kernel<T>, dim3((unsigned)((batch + kTileThreads - 1) / kTileThreads)),
                       dim3(kTileThreads), 0, s, stage, perm, batch, dst);
}

}  // namespace

int ragged_plan_on_device(const int64_t *offsets_dev, int64_t batch, int max_layers, const RaggedWorkspace &w,
                          void *ws, hipStream_t stream, RaggedPlan &p)
{
    char *base = (char *)ws;
    RaggedTotals *totals = (RaggedTotals *)(base + w.totals);
    uint32_t *hist = (uint32_t *)(base + w.hist);
    static_assert(sizeof(RaggedTotals) % 4 == 0, "cleared as 32-bit words");
    // the totals and the counts lie behind each other: one fill clears both
    const int64_t words = (int64_t)((w.hist - w.totals) / 4) + max_layers + 1;
    hipLaunchKernelGGL(ragged_clear_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream,
                       (int32_t *)totals, (int)words);
    hipLaunchKernelGGL(ragged_count_kernel, dim3((unsigned)((batch + kCountThreads - 1) / kCountThreads)),
                       dim3(kCountThreads), 0, stream, offsets_dev, batch, max_layers, hist, totals);
    hipLaunchKernelGGL(ragged_layout_kernel, dim3(1), dim3(kCountThreads), 0, stream, hist, max_layers,
                       (RaggedGroupDev *)(base + w.groups), (int64_t *)(base + w.tiles2), totals);
    if (hipGetLastError() != hipSuccess) return CKPT_ERR_DEVICE;
    // the call's one wait: the launches that follow are sized by the totals
    if (hipMemcpyAsync(&p.t, totals, sizeof(RaggedTotals), hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return CKPT_ERR_DEVICE;
    if (p.t.bad) return CKPT_ERR_SHAPE;
    return ragged_check_totals(p.t, batch);
}

int ragged_run(int which, const int64_t *d, const uint8_t *mask_in, const int64_t *offsets_host,
               const int64_t *offsets_dev, int64_t batch, int objective, uint8_t *mask_out, int64_t *peak_out,
               int64_t *budget_out, int64_t *timeline_out, int32_t *status_out, const RaggedPlan &p,
               const RaggedWorkspace &w, void *ws, hipStream_t stream)
{
    const bool eval = which == CKPT_CALL_EVAL_PEAK || which == CKPT_CALL_EVAL_TIMELINE;
    char *base = (char *)ws;
    const int64_t *off = offsets_dev ? offsets_dev : (const int64_t *)(base + w.off);
    int32_t *perm = (int32_t *)(base + w.perm);
    const RaggedGroupDev *groups = (const RaggedGroupDev *)(base + w.groups);
    const int64_t *tile_first2 = (const int64_t *)(base + w.tiles2);
    int32_t *cursor = (int32_t *)(base + w.cursor);
    int64_t *sd = (int64_t *)(base + w.d), *swide = (int64_t *)(base + w.wide);
    int64_t *speak = (int64_t *)(base + w.peak), *sbudget = (int64_t *)(base + w.budget);
    uint8_t *smask = (uint8_t *)(base + w.mask);
    int32_t *sstatus = (int32_t *)(base + w.status);
    const int n_groups = p.t.n_groups;
    if (!p.groups.empty()) {
        // The host made the plan.  The group table lives in host memory that ends with this call (and
        // the caller's offsets may end with it too): wait until the copies have read them.
        if (hipMemcpyAsync(base + w.groups, p.groups.data(), p.groups.size() * sizeof(RaggedGroupDev),
                           hipMemcpyHostToDevice, stream) != hipSuccess ||
            hipMemcpyAsync(base + w.tiles2, p.tile_first2.data(), p.tile_first2.size() * 8, hipMemcpyHostToDevice,
                           stream) != hipSuccess)
            return CKPT_ERR_DEVICE;
        if (!offsets_dev && hipMemcpyAsync(base + w.off, offsets_host, (size_t)(batch + 1) * 8,
                                           hipMemcpyHostToDevice, stream) != hipSuccess)
            return CKPT_ERR_DEVICE;
        if (hipStreamSynchronize(stream) != hipSuccess) return CKPT_ERR_DEVICE;
    }
    hipLaunchKernelGGL(ragged_clear_kernel, dim3((unsigned)((n_groups + 255) / 256)), dim3(256), 0, stream, cursor,
                       n_groups);
    hipLaunchKernelGGL(ragged_perm_kernel, dim3((unsigned)((batch + kPermThreads - 1) / kPermThreads)),
                       dim3(kPermThreads), 0, stream, off, batch, groups, n_groups, cursor, perm);
    // every group's chains into the position-major staging
    hipLaunchKernelGGL(ragged_gather_kernel<int64_t>, dim3((unsigned)p.t.tiles), dim3(kTileThreads), 0, stream, d, off, perm,
                       groups, tile_first2, n_groups, 1, sd);
    if (eval)
        hipLaunchKernelGGL(ragged_gather_kernel<uint8_t>, dim3((unsigned)p.t.tiles), dim3(kTileThreads), 0, stream, mask_in,
                           off, perm, groups, tile_first2, n_groups, 1, smask);
    hipError_t e = hipSuccess;
    if (which == CKPT_CALL_EVAL_PEAK) {
        e = launch_eval_peak_ragged(sd, smask, groups, n_groups, p.t.waves, batch, objective, speak, sstatus, stream);
    } else if (which == CKPT_CALL_SOLVE_LINEAR) {
        e = launch_solve_linear_ragged(sd, groups, n_groups, p.t.waves, batch, p.t.max_layers, smask, speak, sstatus,
                                       base + w.inner, stream);
    } else if (which == CKPT_CALL_EVAL_TIMELINE) {
        e = launch_eval_timeline_ragged(sd, smask, groups, n_groups, p.t.waves, objective, swide, sstatus, stream);
    } else {
        // the cubic solver takes the groups one after the other, each where it is staged (its tables
        // and launches are sized by the group's length)
        for (const RaggedGroupDev &g : p.groups) {
            e = launch_solve_cubic(sd + g.stage_off, g.count, g.n, Strides{1, g.pitch}, smask + g.stage_off,
                                   speak + g.first, sbudget + g.first, sstatus + g.first, false, nullptr, nullptr,
                                   nullptr, base + w.inner, stream);
            if (e != hipSuccess) return CKPT_ERR_DEVICE;
        }
    }
    if (e != hipSuccess) return CKPT_ERR_DEVICE;
    if (which == CKPT_CALL_EVAL_TIMELINE) {
        hipLaunchKernelGGL(ragged_scatter_kernel<int64_t>, dim3((unsigned)p.t.tiles2), dim3(kTileThreads), 0, stream, swide,
                           off, perm, groups, tile_first2, n_groups, 2, timeline_out);
    } else {
        if (!eval)
            hipLaunchKernelGGL(ragged_scatter_kernel<uint8_t>, dim3((unsigned)p.t.tiles), dim3(kTileThreads), 0, stream,
                               smask, off, perm, groups, tile_first2, n_groups, 1, mask_out);
        scatter_value(speak, perm, batch, peak_out, stream);
        if (which == CKPT_CALL_EVAL_PEAK && objective == CKPT_OBJ_BOTH)  // the dynamic peaks behind the static ones
            scatter_value(speak + batch, perm, batch, peak_out + batch, stream);
        if (which == CKPT_CALL_SOLVE_CUBIC) scatter_value(sbudget, perm, batch, budget_out, stream);
    }
    scatter_value(sstatus, perm, batch, status_out, stream);
    return hipGetLastError() == hipSuccess ? CKPT_OK : CKPT_ERR_DEVICE;
}

}  // namespace ckpt
