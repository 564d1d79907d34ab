// Checkpoint selection under Equation (cost) by the two-step scheme of
// Section 3.2 (Equation (T), Algorithm 4, Theorem 1).
//
// For a segment budget s let F_s(0) = d_0 and
//     F_s(j) = d_j + min{ F_s(h) : h < j, P[j-1] - P[h] <= s },   P[k] = d_0+..+d_k,
// i.e. F_s(j) = d_j + M(j-1,s) in the paper's notation; c_s = F_s(n) is the
// least checkpoint memory whose segments all fit in s (d_0, d_n forced), and
// the answer is min_s (s + c_s) over the budgets s = 0 and s = P[b] - P[a-1],
// 1 <= a <= b <= n-1.
//
// Kernels, all on the caller's stream, in this order (from 1024 layers on, links
// and slices share one launch: neither needs the other):
//   prologue  one wave per chain: validates the sizes, builds P by a wave scan,
//             divides everything by the largest common power of two and picks
//             32-bit arithmetic when sum(d)+max(d) then fits (it does for
//             aligned tensor sizes), else 64-bit.  Writes the table
//             pd[j] = (P[j-1], d_j).
//   32-bit chains:
//   links     the monotone stack of the sizes themselves: for every position
//             the nearest earlier smaller size, the stack depth, and a snapshot
//             of the stack's next eight entries; for every eight positions their
//             smallest size and depth and last prefix sum.
//   slices    the budget values laid out by slices of their value range (any
//             order inside a slice), so that the 64 lanes of a wave hold nearly
//             equal budgets and meet the same events at the same cells.
//   shared    one LANE per budget, all lanes walking j together.  F_s(j) is
//             d_j + m with m the value at the window's head; as long as a lane's
//             head stays, the part of Algorithm 4's queue that the lane builds
//             is the stack of the sizes (cut off at a lane-specific depth), the
//             same for every lane and every budget, so it is not stored at all.
//             A cell is one min and two compares against wave-uniform values,
//             and eight cells in which no lane's compare can pass are taken as
//             one such step on their summary;
//             only when a head leaves does the lane write that part of its queue
//             out to its ring in LDS (from the snapshot), and only such
//             written-out entries are ever dropped by value.  See the comment
//             at cubic_shared_kernel.  Waves whose 16-entry ring was too small
//             are listed and run again with 64 entries.
//   64-bit chains:
//   budgets   one LANE per budget, 64 budgets of equal range length and
//             consecutive start per wave, the queue kept per lane as a 16-entry
//             ring in LDS laid out [slot][lane], the entries at its two ends
//             mirrored in registers, keys stored as P[h] + s so that expiry is
//             one compare with P[j-1].  A value that finds the ring full is not
//             stored but remembered as a "hole" (smallest value, oldest and
//             newest key); holes vanish when a later value not above them
//             arrives or when they leave the window; the lane is exact unless
//             the head moves past the oldest live hole, and only then flagged.
//   both:
//   overflow  one WAVE per budget still flagged: F_s kept in LDS, the window
//             minimum taken by a wave reduction.  Any queue depth.
//   reduce    (long chains) folds the per-wave results.
//   epilogue  one wave per chain: lexicographic minimum of (s + c_s, s) over the
//             partial results (the smallest optimal budget value s*), then the
//             predecessors for s* (smallest minimal predecessor of every j) and
//             the walk back from n that writes the mask.

#include <limits>
#include <atomic>
#include <cstddef>

#include "ckpt_internal.h"

namespace ckpt {
namespace {

constexpr int64_t kInf = INT64_MAX;
constexpr int kCells = 8;  // cells per fetch of the (P, d) table
constexpr int kPad = 16;   // table entries past n+1, so a fetch never leaves the table
constexpr int kReduceBlocks = 64;      // second-level reduction: workgroups per chain
constexpr int64_t kReduceFrom = 4096;  // ... used when a chain has more per-wave partial results than this


struct ChainMeta {
    int32_t status;
    int32_t mode32;   // 1: normalised values fit 32-bit arithmetic
    int32_t shift;    // sizes were divided by 2^shift
    int32_t pad;
};

struct Partial {
    int64_t cost;     // s + c_s, normalised; kInf if none
    int64_t s;
};

template <typename V>
struct alignas(2 * sizeof(V)) PD {
    V P;  // P[j-1] (0 for j = 0)
    V d;  // d_j
};

// What cell j = t+1 of a 32-bit chain consumes about position t, and the links
// of the monotone stack of sizes: below(t) is the nearest earlier position with
// a strictly smaller size (-1: none), depth(t) the length of the chain
// t, below(t), below(below(t)), ...  That chain is the set of positions h <= t
// with d_h < d_h' for every h' in (h, t]: what a monotone queue of the values
// d_h + const would hold after position t.
constexpr int kSnap = 8;  // chain elements per snapshot
struct alignas(16) El {
    int32_t P;      // P[t]
    int32_t d;      // d_t
    int32_t below;  // the chain element kSnap places below t, the snapshot's last (-1: the chain is shorter)
    int32_t depth;
};
// What every cell reads about its position
struct alignas(8) Step {
    int32_t d;      // d_t
    int32_t under;  // depth(t) - 1: the depth the size stack drops to before t goes on it
};
// What a wave reads about kGroup consecutive positions g*kGroup .. g*kGroup + kGroup - 1 before it
// looks at any of them: if no lane's top entry is reached by the smallest size and no lane's
// head is left behind by the last prefix sum, nothing happens in the whole group.
constexpr int kGroup = 8;
struct alignas(16) Group {
    int32_t dmin;   // smallest d_t of the group
    int32_t pend;   // P[t] of its last position
    int32_t umin;   // smallest depth(t) - 1
    int32_t pair;   // for the pair of groups in slots (2k, 2k+1): in the first the smaller of the two dmin,
                    // in the second the smaller of the two umin
};
// (P[h], d_h) of the kSnap elements of t's chain that follow t itself; zeros past its end
struct alignas(64) Snap {
    PD<int32_t> e[kSnap];
};

struct CubicWs {
    ChainMeta *meta;      // [batch]
    char *pd;             // [batch][table_len(n)] of PD<int64_t> (PD<int32_t> in the same bytes when mode32)
    El *el;               // [batch][table_len(n)], 32-bit chains only
    Snap *snap;           // [batch][table_len(n)], 32-bit chains only
    Step *step;           // [batch][step_len(n)], 32-bit chains only
    Group *group;         // [batch][group_len(n)], 32-bit chains only
    int32_t *sorted;      // [batch][K] the budget values, slice after slice: lane i of wave w takes sorted[w*64 + i]
    int32_t *redo_count;  // number of waves whose ring was too small ...
    int64_t *redo;        // [batch * waves_per_chain] ... and their slots, for a second run with a larger ring
    int64_t *trace_s;     // [batch][waves_per_chain][64] or null: every lane's budget in bytes (-1: lane past the list) ...
    int64_t *trace_cost;  // ... and its cost s + c_s in bytes (Equation (T)); set by ckpt_solve_cubic_costs only
    Partial *partial;     // [batch][waves_per_chain]
    uint64_t *flags;      // [batch][waves_per_chain] lanes to recompute
    Partial *partial2;    // [batch][kReduceBlocks] second-level partial results (long chains only)
    int32_t *pred;        // [batch][n+1]
    int32_t *prune;       // [batch] budgets above this (normalised) value cannot be optimal; pruned calls only
    int32_t *prune_lo;    // [batch] ... nor budgets below this one
    int32_t *skip_sample; // [batch] 1: the first bounds leave so few budgets that no sample is run first
    int32_t *wsum;        // [batch][n+1] wsum[m] = sum of the m smallest interior sizes; pruned calls only
    unsigned long long *evaluated;  // [batch] budgets whose recurrence was run; pruned calls only
};

__host__ __device__ inline int64_t num_budgets(int n) { return (int64_t)n * (n - 1) / 2 + 1; }
__host__ __device__ inline int64_t waves_per_chain(int n) { return (num_budgets(n) + kWave - 1) / kWave; }
__host__ __device__ inline size_t table_len(int n) { return ((size_t)n + 1 + kPad + kCells - 1) / kCells * kCells; }

__host__ __device__ inline size_t step_len(int n) { return table_len(n) + 32; }  // read up to two blocks of 16 past n
// Group g sits in slot g + 1, so that the pair of groups (1, 2), where the loop starts, and every
// pair after it is 32-byte aligned; the loop reads up to three pairs past the last group it uses.
__host__ __device__ inline size_t group_slot(int g) { return (size_t)g + 1; }
__host__ __device__ inline size_t group_len(int n) { return (table_len(n) / kGroup + 10) / 2 * 2; }

template <typename V>
__device__ inline const PD<V> *chain_table(const CubicWs &w, int64_t c, int n)
{
    return (const PD<V> *)(w.pd + (size_t)c * table_len(n) * sizeof(PD<int64_t>));
}

// ---- ordering the budget values --------------------------------------------------
//
// Lanes of a wave that hold nearly equal budgets see the same head leave at the same cell, so the
// rare part of a cell runs once for all of them.  That needs no total order, only that the 64
// budgets of a wave lie close together: the budgets of a 32-bit chain are laid out by slices of
// the value range, slices in ascending order, any order inside a slice.  A slice is 2^w wide, w
// chosen so that a slice holds 32 to 128 budgets on average: narrower than most layer sizes, so
// the lanes of a wave nearly always agree on which prefix sum their head's key lies behind.
// The budgets are the differences Q[x] - Q[a] of the prefix sums Q (1 <= a < x <= n) and 0, so
// for a fixed start a they ascend with x: the budgets of a below a bound are found by bisection.
// One workgroup lays out a group of kSliceGroup consecutive slices: the number of budgets below
// the group's lower bound (a sum over the starts) is where the group begins in the list; the
// budgets of each start inside the group's range are counted per slice in LDS, the counts scanned,
// and the budgets written to their slices' places.  No pass over the whole list, no global counters.
constexpr int kSliceGroup = 256;     // slices per workgroup
__host__ __device__ inline int slices_log2(int n)
{
    const int64_t K = num_budgets(n);
    int b = 0;
    while (b < 20 && ((int64_t)64 << b) <= K) ++b;
    return b;
}
// log2 of the slice width for a chain whose largest budget is smax: at most 2^slices_log2(n) slices.
__device__ inline int slice_shift(int32_t smax, int n)
{
    const int bits = 32 - __clz(smax | 1);  // smax < 2^bits
    const int sh = bits - slices_log2(n);
    return sh > 0 ? sh : 0;
}
// Workgroups per chain: enough groups for the most slices a chain of n layers can have.
__host__ __device__ inline int64_t slice_groups(int n)
{
    return (((int64_t)1 << slices_log2(n)) + kSliceGroup - 1) / kSliceGroup;
}

__host__ CubicWs carve_cubic(void *ws, int64_t batch, int n)
{
    char *p = (char *)ws;
    const size_t n1 = (size_t)n + 1, B = (size_t)batch, wpc = (size_t)waves_per_chain(n);
    CubicWs w;
    w.meta = (ChainMeta *)p;    p += align_up(B * sizeof(ChainMeta));
    w.pd = p;                   p += align_up(B * table_len(n) * sizeof(PD<int64_t>));
    w.el = (El *)p;             p += align_up(B * table_len(n) * sizeof(El));
    w.snap = (Snap *)p;         p += align_up(B * table_len(n) * sizeof(Snap));
    w.step = (Step *)p;         p += align_up(B * step_len(n) * sizeof(Step));
    w.group = (Group *)p;       p += align_up(B * group_len(n) * sizeof(Group));
    w.sorted = (int32_t *)p;    p += align_up(B * (size_t)num_budgets(n) * 4);
    w.redo_count = (int32_t *)p; p += 256;
    w.redo = (int64_t *)p;      p += align_up(B * wpc * 8);
    w.trace_s = nullptr;
    w.trace_cost = nullptr;
    w.partial = (Partial *)p;   p += align_up(B * wpc * sizeof(Partial));
    w.flags = (uint64_t *)p;    p += align_up(B * wpc * 8);
    w.partial2 = (Partial *)p;  p += align_up(B * kReduceBlocks * sizeof(Partial));
    w.pred = (int32_t *)p;      p += align_up(B * n1 * 4);
    w.prune = (int32_t *)p;     p += align_up(B * 4);
    w.prune_lo = (int32_t *)p;  p += align_up(B * 4);
    w.skip_sample = (int32_t *)p; p += align_up(B * 4);
    w.wsum = (int32_t *)p;      p += align_up(B * n1 * 4);
    w.evaluated = (unsigned long long *)p; p += align_up(B * 8);
    return w;
}

// ---- wave helpers -----------------------------------------------------------

__device__ inline int64_t shfl_i64(int64_t v, int src) { return __shfl(v, src, kWave); }
__device__ inline int64_t shfl_xor_i64(int64_t v, int m) { return __shfl_xor(v, m, kWave); }
__device__ inline int64_t shfl_up_i64(int64_t v, int d) { return __shfl_up(v, d, kWave); }

// Lexicographic minimum of (a, b) over the wave; every lane gets the result.  Both values are
// non-negative wherever this is used (costs, budgets, indices, kInf), so they order as unsigned:
// the smallest a, then the smallest b among the lanes that hold it.
__device__ inline void wave_min_pair(int64_t &a, int64_t &b)
{
    const uint64_t am = wave_min_u64((uint64_t)a);
    const uint64_t bm = wave_min_u64((uint64_t)a == am ? (uint64_t)b : ~0ull);
    a = (int64_t)am;
    b = (int64_t)bm;
}

// ---- prologue ---------------------------------------------------------------

__global__ __launch_bounds__(kWave) void cubic_prologue_kernel(const int64_t *__restrict__ d, int64_t batch,
                                                               int n, int64_t cstride, int64_t pstride,
                                                               CubicWs w)
{
    const int64_t c = blockIdx.x;
    const int lane = threadIdx.x;
    if (c == 0 && lane == 0) *w.redo_count = 0;
    if (lane == 0) {
        w.prune[c] = INT32_MAX;
        w.skip_sample[c] = 0;
        w.prune_lo[c] = 0;
        w.evaluated[c] = 0;
    }
    const int64_t *dp = d + c * cstride;
    const int n1 = n + 1;
    const int chunk = (n1 + kWave - 1) / kWave;
    const int k0 = lane * chunk;
    const int k1 = min(k0 + chunk, n1);

    uint64_t sum = 0, bits = 0;
    int64_t mx = 0;
    bool bad = false, ovf = false;
    // (eight loads in flight per lane; positions past the lane's part repeat its last one and are not used)
    constexpr int kAhead = 8;
    for (int kb = k0; kb < k1; kb += kAhead) {
        int64_t xs[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) xs[u] = dp[(int64_t)min(kb + u, k1 - 1) * pstride];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            if (kb + u < k1) {
                const int64_t x = xs[u];
                bad |= x <= 0;
                bits |= (uint64_t)x;
                mx = x > mx ? x : mx;
                sum += (uint64_t)x;
                ovf |= sum > (uint64_t)INT64_MAX;
            }
        }
    }
    // inclusive scan of the lane sums (all terms positive: any wrap shows as > INT64_MAX first)
    uint64_t incl = sum;
#pragma unroll
    for (int dlt = 1; dlt < kWave; dlt <<= 1) {
        const uint64_t o = (uint64_t)shfl_up_i64((int64_t)incl, dlt);
        const bool oo = __shfl_up((int)ovf, dlt, kWave);
        if (lane >= dlt) {
            incl += o;
            ovf |= oo | (incl > (uint64_t)INT64_MAX);
        }
    }
    const uint64_t total = (uint64_t)shfl_i64((int64_t)incl, kWave - 1);
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) {
        bits |= (uint64_t)shfl_xor_i64((int64_t)bits, m);
        const int64_t om = shfl_xor_i64(mx, m);
        mx = om > mx ? om : mx;
    }
    const bool any_bad = __any(bad);
    bool any_ovf = __any(ovf);
    any_ovf |= (total + (uint64_t)mx) > (uint64_t)INT64_MAX;

    ChainMeta meta;
    meta.status = any_bad ? CKPT_ERR_SIZE : (any_ovf ? CKPT_ERR_OVERFLOW : CKPT_OK);
    meta.shift = 0;
    meta.mode32 = 0;
    meta.pad = 0;
    if (meta.status == CKPT_OK) {
        meta.shift = __ffsll((unsigned long long)bits) - 1;
        meta.mode32 = ((total + (uint64_t)mx) >> meta.shift) < (1ull << 30);
    }
    if (lane == 0) w.meta[c] = meta;
    if (meta.status != CKPT_OK) return;

    // pd[j] = (P[j-1], d_j): lane chunks write their own j; the padding is zeroed
    uint64_t run = incl - sum;  // P[k0-1]
    PD<int64_t> *pd64 = (PD<int64_t> *)chain_table<int64_t>(w, c, n);
    PD<int32_t> *pd32 = (PD<int32_t> *)pd64;
    for (int kb = k0; kb < k1; kb += kAhead) {
        uint64_t xs[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) xs[u] = (uint64_t)dp[(int64_t)min(kb + u, k1 - 1) * pstride];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int k = kb + u;
            if (k < k1) {
                if (meta.mode32)
                    pd32[k] = PD<int32_t>{(int32_t)(run >> meta.shift), (int32_t)(xs[u] >> meta.shift)};
                else
                    pd64[k] = PD<int64_t>{(int64_t)(run >> meta.shift), (int64_t)(xs[u] >> meta.shift)};
                run += xs[u];
            }
        }
    }
    const int len = (int)table_len(n);
    for (int k = n1 + lane; k < len; k += kWave) {
        const uint64_t last = k == n1 ? total : 0;  // pd[n+1].P = P[n]
        if (meta.mode32)
            pd32[k] = PD<int32_t>{(int32_t)(last >> meta.shift), 0};
        else
            pd64[k] = PD<int64_t>{(int64_t)(last >> meta.shift), 0};
    }
}

// ---- links of the monotone stack of sizes (32-bit chains) ---------------------------

extern __shared__ __align__(16) unsigned char dyn_lds[];

constexpr int kLinksBlock = 1024;

__host__ __device__ constexpr size_t links_lds_bytes(int n) { return ((size_t)n + 2) * 10 + 16; }

// One workgroup per chain.  below(t) comes from a backward search per position (its own block
// of 64 positions, then the blocks' minima, then the block that answers); depth(t) from below(t)
// by pointer jumping; then every position's snapshot.  LDS: 10 bytes per position.
template <int THREADS>
__device__ inline void links_chain(int n, const CubicWs &w, int64_t c)
{
    const ChainMeta meta = w.meta[c];
    if (meta.status != CKPT_OK || !meta.mode32) return;
    const int tid = threadIdx.x;
    const int n1 = n + 1;
    const PD<int32_t> *__restrict__ pd = chain_table<int32_t>(w, c, n);
    El *__restrict__ el = w.el + (size_t)c * table_len(n);
    Snap *__restrict__ snap = w.snap + (size_t)c * table_len(n);

    // link[t] = (jump << 16) | dist: jump is a position further down t's chain (n1: past its
    // end), dist the number of chain elements from t (inclusive) to jump (exclusive)
    uint32_t *link = (uint32_t *)dyn_lds;              // [n1 + 1]
    int32_t *dl = (int32_t *)(link + n1 + 1);          // [n1] the sizes
    uint16_t *stk = (uint16_t *)(dl + n1);             // [n1 + 1] below(t)
    constexpr int kBlk = 64;                            // positions per block of the search below
    constexpr int kMaxBlks = (CKPT_CUBIC_MAX_LAYERS + 1 + kBlk - 1) / kBlk;
    __shared__ int32_t blk_min[kMaxBlks];               // smallest size of each block
    __shared__ int32_t blks_min[kMaxBlks];              // ... of blocks 0..b
    const uint32_t kEnd = (uint32_t)n1;

    for (int t = tid; t < n1; t += THREADS) dl[t] = pd[t].d;
    __syncthreads();
    const int nblk = (n1 + kBlk - 1) / kBlk;
    for (int q = tid; q < nblk; q += THREADS) {
        int32_t low = INT32_MAX;
        const int t1 = min((q + 1) * kBlk, n1);
        for (int t = q * kBlk; t < t1; ++t) low = min(low, dl[t]);
        blk_min[q] = low;
    }
    __syncthreads();
    if (tid == 0) {
        int32_t run = INT32_MAX;
        for (int q = 0; q < nblk; ++q) {
            run = min(run, blk_min[q]);
            blks_min[q] = run;
        }
        link[n1] = kEnd << 16;
    }
    __syncthreads();
    // below(t), every position on its own: backwards through its block; if nothing smaller is
    // there, backwards over the blocks' minima to the nearest block that holds something smaller
    // (none if even the minimum of all earlier blocks is not), then backwards through that block.
    // The nearest smaller size is a few positions away for most positions of most chains; the
    // worst case is two blocks' lengths plus the number of blocks.
    static_assert(kBlk == kWave && THREADS % kWave == 0, "a wave holds one block");
    const int lane = tid & (kWave - 1);
    for (int t0 = tid - lane; t0 < n1; t0 += THREADS) {  // the same trip count for the whole wave
        const int t = t0 + lane;
        const int32_t x = t < n1 ? dl[t] : INT32_MAX;
        // inside the block the sizes are the wave's own registers: the nearest lower lane with a
        // smaller size (ascending j, so the last hit stays)
        int near = -1;
        for (int j = 0; j < kWave - 1; ++j) {
            const int32_t v = __builtin_amdgcn_readlane(x, j);
            near = (j < lane && v < x) ? j : near;
        }
        if (t >= n1) continue;
        uint32_t found = kEnd;
        if (near >= 0) {
            found = (uint32_t)(t0 + near);
        } else {
            int q = t0 / kBlk - 1;
            if (q >= 0 && blks_min[q] < x) {
                while (blk_min[q] >= x) --q;  // stops: some block up to q holds a smaller size
                int h = (q + 1) * kBlk - 1;   // (q is not the last block: it is a full one)
                while (dl[h] >= x) --h;       // stops inside block q
                found = (uint32_t)h;
            }
        }
        link[t] = (found << 16) | 1u;
    }
    __syncthreads();
    // below(t) on its own, as 16-bit positions
    for (int t = tid; t <= n1; t += THREADS) stk[t] = (uint16_t)(link[t] >> 16);  // link[n1] points at itself
    uint16_t *below = stk;
    __syncthreads();

    // depth by pointer jumping, in place: every update keeps "dist = elements from t to jump"
    // (a word is read and written whole, so any mix of old and new words is consistent)
    for (;;) {
        int moved = 0;
        for (int t = tid; t < n1; t += THREADS) {
            const uint32_t a = link[t];
            if ((a >> 16) == kEnd) continue;
            const uint32_t b = link[a >> 16];
            link[t] = (b & 0xffff0000u) | ((a & 0xffffu) + (b & 0xffffu));
            moved = 1;
        }
        if (!__syncthreads_or(moved)) break;
    }

    for (int t = tid; t < (int)table_len(n); t += THREADS) {
        El e;
        Snap sn;
        if (t < n1) {
            uint32_t h = (uint32_t)t;
#pragma unroll
            for (int k = 0; k < kSnap; ++k) {
                h = below[h];  // below[kEnd] is kEnd
                const bool in = h != kEnd;
                sn.e[k].P = in ? pd[h + 1].P : 0;
                sn.e[k].d = in ? dl[h] : 0;
            }
            e.P = pd[t + 1].P;
            e.d = dl[t];
            e.below = h == kEnd ? -1 : (int32_t)h;
            e.depth = (int32_t)(link[t] & 0xffffu);
        } else {
#pragma unroll
            for (int k = 0; k < kSnap; ++k) sn.e[k] = PD<int32_t>{0, 0};
            e.P = pd[n1].P; e.d = 0; e.below = -1; e.depth = 1;
        }
        el[t] = e;
        snap[t] = sn;
    }
    Step *__restrict__ st = w.step + (size_t)c * step_len(n);
    for (int t = tid; t < (int)step_len(n); t += THREADS)
        st[t] = t < n1 ? Step{dl[t], (int32_t)(link[t] & 0xffffu) - 1} : Step{0, 0};
    // the groups' summaries; a group that reaches past n is never used as one
    Group *__restrict__ gr = w.group + (size_t)c * group_len(n);
    auto summary = [&](const int slot) -> Group {
        Group G{std::numeric_limits<int32_t>::max(), 0, std::numeric_limits<int32_t>::max(), 0};
        const int g = slot - 1;
        const int t_last = g * kGroup + kGroup - 1;
        if (g >= 0 && t_last < n1) {
            for (int t = g * kGroup; t <= t_last; ++t) {
                G.dmin = min(G.dmin, dl[t]);
                G.umin = min(G.umin, (int32_t)(link[t] & 0xffffu) - 1);
            }
            G.pend = pd[t_last + 1].P;
        }
        return G;
    };
    for (int slot = tid; slot < (int)group_len(n); slot += THREADS) {  // group_len is even
        Group G = summary(slot);
        const Group other = summary(slot ^ 1);
        G.pair = (slot & 1) == 0 ? min(G.dmin, other.dmin) : min(G.umin, other.umin);
        gr[slot] = G;
    }
}

// (short chains: a smaller workgroup, most of a large one would sit idle at the barriers)
constexpr int kLinksShortBlock = 256;
__global__ __launch_bounds__(kLinksShortBlock) void cubic_links_kernel(int n, CubicWs w)
{
    links_chain<kLinksShortBlock>(n, w, blockIdx.x);
}

// ---- budget index -> (range length, start) ------------------------------------

// Budget 0 is s = 0.  Budget t+1, 0 <= t < m(m+1)/2 with m = n-1, is the range of
// length len starting at a, ranges ordered by length, then start.  Counting t
// from the far end turns the rows of sizes m, m-1, .., 1 into rows of sizes
// 1, 2, .., m whose starts are the triangular numbers.
__device__ inline void budget_range(int64_t idx, int n, int &a, int &len)
{
    const int64_t m = n - 1;
    const int64_t tri = m * (m + 1) / 2;
    const int64_t tr = tri - 1 - (idx - 1);
    int64_t r = (int64_t)((1.0 + sqrt(1.0 + 8.0 * (double)tr)) * 0.5);
    while (r * (r - 1) / 2 > tr) --r;
    while (r * (r + 1) / 2 <= tr) ++r;
    const int64_t off = tr - r * (r - 1) / 2;  // 0 .. r-1 from the far end of the row
    len = (int)(m - r + 1);
    a = (int)(r - off);
}

template <typename V>
__device__ inline V budget_value(const PD<V> *__restrict__ pd, int64_t idx, int n)
{
    if (idx == 0) return 0;
    int a, len;
    budget_range(idx, n, a, len);
    return pd[a + len].P - pd[a].P;  // P[a+len-1] - P[a-1]
}

// ---- budgets kernel: one lane per budget -----------------------------------------

template <typename V>
struct alignas(2 * sizeof(V)) QueueEntry {
    V F;  // F_s(h)
    V K;  // P[h] + s: the entry leaves the window once this is below P[j-1]
};

// RING slots per lane, BLOCK lanes per workgroup: RING * BLOCK * sizeof(QueueEntry) bytes of LDS.
constexpr int64_t kBudgetBlocksPerChain = 4096;

template <typename V, int RING, int BLOCK>
__global__ __launch_bounds__(BLOCK) void cubic_budgets_kernel(int n, int64_t blocks_per_chain, CubicWs w)
{
    __shared__ __attribute__((aligned(65536))) QueueEntry<V> ring[RING][BLOCK];
    constexpr V kLow = std::numeric_limits<V>::min();
    constexpr V kHigh = std::numeric_limits<V>::max();
    // Queue positions are kept pre-multiplied by the byte stride of a ring slot,
    // so the LDS address of a position is one AND-OR away.
    constexpr uint32_t kStep = (uint32_t)(BLOCK * sizeof(QueueEntry<V>));
    constexpr uint32_t kSlotMask = (uint32_t)(RING - 1) * kStep;
    constexpr uint32_t kFull = (uint32_t)(RING - 1) * kStep;  // tl - hd at RING entries
    static_assert((kStep & (kStep - 1)) == 0 && (RING & (RING - 1)) == 0, "power-of-two ring");

    // A chain has at most kBudgetBlocksPerChain workgroups, each taking every so-many-th tile of
    // its budgets: a chain that is not this kernel's costs a handful of workgroups, not one per tile.
    const int64_t per_chain = blocks_per_chain < kBudgetBlocksPerChain ? blocks_per_chain : kBudgetBlocksPerChain;
    const int64_t c = blockIdx.x / per_chain;
    const ChainMeta meta = w.meta[c];
    if (meta.status != CKPT_OK || (meta.mode32 != 0) != (sizeof(V) == 4)) return;
    for (int64_t tile = blockIdx.x % per_chain; tile < blocks_per_chain; tile += per_chain) {

    const int tid = threadIdx.x;
    const PD<V> *__restrict__ pd = chain_table<V>(w, c, n);
    const int64_t K = num_budgets(n);
    const int64_t idx = tile * BLOCK + tid;
    const int64_t wave_in_chain = idx / kWave;   // uniform per wave
    if (wave_in_chain * kWave >= K) continue;    // whole wave beyond the list
    const bool live = idx < K;
    // lanes past the list take the largest budget (all interior layers), the one with the least to do
    const V s = live ? budget_value<V>(pd, idx, n) : (V)(pd[n].P - pd[1].P);

    // LDS byte address of this lane's slot 0 (the ring is aligned to its own size,
    // so a position's address is (pos & kSlotMask) | lane_base)
    typedef __attribute__((address_space(3))) V *LdsPtr;  // [0] = F, [1] = K of an entry
    const uint32_t lane_base = (uint32_t)(uintptr_t)(LdsPtr)&ring[0][tid].F;
    auto slot = [&](uint32_t pos) -> LdsPtr { return (LdsPtr)(uintptr_t)((pos & kSlotMask) | lane_base); };
    auto store_entry = [&](uint32_t pos, V F, V key) {
        LdsPtr e = slot(pos);
        e[0] = F;
        e[1] = key;
    };

    // The queue occupies positions hd..tl; the head entry and the tail value are
    // mirrored in registers.  It starts as {h = 0}.
    uint32_t hd = 0, tl = 0;
    V hF = pd[0].d, hK = pd[1].P + s, tF = hF;
    store_entry(0, hF, hK);
    V holeF = kLow, holeOld = kHigh, holeNew = kLow;  // no hole
    uint64_t hole_lanes = 0;                          // lanes with a live hole (wave-uniform)
    bool over = false;
    V Fprev = pd[1].d + hF;  // F(1) = d_1 + F(0)

    // One cell: insert h = j-1 (value Fprev, key Pj1 + s), expire, F(j) = d_j + head.
    // The two queue loops run while ANY lane of the wave still has work; lanes
    // that are done sit out under the exec mask.
    //  - tails not smaller than the new value are dropped.  The head is smaller
    //    than F(j-1) = d_{j-1} + head, and tF = hF when one entry is left, so
    //    the head always stays.
    //  - heads whose segment h+1..j-1 no longer fits in s are dropped.  When the
    //    new value has been stored that loop stops at it at the latest (it fits).
    //  - when some lane's ring is full or has a live hole the whole wave takes
    //    the slow path, which is the same cell with the hole bookkeeping.
    // The values of the two entries under the tail and the entry after the head are mirrored in
    // registers as well (read back at the end of every cell, when nothing waits for them), so that
    // the usual one to three drops and the usual single expiry are decided without a trip to LDS.
    // What the mirrors hold beyond the head is never looked at: the head's value is below every
    // new value, so the nested tests stop at it at the latest.
    V t1F = kLow, t2F = kLow, h1F = kLow, h1K = kLow;
    auto cell_generic = [&](const V Pj1, const V dj) {
        const bool p0 = tF >= Fprev;
        const bool p1 = p0 & (t1F >= Fprev);
        const bool p2 = p1 & (t2F >= Fprev);
        tl -= (p0 ? kStep : 0u) + (p1 ? kStep : 0u) + (p2 ? kStep : 0u);
        tF = p1 ? t2F : (p0 ? t1F : tF);  // the value now at the tail (p2: read below)
        if (__builtin_amdgcn_ballot_w64(p2) != 0) {
            if (p2) tF = slot(tl)[0];
            for (;;) {
                const bool more = p2 & (tF >= Fprev);
                if (__builtin_amdgcn_ballot_w64(more) == 0) break;
                if (more) {
                    tl -= kStep;
                    tF = slot(tl)[0];
                }
            }
        }
        const V key = Pj1 + s;
        const bool full = (tl - hd) >= kFull;
        if ((__builtin_amdgcn_ballot_w64(full) | hole_lanes) != 0) {
            // holes vanish when this value would have dropped them, or when they left the window
            const bool gone = (Fprev <= holeF) | (holeNew < Pj1);
            holeF = gone ? kLow : holeF;
            holeOld = gone ? kHigh : holeOld;
            holeNew = gone ? kLow : holeNew;
            if (full) {  // not stored: becomes a hole
                holeF = holeOld == kHigh ? Fprev : holeF;
                holeOld = key < holeOld ? key : holeOld;
                holeNew = key;
            }
        }
        if (!full) {
            tl += kStep;
            store_entry(tl, Fprev, key);
            tF = Fprev;
            const bool second = tl == hd + kStep;  // the new entry is the one after the head
            h1F = second ? Fprev : h1F;
            h1K = second ? key : h1K;
        }
        const bool e0 = (hK < Pj1) & (hd != tl);
        if (__builtin_amdgcn_ballot_w64(e0) != 0) {
            if (e0) {
                hd += kStep;
                hF = h1F;
                hK = h1K;
            }
            for (;;) {
                const bool more = e0 & (hK < Pj1) & (hd != tl);
                if (__builtin_amdgcn_ballot_w64(more) == 0) break;
                if (more) {
                    hd += kStep;
                    hF = slot(hd)[0];
                    hK = slot(hd)[1];
                }
            }
        }
        over |= (hK < Pj1) | (hK > holeOld);  // nothing valid left, or the head passed a hole
        hole_lanes = __builtin_amdgcn_ballot_w64(holeOld != kHigh);
        Fprev = dj + hF;
        {
            LdsPtr a1 = slot(tl - kStep), a2 = slot(tl - 2 * kStep), b1 = slot(hd + kStep);
            t1F = a1[0];
            t2F = a2[0];
            h1F = b1[0];
            h1K = b1[1];
        }
    };

    auto cell = [&](const V Pj1, const V dj) { cell_generic(Pj1, dj); };

    // pd[j] is fetched kCells cells ahead of its use
    PD<V> cur[kCells], ahead[kCells];
#pragma unroll
    for (int u = 0; u < kCells; ++u) cur[u] = pd[u];
    auto chunk = [&](const int j0, const bool guarded) {
#pragma unroll
        for (int u = 0; u < kCells; ++u) ahead[u] = pd[j0 + kCells + u];
#pragma unroll
        for (int u = 0; u < kCells; ++u) {
            const int j = j0 + u;
            if (!guarded || (j >= 2 && j <= n)) cell(cur[u].P, cur[u].d);
        }
#pragma unroll
        for (int u = 0; u < kCells; ++u) cur[u] = ahead[u];
    };
    const int last_full = (n + 1) / kCells * kCells;  // chunks [kCells, last_full) lie inside 2..n
    chunk(0, true);
    for (int j0 = kCells; j0 < last_full; j0 += kCells) chunk(j0, false);
    if (last_full >= kCells && last_full <= n) chunk(last_full, true);

    const bool redo = live && over;
    const uint64_t flag = __ballot(redo);
    int64_t cost = (live && !over) ? (int64_t)s + (int64_t)Fprev : kInf;
    int64_t sv = (int64_t)s;
    if (w.trace_s) {  // (a flagged lane's cost is written when it is computed again)
        const int64_t at = (c * waves_per_chain(n) + wave_in_chain) * kWave + (tid & (kWave - 1));
        const int shift = w.meta[c].shift;
        w.trace_s[at] = live ? (int64_t)((uint64_t)sv << shift) : -1;
        w.trace_cost[at] = (live && !over) ? (int64_t)((uint64_t)cost << shift) : -1;
    }
    wave_min_pair(cost, sv);
    if ((tid & (kWave - 1)) == 0) {
        const int64_t slot_id = c * waves_per_chain(n) + wave_in_chain;
        w.partial[slot_id] = Partial{cost, sv};
        w.flags[slot_id] = flag;
    }
    }
}

template <typename V, int RING, int BLOCK>
void launch_budgets(int n, int64_t batch, CubicWs w, hipStream_t stream)
{
    const int64_t blocks_per_chain = (num_budgets(n) + BLOCK - 1) / BLOCK;
    const int64_t per_chain = blocks_per_chain < kBudgetBlocksPerChain ? blocks_per_chain : kBudgetBlocksPerChain;
    hipLaunchKernelGGL((cubic_budgets_kernel<V, RING, BLOCK>), dim3((unsigned)(per_chain * batch)),
                       dim3(BLOCK), 0, stream, n, blocks_per_chain, w);
}

// ---- budget values of the 32-bit chains, laid out by slices of the value range -----------------
extern __shared__ __align__(16) unsigned char order_lds[];

// kBisect: starts whose bisections a thread runs side by side

// For kBisect starts a[j] at once: x[j] = the largest x in [a[j], n] with Q[x] - Q[a[j]] < bound
// (Q ascending; bound >= 1).  The reads of the kBisect searches are independent of each other,
// so their LDS latencies overlap.  A start a >= n gets x = a.
template <int kBisect>
__device__ inline void ends_below(const int32_t *Q, int n, const int (&a)[kBisect], int64_t bound, int (&x)[kBisect])
{
    int lo[kBisect], hi[kBisect];
#pragma unroll
    for (int j = 0; j < kBisect; ++j) {
        lo[j] = a[j];
        hi[j] = a[j] < n ? n : a[j];
    }
    for (int span = n; span > 0; span >>= 1) {  // hi - lo at most halves (rounded down) each turn
        int32_t q[kBisect];
        int mid[kBisect];
#pragma unroll
        for (int j = 0; j < kBisect; ++j) {
            mid[j] = (lo[j] + hi[j] + 1) >> 1;
            q[j] = Q[mid[j] <= n ? mid[j] : n];
        }
#pragma unroll
        for (int j = 0; j < kBisect; ++j) {
            if (lo[j] < hi[j]) {
                const int32_t qa = Q[a[j] <= n ? a[j] : n];
                if ((int64_t)q[j] - qa < bound) lo[j] = mid[j]; else hi[j] = mid[j] - 1;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kBisect; ++j) x[j] = lo[j];
}

// One workgroup of THREADS threads per group of kSliceGroup slices of a chain.  A long chain has
// few groups (256 at n = 4096, one per CU): with 1024 threads a CU holds four waves per SIMD, whose
// bisections and scattered stores hide each other's latency; a short chain has fewer starts than
// that many threads could take.
template <int THREADS, int kBisect>
__device__ inline void slice_group(int n, const CubicWs &w, int64_t block)
{
    __shared__ int32_t tally[kSliceGroup];   // budgets per slice, then each slice's next free place
    __shared__ int32_t below;                // budgets below the group's range
    const int64_t groups = slice_groups(n);
    const int64_t c = block / groups;
    const int64_t g = block % groups;
    const ChainMeta meta = w.meta[c];
    if (meta.status != CKPT_OK || !meta.mode32) return;
    const PD<int32_t> *pd = chain_table<int32_t>(w, c, n);
    int32_t *Q = (int32_t *)order_lds;  // Q[j] = P[j-1], j = 0..n
    const int tid = threadIdx.x;
    const int32_t smax = pd[n].P - pd[1].P;   // the largest budget: every interior layer
    const int wshift = slice_shift(smax, n);
    const int64_t lo = (g * kSliceGroup) << wshift, hi = ((g + 1) * kSliceGroup) << wshift;  // lo <= s < hi
    if (lo > smax) return;                   // (the same for the whole workgroup)
    for (int j = tid; j <= n; j += THREADS) Q[j] = pd[j].P;
    for (int k = tid; k < kSliceGroup; k += THREADS) tally[k] = 0;
    if (tid == 0) below = lo > 0 ? 1 : 0;    // the empty range, s = 0
    __syncthreads();
    int32_t *out = w.sorted + c * num_budgets(n);

    // pass 1: the ends of every start's budgets inside the range; counts
    int32_t mine_below = 0;
    for (int a0 = 1 + tid; a0 < n; a0 += THREADS * kBisect) {
        int a[kBisect], x0[kBisect], x1[kBisect];
#pragma unroll
        for (int j = 0; j < kBisect; ++j) a[j] = a0 + THREADS * j;
        if (lo > 0) {
            ends_below<kBisect>(Q, n, a, lo, x0);
        } else {
#pragma unroll
            for (int j = 0; j < kBisect; ++j) x0[j] = a[j];
        }
        ends_below<kBisect>(Q, n, a, hi, x1);
#pragma unroll
        for (int j = 0; j < kBisect; ++j) {
            if (a[j] < n) {
                mine_below += x0[j] - a[j];
                const int32_t qa = Q[a[j]];
                for (int x = x0[j] + 1; x <= x1[j]; ++x)
                    atomicAdd(&tally[((Q[x] - qa) >> wshift) - (int)(g * kSliceGroup)], 1);
            }
        }
    }
    if (tid == 0 && lo == 0) atomicAdd(&tally[0], 1);  // the empty range lies in slice 0
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) mine_below += __shfl_xor(mine_below, m, kWave);
    if ((tid & (kWave - 1)) == 0) atomicAdd(&below, mine_below);
    __syncthreads();
    // exclusive scan of the slice counts (one wave, four slices to a lane), offset by the group's
    // place in the list
    if (tid < kWave) {
        int32_t v[4], sum = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[k] = tally[4 * tid + k];
            sum += v[k];
        }
        int32_t incl = sum;
#pragma unroll
        for (int dlt = 1; dlt < kWave; dlt <<= 1) {
            const int32_t o = __shfl_up(incl, dlt, kWave);
            if (tid >= dlt) incl += o;
        }
        int32_t run = below + incl - sum;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            tally[4 * tid + k] = run;
            run += v[k];
        }
    }
    static_assert(kSliceGroup == 4 * kWave, "one wave scans the counts, four to a lane");
    __syncthreads();
    // pass 2: the same budgets again, to their places
    if (tid == 0 && lo == 0) out[atomicAdd(&tally[0], 1)] = 0;
    for (int a0 = 1 + tid; a0 < n; a0 += THREADS * kBisect) {
        int a[kBisect], x0[kBisect], x1[kBisect];
#pragma unroll
        for (int j = 0; j < kBisect; ++j) a[j] = a0 + THREADS * j;
        if (lo > 0) {
            ends_below<kBisect>(Q, n, a, lo, x0);
        } else {
#pragma unroll
            for (int j = 0; j < kBisect; ++j) x0[j] = a[j];
        }
        ends_below<kBisect>(Q, n, a, hi, x1);
#pragma unroll
        for (int j = 0; j < kBisect; ++j) {
            if (a[j] < n) {
                const int32_t qa = Q[a[j]];
                for (int x = x0[j] + 1; x <= x1[j]; ++x) {
                    const int32_t sv = Q[x] - qa;
                    out[atomicAdd(&tally[(sv >> wshift) - (int)(g * kSliceGroup)], 1)] = sv;
                }
            }
        }
    }
}

constexpr int kSliceLongFrom = 1024;  // chains from this length on take the 1024-thread form
constexpr int kSliceShortUpTo = 128;  // chains up to this length have no more starts than two per lane of one wave

static_assert(links_lds_bytes(kSliceLongFrom) >= ((size_t)kSliceLongFrom + 1) * 4, "the links' LDS covers the prefix sums");

template <int THREADS, int kBisect>
__global__ __launch_bounds__(THREADS) void cubic_slice_kernel(int n, CubicWs w)
{
    slice_group<THREADS, kBisect>(n, w, blockIdx.x);
}

// Long chains: the links of the size stack and the layout of the budgets need the prologue's table
// and nothing of each other, and a single long chain fills the chip with neither (one workgroup, and
// one workgroup per CU).  One launch runs both: the first `batch` workgroups take the links of a
// chain each (they run longest, so they start first), the others a group of slices each.
static_assert(kLinksBlock == 1024, "the two parts share a launch of 1024 threads");
__global__ __launch_bounds__(kLinksBlock) void cubic_prepare_kernel(int n, int64_t batch, CubicWs w)
{
    if ((int64_t)blockIdx.x < batch)
        links_chain<kLinksBlock>(n, w, blockIdx.x);
    else
        slice_group<kLinksBlock, 4>(n, w, (int64_t)blockIdx.x - batch);
}

// ---- budgets kernel for 32-bit chains: the queue's shared part factored out -------------
//
// F_s(j) = d_j + m with m the head's value, and m changes only when the head
// leaves the window.  Between two such changes every value a lane inserts is
// d_h + m with the same m, so which of them survive at the tail does not depend
// on the lane: they are the chain t, below(t), .. of the size stack (El), cut
// off at the depth the stack had when the lane's head last changed, or has
// dropped to since (`base`).  A lane therefore stores nothing while its head
// stays.  When the head leaves, the lane writes that implicit part of its queue
// out to its ring (values d_h + m with the old m: they no longer compare like
// their sizes against what comes next), takes the new head from the ring's
// bottom, and starts an empty implicit part.  Entries in the ring are dropped
// from the top by the usual comparison with the incoming value; if the implicit
// part is not empty that comparison is false by itself (its bottom entry is
// below the incoming value and above everything in the ring).
// Per cell: one min (base) and two compares, "is the ring's top entry at least
// F(t) = d_t + m" taken as d_t <= X - m with X - m kept in a register, and
// "has the head left"; F(t) itself is formed when it is stored.  The rest is rare.
// A value that is the same in every lane, moved to scalar registers so that the
// arithmetic that follows runs on the scalar unit.
__device__ inline int32_t uniform(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline int64_t uniform(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Reads of the per-chain tables at a wave-uniform index, through the constant
// address space: they then go through the scalar unit whatever the compiler can
// or cannot prove about stores in between.  (The tables are written by an
// earlier kernel and only read here.)
typedef int32_t i32x2 __attribute__((ext_vector_type(2)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x16 __attribute__((ext_vector_type(16)));
#define CKPT_CONST_AS __attribute__((address_space(4)))
__device__ inline Step uniform_load(const Step *p, int i)
{
    const i32x2 v = ((const CKPT_CONST_AS i32x2 *)p)[i];
    return Step{v.x, v.y};
}

struct SharedLane {
    uint32_t hd, tl;   // the ring holds the written-out entries above the head at positions (hd, tl]
    int32_t hF, hK;    // the head: its value, its key P[h] + s
    int32_t X;         // value of the ring's top entry (kLow: the ring is empty)
    int32_t base;      // stack depth below the implicit part
    uint32_t over;     // the ring was too small at some point: the lane's result is not to be used
};


// With REDO the workgroups (one wave each) take the waves listed in w.redo
// instead of the waves of their own index.
// Otherwise workgroup b of a chain takes tile b * tile_stride of the laid-out
// budgets (tile_stride > 1: a sample of the budgets).  mode kSharedAll runs
// every tile it is given; kSharedPrune skips a wave whose smallest budget is
// above w.prune[c] or whose largest is below w.prune_lo[c] (no budget of the
// wave can then be optimal), and adds the budgets it does run to w.evaluated.
constexpr int kSharedAll = 0, kSharedPrune = 1;

template <int RING, int BLOCK, bool REDO>
__global__ __launch_bounds__(BLOCK) void cubic_shared_kernel(int n, int64_t blocks_per_chain, int tile_stride,
                                                             int mode, CubicWs w)
{
    typedef int32_t V;
    __shared__ __attribute__((aligned(RING * BLOCK * 8))) QueueEntry<V> ring[RING][BLOCK];
    constexpr V kLow = std::numeric_limits<V>::min();
    static_assert((BLOCK & (BLOCK - 1)) == 0 && (RING & (RING - 1)) == 0, "power-of-two ring");
    static_assert(!REDO || BLOCK == kWave, "the list is taken one wave at a time");

    const int64_t items = REDO ? *w.redo_count : 1;
    for (int64_t item = REDO ? blockIdx.x : 0; item < items; item += REDO ? gridDim.x : 1) {
    const int64_t listed = REDO ? w.redo[item] : 0;
    const int64_t launched = (blocks_per_chain + tile_stride - 1) / tile_stride;  // workgroups per chain
    const int64_t c = REDO ? listed / waves_per_chain(n) : blockIdx.x / launched;
    const int64_t tile = REDO ? listed % waves_per_chain(n) : (blockIdx.x % launched) * tile_stride;
    const ChainMeta meta = w.meta[c];
    if (meta.status != CKPT_OK || !meta.mode32) continue;

    const int tid = threadIdx.x;
    const El *__restrict__ el = w.el + (size_t)c * table_len(n);
    const Snap *__restrict__ snap = w.snap + (size_t)c * table_len(n);
    const Step *__restrict__ st = w.step + (size_t)c * step_len(n);
    const Group *__restrict__ gr = w.group + (size_t)c * group_len(n);
    const int64_t K = num_budgets(n);
    const int64_t idx = tile * BLOCK + tid;
    const int64_t wave_in_chain = idx / kWave;
    if (wave_in_chain * kWave >= K) continue;
    const bool live = idx < K;
    // lanes past the list take the largest budget, whose head never leaves, and are not counted:
    // a budget of 0 there would make this wave the slowest of the launch, and it starts last
    const V s = w.sorted[c * K + (live ? idx : K - 1)];
    if (!REDO && mode != kSharedAll) {
        const bool first = (tid & (kWave - 1)) == 0;
        // the wave's smallest and largest budget (slices ascend along the list, inside a slice any
        // order; lanes past the list hold a large budget and count as large)
        const V s_first = (V)wave_min_u32((uint32_t)s);
        const V s_last = (V)~wave_min_u32(~(uint32_t)(live ? s : std::numeric_limits<V>::max()));
        if (s_first > w.prune[c] || s_last < w.prune_lo[c] ||
            (tile_stride > 1 && w.skip_sample[c] != 0)) {
            if (first) {
                const int64_t slot_id = c * waves_per_chain(n) + wave_in_chain;
                w.partial[slot_id] = Partial{kInf, (int64_t)s};
                w.flags[slot_id] = 0;
            }
            continue;
        }
        const unsigned long long lanes = (unsigned long long)__popcll(__ballot(live));
        if (first) atomicAdd(w.evaluated + c, lanes);
    }

    typedef __attribute__((address_space(3))) V *LdsPtr;
    const uint32_t lane_base = (uint32_t)(uintptr_t)(LdsPtr)&ring[0][tid].F;

    SharedLane L;
    L.hd = 0; L.tl = 0;
    L.hF = el[0].d; L.hK = el[0].P + s; L.X = kLow;
    L.base = 1;  // the chain of position 0 is the head itself
    L.over = 0;
    V P = el[0].P;  // P[t], carried along on the scalar unit

    // cell t + 1: insert position t (implicitly), drop ring entries, check the head
    // Written out: 4 vector instructions when nothing happens; the rare part is
    // the same as shared_rare, with the wave's exec mask narrowed to the lanes
    // concerned.  t = t0 + u with u a literal, so that nothing is computed for the
    // rare part until it runs.  s84..s99 receive a snapshot.
    constexpr uint32_t kStep = (uint32_t)(BLOCK * sizeof(QueueEntry<V>));
    constexpr uint32_t kSlotMask = (uint32_t)(RING - 1) * kStep;
    constexpr int kShift = __builtin_ctz(kStep);
    const uint32_t snap_lo = (uint32_t)(uintptr_t)snap, snap_hi = (uint32_t)((uintptr_t)snap >> 32);
    const uint32_t el_lo = (uint32_t)(uintptr_t)el, el_hi = (uint32_t)((uintptr_t)el >> 32);
    const uint64_t snap_base = ((uint64_t)snap_hi << 32) | snap_lo, el_base = ((uint64_t)el_hi << 32) | el_lo;
    const V vLow = kLow;
#define CKPT_SNAP_STEP(PREG, DREG)                         \
    "v_cmp_lt_u32 vcc, %[sK], %[cnt]\n\t"                   \
    "s_cbranch_vccz Lmat_done_%=\n\t"                       \
    "s_mov_b64 exec, vcc\n\t"                               \
    "v_add_u32 %[f], " DREG ", %[m]\n\t"                    \
    "v_mov_b32 %[k], " PREG "\n\t"                          \
    "v_and_or_b32 %[ad], %[wp], %[mask], %[lo]\n\t"         \
    "ds_write2_b32 %[ad], %[f], %[k] offset1:1\n\t"         \
    "v_subrev_u32 %[wp], %[step], %[wp]\n\t"                \
    "s_add_u32 %[sK], %[sK], 1\n\t"
#define CKPT_SHARED_CELL(T0, U, E)                                                                        \
    {                                                                                                     \
        P += (E).d;                                                                                       \
        V Y;                                                                                              \
        uint32_t ad, f, k, cnt, wp, m, sK, sOff, sNext;                                                   \
        uint64_t sv0, sgone, st;                                                                          \
        asm volatile( \
            "v_add_u32 %[Y], %[sd], %[hF]\n\t" \
            "v_min_i32 %[base], %[su], %[base]\n\t" \
            "v_cmp_ge_i32 vcc, %[X], %[Y]\n\t" \
            "v_cmp_gt_i32 %[sgone], %[sP], %[hK]\n\t" \
            "s_or_b64 %[st], vcc, %[sgone]\n\t" \
            "s_cbranch_scc0 Lend_%=\n\t" \
            /* ---- rare.  If a head has left, ask for the snapshot of t now. */ \
            "s_cmp_eq_u64 %[sgone], 0\n\t" \
            "s_cbranch_scc1 Lpop_%=\n\t" \
            "s_add_u32 %[sOff], %[t0], %[u]\n\t" \
            "s_lshl_b32 %[sNext], %[sOff], 6\n\t" \
            "s_load_dwordx16 s[84:99], %[snapb], %[sNext]\n\t" \
            "s_lshl_b32 %[sOff], %[sOff], 4\n\t" \
            "s_add_u32 %[sOff], %[sOff], 8\n\t" \
            "s_load_dword %[sNext], %[elb], %[sOff]\n\t" \
            /* ---- ring entries not below the incoming value go */ \
            "Lpop_%=:\n\t" \
            "s_cbranch_vccz Lpop_done_%=\n\t" \
            "s_and_saveexec_b64 %[sv0], vcc\n\t" \
            "v_subrev_u32 %[tl], %[step], %[tl]\n\t" \
            "v_and_or_b32 %[ad], %[tl], %[mask], %[lo]\n\t" \
            "v_cmp_ne_u32 vcc, %[tl], %[hd]\n\t" \
            "v_mov_b32 %[X], %[vLow]\n\t" \
            "s_and_b64 exec, exec, vcc\n\t" \
            "ds_read_b32 %[X], %[ad]\n\t" \
            "s_waitcnt lgkmcnt(0)\n\t" \
            "s_mov_b64 exec, %[sv0]\n\t" \
            "v_cmp_ge_i32 vcc, %[X], %[Y]\n\t" \
            "s_branch Lpop_%=\n\t" \
            "Lpop_done_%=:\n\t" \
            "s_cmp_eq_u64 %[sgone], 0\n\t" \
            "s_cbranch_scc1 Lend_%=\n\t" \
            /* ---- the head has left (lanes sgone): write the implicit entries out, top first */ \
            "s_and_saveexec_b64 %[sv0], %[sgone]\n\t" \
            "s_add_u32 %[sOff], %[su], 1\n\t" \
            "v_sub_u32 %[cnt], %[sOff], %[base]\n\t" \
            "v_mov_b32 %[base], %[sOff]\n\t" \
            "v_mov_b32 %[m], %[hF]\n\t" \
            "v_lshl_add_u32 %[tl], %[cnt], %[shift], %[tl]\n\t" \
            "v_mov_b32 %[X], %[Y]\n\t" \
            "v_sub_u32 %[f], %[tl], %[hd]\n\t" \
            "v_cmp_lt_u32 vcc, %[cap], %[f]\n\t" \
            "v_cndmask_b32_e64 %[over], %[over], 1, vcc\n\t" \
            "v_mov_b32 %[k], %[sP]\n\t" \
            "v_and_or_b32 %[ad], %[tl], %[mask], %[lo]\n\t" \
            "ds_write2_b32 %[ad], %[Y], %[k] offset1:1\n\t" \
            "v_subrev_u32 %[wp], %[step], %[tl]\n\t" \
            "v_cmp_lt_u32 vcc, 1, %[cnt]\n\t" \
            "s_cbranch_vccz Lmat_done_%=\n\t" \
            "s_mov_b32 %[sK], 1\n\t" \
            "Lgroup_%=:\n\t" \
            "s_waitcnt lgkmcnt(0)\n\t" \
            CKPT_SNAP_STEP("s84", "s85") CKPT_SNAP_STEP("s86", "s87") CKPT_SNAP_STEP("s88", "s89") \
            CKPT_SNAP_STEP("s90", "s91") CKPT_SNAP_STEP("s92", "s93") CKPT_SNAP_STEP("s94", "s95") \
            CKPT_SNAP_STEP("s96", "s97") CKPT_SNAP_STEP("s98", "s99") \
            "v_cmp_lt_u32 vcc, %[sK], %[cnt]\n\t" \
            "s_cbranch_vccz Lmat_done_%=\n\t" \
            /* longer than a snapshot: go on with the snapshot of its last element */ \
            "s_lshl_b32 %[sOff], %[sNext], 6\n\t" \
            "s_load_dwordx16 s[84:99], %[snapb], %[sOff]\n\t" \
            "s_lshl_b32 %[sOff], %[sNext], 4\n\t" \
            "s_add_u32 %[sOff], %[sOff], 8\n\t" \
            "s_load_dword %[sNext], %[elb], %[sOff]\n\t" \
            "s_branch Lgroup_%=\n\t" \
            "Lmat_done_%=:\n\t" \
            "s_mov_b64 exec, %[sgone]\n\t" \
            /* ---- new head: the lowest entry still inside the window (the top one always is) */ \
            "Lseek_%=:\n\t" \
            "v_add_u32 %[hd], %[step], %[hd]\n\t" \
            "v_and_or_b32 %[ad], %[hd], %[mask], %[lo]\n\t" \
            "ds_read_b32 %[hF], %[ad]\n\t" \
            "ds_read_b32 %[k], %[ad] offset:4\n\t" \
            "s_waitcnt lgkmcnt(0)\n\t" \
            "v_add_u32 %[hK], %[k], %[s]\n\t" \
            "v_cmp_gt_i32 vcc, %[sP], %[hK]\n\t" \
            "v_cmp_ne_u32 %[st], %[hd], %[tl]\n\t" \
            "s_and_b64 vcc, vcc, %[st]\n\t" \
            "s_cbranch_vccz Lseek_done_%=\n\t" \
            "s_mov_b64 exec, vcc\n\t" \
            "s_branch Lseek_%=\n\t" \
            "Lseek_done_%=:\n\t" \
            "s_mov_b64 exec, %[sgone]\n\t" \
            "v_cmp_eq_u32 vcc, %[hd], %[tl]\n\t" \
            "v_cndmask_b32 %[X], %[X], %[vLow], vcc\n\t" \
            "s_mov_b64 exec, %[sv0]\n\t" \
            "Lend_%=:\n\t" \
            : [hd] "+v"(L.hd), [tl] "+v"(L.tl), [hF] "+v"(L.hF), [hK] "+v"(L.hK), [X] "+v"(L.X), [base] "+v"(L.base), \
              [over] "+v"(L.over), [Y] "=&v"(Y), [ad] "=&v"(ad), [f] "=&v"(f), [k] "=&v"(k), [cnt] "=&v"(cnt), \
              [wp] "=&v"(wp), [m] "=&v"(m), [sK] "=&s"(sK), [sOff] "=&s"(sOff), [sNext] "=&s"(sNext), [sv0] "=&s"(sv0), \
              [sgone] "=&s"(sgone), [st] "=&s"(st) \
            : [sd] "s"((E).d), [su] "s"((E).under), [sP] "s"(P), [t0] "s"(T0), [u] "i"(U), \
              [snapb] "s"(snap_base), [elb] "s"(el_base), [lo] "v"(lane_base), [s] "v"(s), [vLow] "v"(vLow), \
              [mask] "s"(kSlotMask), [step] "i"(kStep), [shift] "i"(kShift), [cap] "i"(RING * kStep) \
            : "vcc", "scc", "memory", "s84", "s85", "s86", "s87", "s88", "s89", "s90", "s91", "s92", "s93", "s94", "s95", \
              "s96", "s97", "s98", "s99"); \
    }
    // ---- the unguarded middle of the chain as one loop in assembly ------------------
    // A cell is
    //     P += d;  base = min(base, under);  pop = d <= Xr;  gone = P > hK
    // with Xr = X - hF (so that F(t) = d + hF need not be formed to compare it),
    // and does nothing else unless some lane pops or has lost its head.  As long as
    // no cell does more, X, hF and hK stay as they are; so none of kGroup consecutive
    // cells does exactly when the group's smallest size and last prefix sum do not,
    // and then the whole group is
    //     pop = dmin <= Xr;  gone = pend > hK;  base = min(base, umin);  P = pend.
    // Thirty-two cells per round: four groups, whose summaries come two at a time
    // into s[36:43] and s[44:51], loaded in turn one pair ahead (the summaries of a
    // chain are a quarter of its sizes and stay in the scalar cache).  The two groups
    // of a load are first tested as one (the smaller dmin and umin, which the
    // summaries carry as well, and the second pend), and singly only if that passes.  A group that passes the test loads
    // its eight (d, under) pairs into s[52:67] and takes its cells one by one; the
    // single groups, the cells and the rare parts of the cells sit behind the loop
    // and jump back.
    // Fixed registers: v80 Y, v81 address, v82/v83 entry, v84 count, v85 write
    // position, v86 old head value; s[68:83] snapshot, s[84:85] summaries' address,
    // s[86:87] saved exec, s[88:89] lanes whose head left, s[90:91] scratch mask,
    // s92 element counter, s93 offset, s94 next snapshot's position, s95 t of the
    // round's first cell, s96 rounds left.
#define SH_FAST(D, U, TAG)                                   \
    "s_add_u32 %[P], %[P], " D "\n\t"                        \
    "v_min_i32 %[base], " U ", %[base]\n\t"                  \
    "v_cmp_le_i32 vcc, " D ", %[Xr]\n\t"                     \
    "v_cmp_gt_i32 s[88:89], %[P], %[hK]\n\t"                 \
    "s_or_b64 s[90:91], vcc, s[88:89]\n\t"                   \
    "s_cbranch_scc1 Lrare_" TAG "_%=\n\t"                    \
    "Lback_" TAG "_%=:\n\t"
#define SH_SNAP_STEP(PREG, DREG, TAG)                        \
    "v_cmp_lt_u32 vcc, s92, v84\n\t"                         \
    "s_cbranch_vccz Lmat_done_" TAG "_%=\n\t"                \
    "s_mov_b64 exec, vcc\n\t"                                \
    "v_add_u32 v82, " DREG ", v86\n\t"                       \
    "v_mov_b32 v83, " PREG "\n\t"                            \
    "v_and_or_b32 v81, v85, %[mask], %[lo]\n\t"              \
    "ds_write2_b32 v81, v82, v83 offset1:1\n\t"              \
    "v_subrev_u32 v85, %[step], v85\n\t"                     \
    "s_add_u32 s92, s92, 1\n\t"
#define SH_RARE(D, U, TAG, TOFF)                             \
    "Lrare_" TAG "_%=:\n\t"                                  \
    "v_add_u32 v80, " D ", %[hF]\n\t"                        \
    "s_cmp_eq_u64 s[88:89], 0\n\t"                           \
    "s_cbranch_scc1 Lpop_" TAG "_%=\n\t"                     \
    "s_add_u32 s93, s95, " TOFF "\n\t"                       \
    "s_lshl_b32 s94, s93, 6\n\t"                             \
    "s_load_dwordx16 s[68:83], %[snapb], s94\n\t"            \
    "s_lshl_b32 s93, s93, 4\n\t"                             \
    "s_add_u32 s93, s93, 8\n\t"                              \
    "s_load_dword s94, %[elb], s93\n\t"                      \
    /* ring entries not below the incoming value go */       \
    "Lpop_" TAG "_%=:\n\t"                                   \
    "s_cbranch_vccz Lpop_done_" TAG "_%=\n\t"                \
    "s_and_saveexec_b64 s[86:87], vcc\n\t"                   \
    "v_subrev_u32 %[tl], %[step], %[tl]\n\t"                 \
    "v_and_or_b32 v81, %[tl], %[mask], %[lo]\n\t"            \
    "v_cmp_ne_u32 vcc, %[tl], %[hd]\n\t"                     \
    "v_mov_b32 %[X], %[vLow]\n\t"                            \
    "s_and_b64 exec, exec, vcc\n\t"                          \
    "ds_read_b32 %[X], v81\n\t"                              \
    "s_waitcnt lgkmcnt(0)\n\t"                               \
    "s_mov_b64 exec, s[86:87]\n\t"                           \
    "v_cmp_ge_i32 vcc, %[X], v80\n\t"                        \
    "s_branch Lpop_" TAG "_%=\n\t"                           \
    "Lpop_done_" TAG "_%=:\n\t"                              \
    "s_cmp_eq_u64 s[88:89], 0\n\t"                           \
    "s_cbranch_scc1 Lfin_" TAG "_%=\n\t"                     \
    /* the head has left (lanes s[88:89]): write the implicit entries out, top first */ \
    "s_and_saveexec_b64 s[86:87], s[88:89]\n\t"              \
    "s_add_u32 s93, " U ", 1\n\t"                            \
    "v_sub_u32 v84, s93, %[base]\n\t"                        \
    "v_mov_b32 %[base], s93\n\t"                             \
    "v_mov_b32 v86, %[hF]\n\t"                               \
    "v_lshl_add_u32 %[tl], v84, %[shift], %[tl]\n\t"         \
    "v_mov_b32 %[X], v80\n\t"                                \
    "v_sub_u32 v82, %[tl], %[hd]\n\t"                        \
    "v_cmp_lt_u32 vcc, %[cap], v82\n\t"                      \
    "v_cndmask_b32_e64 %[over], %[over], 1, vcc\n\t"         \
    "v_mov_b32 v83, %[P]\n\t"                                \
    "v_and_or_b32 v81, %[tl], %[mask], %[lo]\n\t"            \
    "ds_write2_b32 v81, v80, v83 offset1:1\n\t"              \
    "v_subrev_u32 v85, %[step], %[tl]\n\t"                   \
    "v_cmp_lt_u32 vcc, 1, v84\n\t"                           \
    "s_cbranch_vccz Lmat_done_" TAG "_%=\n\t"                \
    "s_mov_b32 s92, 1\n\t"                                   \
    "Lgroup_" TAG "_%=:\n\t"                                 \
    "s_waitcnt lgkmcnt(0)\n\t"                               \
    SH_SNAP_STEP("s68", "s69", TAG) SH_SNAP_STEP("s70", "s71", TAG) SH_SNAP_STEP("s72", "s73", TAG) \
    SH_SNAP_STEP("s74", "s75", TAG) SH_SNAP_STEP("s76", "s77", TAG) SH_SNAP_STEP("s78", "s79", TAG) \
    SH_SNAP_STEP("s80", "s81", TAG) SH_SNAP_STEP("s82", "s83", TAG) \
    "v_cmp_lt_u32 vcc, s92, v84\n\t"                         \
    "s_cbranch_vccz Lmat_done_" TAG "_%=\n\t"                \
    /* longer than a snapshot: go on with the snapshot of its last element */ \
    "s_lshl_b32 s93, s94, 6\n\t"                             \
    "s_load_dwordx16 s[68:83], %[snapb], s93\n\t"            \
    "s_lshl_b32 s93, s94, 4\n\t"                             \
    "s_add_u32 s93, s93, 8\n\t"                              \
    "s_load_dword s94, %[elb], s93\n\t"                      \
    "s_branch Lgroup_" TAG "_%=\n\t"                         \
    "Lmat_done_" TAG "_%=:\n\t"                              \
    "s_mov_b64 exec, s[88:89]\n\t"                           \
    /* new head: the lowest entry still inside the window (the top one always is) */ \
    "Lseek_" TAG "_%=:\n\t"                                  \
    "v_add_u32 %[hd], %[step], %[hd]\n\t"                    \
    "v_and_or_b32 v81, %[hd], %[mask], %[lo]\n\t"            \
    "ds_read_b32 %[hF], v81\n\t"                             \
    "ds_read_b32 v83, v81 offset:4\n\t"                      \
    "s_waitcnt lgkmcnt(0)\n\t"                               \
    "v_add_u32 %[hK], v83, %[s]\n\t"                         \
    "v_cmp_gt_i32 vcc, %[P], %[hK]\n\t"                      \
    "v_cmp_ne_u32 s[90:91], %[hd], %[tl]\n\t"                \
    "s_and_b64 vcc, vcc, s[90:91]\n\t"                       \
    "s_cbranch_vccz Lseek_done_" TAG "_%=\n\t"               \
    "s_mov_b64 exec, vcc\n\t"                                \
    "s_branch Lseek_" TAG "_%=\n\t"                          \
    "Lseek_done_" TAG "_%=:\n\t"                             \
    "s_mov_b64 exec, s[86:87]\n\t"                           \
    /* every lane: the top entry's value again, relative to the head's; none if the ring is empty */ \
    "Lfin_" TAG "_%=:\n\t"                                   \
    "v_cmp_eq_u32 vcc, %[hd], %[tl]\n\t"                     \
    "v_sub_u32 %[Xr], %[X], %[hF]\n\t"                       \
    "v_cndmask_b32 %[X], %[X], %[vLow], vcc\n\t"             \
    "v_cndmask_b32 %[Xr], %[Xr], %[vLow], vcc\n\t"           \
    "s_branch Lback_" TAG "_%=\n\t"
#define SH_GROUP(DMIN, PEND, UMIN, TAG)                      \
    "v_cmp_le_i32 vcc, " DMIN ", %[Xr]\n\t"                  \
    "v_cmp_gt_i32 s[88:89], " PEND ", %[hK]\n\t"             \
    "s_or_b64 s[90:91], vcc, s[88:89]\n\t"                  \
    "s_cbranch_scc1 Lcells_" TAG "_%=\n\t"                  \
    "v_min_i32 %[base], " UMIN ", %[base]\n\t"              \
    "s_mov_b32 %[P], " PEND "\n\t"                          \
    "Lgroup_done_" TAG "_%=:\n\t"
// Two groups at once, on the smaller of their smallest sizes and of their smallest depths (kept in
// the summaries' fourth words) and the second one's last prefix sum; the groups one by one, behind
// the loop, only if that test passes.
#define SH_PAIR(DMIN01, PEND1, UMIN01, TAG)                  \
    "v_cmp_le_i32 vcc, " DMIN01 ", %[Xr]\n\t"               \
    "v_cmp_gt_i32 s[88:89], " PEND1 ", %[hK]\n\t"           \
    "s_or_b64 s[90:91], vcc, s[88:89]\n\t"                  \
    "s_cbranch_scc1 Lpair_open_" TAG "_%=\n\t"              \
    "v_min_i32 %[base], " UMIN01 ", %[base]\n\t"            \
    "s_mov_b32 %[P], " PEND1 "\n\t"                         \
    "Lpair_done_" TAG "_%=:\n\t"
#define SH_CELLS(TAG, TOFF)                                  \
    "Lcells_" TAG "_%=:\n\t"                                \
    "s_add_u32 s93, s95, " TOFF "\n\t"                      \
    "s_lshl_b32 s93, s93, 3\n\t"                            \
    "s_load_dwordx16 s[52:67], %[stb], s93\n\t"             \
    "s_waitcnt lgkmcnt(0)\n\t"                              \
    SH_FAST("s52", "s53", TAG "c0") SH_FAST("s54", "s55", TAG "c1") SH_FAST("s56", "s57", TAG "c2") \
    SH_FAST("s58", "s59", TAG "c3") SH_FAST("s60", "s61", TAG "c4") SH_FAST("s62", "s63", TAG "c5") \
    SH_FAST("s64", "s65", TAG "c6") SH_FAST("s66", "s67", TAG "c7") \
    "s_branch Lgroup_done_" TAG "_%=\n\t"
#define SH_RARE8(TAG, T0, T1, T2, T3, T4, T5, T6, T7)       \
    SH_RARE("s52", "s53", TAG "c0", T0) SH_RARE("s54", "s55", TAG "c1", T1) SH_RARE("s56", "s57", TAG "c2", T2) \
    SH_RARE("s58", "s59", TAG "c3", T3) SH_RARE("s60", "s61", TAG "c4", T4) SH_RARE("s62", "s63", TAG "c5", T5) \
    SH_RARE("s64", "s65", TAG "c6", T6) SH_RARE("s66", "s67", TAG "c7", T7)
    static_assert(kGroup == 8 && sizeof(Group) == 16 && sizeof(Step) == 8, "the loads and shifts below");
    // What the assembly hard-codes: a snapshot is 64 bytes (position << 6), an El 16 bytes with the
    // link to the next snapshot at byte 8 (position << 4, + 8), a ring entry two words written by
    // one ds_write2_b32, a ring aligned to its own size so that an entry's address is
    // (position & mask) | lane base, and 32-bit table offsets (positions stay below 2^13 + padding).
    static_assert(sizeof(Snap) == 64 && sizeof(El) == 16 && offsetof(El, below) == 8, "snapshot and link offsets");
    static_assert(sizeof(QueueEntry<V>) == 8 && offsetof(QueueEntry<V>, K) == 4, "ring entry layout");
    static_assert(sizeof(ring) == (size_t)RING * BLOCK * 8 && alignof(decltype(ring)) >= 8, "ring size");
    static_assert(((size_t)CKPT_CUBIC_MAX_LAYERS + 64) * sizeof(Snap) < ((size_t)1 << 31), "32-bit table offsets");
    auto middle = [&](const int t_first, const int rounds) {
        V Xr = L.hd == L.tl ? kLow : L.X - L.hF;
        const uint64_t summaries = (uint64_t)(uintptr_t)(gr + group_slot(t_first / kGroup));
        const uint64_t st_base = (uint64_t)(uintptr_t)st;
        asm volatile(
            "s_mov_b64 s[84:85], %[summaries]\n\t"
            "s_mov_b32 s95, %[t_first]\n\t"
            "s_mov_b32 s96, %[rounds]\n\t"
            "s_load_dwordx8 s[36:43], s[84:85], 0x0\n\t"
            "Lround_%=:\n\t"
            "s_waitcnt lgkmcnt(0)\n\t"
            "s_load_dwordx8 s[44:51], s[84:85], 0x20\n\t"
            SH_PAIR("s39", "s41", "s43", "p0")
            "s_waitcnt lgkmcnt(0)\n\t"
            "s_load_dwordx8 s[36:43], s[84:85], 0x40\n\t"
            SH_PAIR("s47", "s49", "s51", "p1")
            "s_add_u32 s84, s84, 0x40\n\t"
            "s_addc_u32 s85, s85, 0\n\t"
            "s_add_u32 s95, s95, 32\n\t"
            "s_sub_u32 s96, s96, 1\n\t"
            "s_cmp_lg_u32 s96, 0\n\t"
            "s_cbranch_scc1 Lround_%=\n\t"
            "s_waitcnt lgkmcnt(0)\n\t"
            "s_branch Lexit_%=\n\t"
            "Lpair_open_p0_%=:\n\t"
            SH_GROUP("s36", "s37", "s38", "g0") SH_GROUP("s40", "s41", "s42", "g1")
            "s_branch Lpair_done_p0_%=\n\t"
            "Lpair_open_p1_%=:\n\t"
            SH_GROUP("s44", "s45", "s46", "g2") SH_GROUP("s48", "s49", "s50", "g3")
            "s_branch Lpair_done_p1_%=\n\t"
            SH_CELLS("g0", "0") SH_CELLS("g1", "8") SH_CELLS("g2", "16") SH_CELLS("g3", "24")
            SH_RARE8("g0", "0", "1", "2", "3", "4", "5", "6", "7")
            SH_RARE8("g1", "8", "9", "10", "11", "12", "13", "14", "15")
            SH_RARE8("g2", "16", "17", "18", "19", "20", "21", "22", "23")
            SH_RARE8("g3", "24", "25", "26", "27", "28", "29", "30", "31")
            "Lexit_%=:\n\t"
            : [hd] "+v"(L.hd), [tl] "+v"(L.tl), [hF] "+v"(L.hF), [hK] "+v"(L.hK), [X] "+v"(L.X), [Xr] "+v"(Xr),
              [base] "+v"(L.base), [over] "+v"(L.over), [P] "+s"(P)
            : [summaries] "s"(summaries), [stb] "s"(st_base), [t_first] "s"(t_first), [rounds] "s"(rounds),
              [snapb] "s"(snap_base), [elb] "s"(el_base), [lo] "v"(lane_base), [s] "v"(s), [vLow] "v"(vLow),
              [mask] "s"(kSlotMask), [step] "i"(kStep), [shift] "i"(kShift), [cap] "i"(RING * kStep)
            : "vcc", "scc", "memory", "v80", "v81", "v82", "v83", "v84", "v85", "v86", "s36", "s37", "s38", "s39", "s40",
              "s41", "s42", "s43", "s44", "s45", "s46", "s47", "s48", "s49", "s50", "s51", "s52", "s53", "s54", "s55",
              "s56", "s57", "s58", "s59", "s60", "s61", "s62", "s63", "s64", "s65", "s66", "s67", "s68", "s69", "s70",
              "s71", "s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", "s80", "s81", "s82", "s83", "s84", "s85",
              "s86", "s87", "s88", "s89", "s90", "s91", "s92", "s93", "s94", "s95", "s96");
    };
#undef SH_PAIR
#undef SH_GROUP
#undef SH_CELLS
#undef SH_RARE8
#undef SH_FAST
#undef SH_SNAP_STEP
#undef SH_RARE

    // The (d, depth) stream is read a block of kBlockCells positions ahead; two
    // register sets take turns, so nothing is copied.
    constexpr int kBlockCells = 8;
    Step A[kBlockCells], B[kBlockCells];
#define CKPT_GUARDED_CELL(U)                                         \
    if (!guarded || (t0 + (U) >= 1 && t0 + (U) <= n - 1)) CKPT_SHARED_CELL(t0, U, cur[U])
    auto block = [&](Step(&cur)[kBlockCells], Step(&ahead)[kBlockCells], const int t0, const bool guarded) {
        // Scalar loads return in any order, so waiting for this block's data also
        // waits for whatever else is in flight: make that wait happen here, before
        // the next block's loads are issued, not after.
        asm volatile("" : : "s"(cur[0].d), "s"(cur[kBlockCells - 1].under) : "memory");
#pragma unroll
        for (int u = 0; u < kBlockCells; ++u) ahead[u] = uniform_load(st, t0 + kBlockCells + u);
        CKPT_GUARDED_CELL(0) CKPT_GUARDED_CELL(1) CKPT_GUARDED_CELL(2) CKPT_GUARDED_CELL(3)
        CKPT_GUARDED_CELL(4) CKPT_GUARDED_CELL(5) CKPT_GUARDED_CELL(6) CKPT_GUARDED_CELL(7)
        static_assert(kBlockCells == 8, "eight cells are written out");
    };
#undef CKPT_GUARDED_CELL
#undef CKPT_SHARED_CELL
#undef CKPT_SNAP_STEP
#pragma unroll
    for (int u = 0; u < kBlockCells; ++u) A[u] = uniform_load(st, u);
    // blocks [kBlockCells, last_full) lie inside 1..n-1
    const int last_full = n / kBlockCells * kBlockCells;
    block(A, B, 0, true);
    int t0 = kBlockCells;
    if (last_full - t0 >= 32) {
        const int rounds = (last_full - t0) / 32;
        middle(t0, rounds);
        t0 += 32 * rounds;
#pragma unroll
        for (int u = 0; u < kBlockCells; ++u) B[u] = uniform_load(st, t0 + u);
    }
    for (; t0 + kBlockCells < last_full; t0 += 2 * kBlockCells) {
        block(B, A, t0, false);
        block(A, B, t0 + kBlockCells, false);
    }
    // here the next block's data is in B; at most one more full block and the tail remain
    if (t0 < last_full) {
        block(B, A, t0, false);
        t0 += kBlockCells;
        if (t0 <= n - 1) block(A, B, t0, true);
    } else if (t0 <= n - 1) {
        block(B, A, t0, true);
    }
    const V Fn = el[n].d + L.hF;
    const bool over = L.over != 0;

    const bool redo = live && over;
    const uint64_t flag = __ballot(redo);
    int64_t cost = (live && !over) ? (int64_t)s + (int64_t)Fn : kInf;
    int64_t sv = (int64_t)s;
    if (w.trace_s) {  // (a flagged lane's cost is written when it is computed again)
        const int64_t at = (c * waves_per_chain(n) + wave_in_chain) * kWave + (tid & (kWave - 1));
        w.trace_s[at] = live ? (int64_t)((uint64_t)sv << meta.shift) : -1;
        w.trace_cost[at] = (live && !over) ? (int64_t)((uint64_t)cost << meta.shift) : -1;
    }
    wave_min_pair(cost, sv);
    if ((tid & (kWave - 1)) == 0) {
        const int64_t slot_id = c * waves_per_chain(n) + wave_in_chain;
        w.partial[slot_id] = Partial{cost, sv};
        w.flags[slot_id] = flag;
        if (!REDO && flag != 0) w.redo[atomicAdd(w.redo_count, 1)] = slot_id;
    }
    }
}

constexpr int kRedoBlocks = 2048;

constexpr int kSampleStride = 64;  // a pruned call first runs every 64th tile of the laid-out budgets
// Pruning costs two more passes of at least one wave's running time each, and the budgets it
// keeps are the small ones, whose waves run longest: below this length it does not pay.
constexpr int kPruneFromLayers = 3072;

// The two bounds of a pruned call.  One workgroup per chain.
//
// Above: any s + c_s that was reached bounds the optimum from above (UB), and
// c_s >= d_0 + d_n for every s, so a budget above UB - d_0 - d_n cannot be optimal.
// Below: with m interior checkpoints the other interior layers form at most m+1
// segments of at most s each, so the checkpoints weigh at least
// sum(interior) - (m+1) s, and they weigh at least W(m), the m smallest interior
// sizes; hence c_s - d_0 - d_n >= LB(s) = min_m max(W(m), sum(interior) - (m+1) s),
// which does not grow with s: the budgets with LB(s) > UB - d_0 - d_n are those
// below some s_lo and cannot be optimal either.  (Both comparisons are strict, so
// neither cuts a budget that ties with the optimum.)
//
// Stage 0, before anything has run: UB from the costs of feasible sets (a checkpoint every
// ceil(sqrt(n)) layers; one greedy set per thread), W from a bitonic sort of the sizes in
// LDS, and whether the bounds are tight enough to do without a sample.
// Stage 1, after the sampled tiles (if they ran): UB from their results as well.
constexpr int kBoundThreads = 256;
constexpr int kSkipSampleBelow = 8;  // no sample when the first bounds leave under 1/8 of the budgets

__global__ __launch_bounds__(kBoundThreads) void cubic_bound_kernel(int n, int64_t blocks_per_chain,
                                                                    int tile_stride, int waves_per_tile, int stage,
                                                                    CubicWs w)
{
    __shared__ int64_t part[kBoundThreads];
    __shared__ int32_t srt[CKPT_CUBIC_MAX_LAYERS + 1];
    const int64_t c = blockIdx.x;
    const int tid = threadIdx.x;
    if (stage == 1 && c == 0 && tid == 0) *w.redo_count = 0;  // waves the sample flagged are run again anyway
    const ChainMeta meta = w.meta[c];
    if (meta.status != CKPT_OK || !meta.mode32) return;
    const El *el = w.el + (size_t)c * table_len(n);
    int32_t *W = w.wsum + c * ((int64_t)n + 1);
    const int m_int = n - 1;  // interior layers 1..n-1

    int64_t best = kInf, greedy = kInf;
    if (stage == 0) {
        // the interior sizes in ascending order, then their running sums
        int N = 1;
        while (N < m_int) N <<= 1;
        for (int t = tid; t < N; t += kBoundThreads) srt[t] = t < m_int ? el[t + 1].d : INT32_MAX;
        __syncthreads();
        // Upper bounds from greedy sets, before the sizes are put in order: thread t takes a segment
        // limit on a geometric grid around sqrt(n) mean sizes and walks the chain once, making a
        // checkpoint of every layer that would take its segment beyond the limit.  The set is
        // feasible, so its cost (its checkpoints plus its largest segment) bounds the optimum.
        {
            int seg_len = 1;
            while ((int64_t)seg_len * seg_len < n) ++seg_len;
            const float mean = (float)(el[n].P - el[0].d - el[n].d) / (float)(m_int > 0 ? m_int : 1);
            const float lim_f = mean * (float)seg_len * exp2f((float)(tid - kBoundThreads / 2) * (1.0f / 24.0f));
            // 32-bit sums: the chain's total is below 2^30 in this mode, and so is the limit
            const uint32_t lim = lim_f < 1.0f ? 1u : (lim_f > 1.0e9f ? 1000000000u : (uint32_t)lim_f);
            uint32_t ck = (uint32_t)el[0].d + (uint32_t)el[n].d, seg = 0, seg_max = 0;
#pragma unroll 8
            for (int k = 0; k < m_int; ++k) {
                const uint32_t x = (uint32_t)srt[k];
                const bool fits = seg + x <= lim;
                ck += fits ? 0u : x;
                seg_max = (!fits && seg > seg_max) ? seg : seg_max;
                seg = fits ? seg + x : 0u;
            }
            seg_max = seg > seg_max ? seg : seg_max;
            greedy = (int64_t)ck + seg_max;
        }
        __syncthreads();
        for (int k = 2; k <= N; k <<= 1)
            for (int j = k >> 1; j >= 1; j >>= 1) {
                for (int t = tid; t < N; t += kBoundThreads) {
                    const int o = t ^ j;
                    if (o > t) {
                        const int32_t a = srt[t], b = srt[o];
                        const bool up = (t & k) == 0;
                        if ((a > b) == up) { srt[t] = b; srt[o] = a; }
                    }
                }
                __syncthreads();
            }
        // running sums: every thread sums a contiguous piece, one thread chains the pieces
        const int piece = N / kBoundThreads > 0 ? N / kBoundThreads : 1;
        const int p0 = tid * piece;
        int64_t mine = 0;
        for (int t = p0; t < p0 + piece && t < m_int; ++t) mine += srt[t];
        part[tid] = mine;
        __syncthreads();
        if (tid == 0) {
            int64_t run = 0;
            for (int t = 0; t < kBoundThreads; ++t) { const int64_t x = part[t]; part[t] = run; run += x; }
        }
        __syncthreads();
        {
            int32_t run = (int32_t)part[tid];
            if (tid == 0) W[0] = 0;
            for (int t = p0; t < p0 + piece && t < m_int; ++t) { run += srt[t]; W[t + 1] = run; }
        }
        __syncthreads();
        // the cost of a checkpoint every ceil(sqrt(n)) layers, an upper bound to start from: thread g
        // takes the checkpoint at g * seg_len (position n for the last) and the segment after it
        int seg_len = 1;
        while ((int64_t)seg_len * seg_len < n) ++seg_len;
        int64_t ckpt = 0, seg_max = 0;
        for (int g = tid; g * seg_len <= n; g += kBoundThreads) {
            const int k0 = g * seg_len;
            ckpt += el[k0].d;
            int64_t seg = 0;
            for (int k = k0 + 1; k < k0 + seg_len && k < n; ++k) seg += el[k].d;
            seg_max = seg > seg_max ? seg : seg_max;
            if (k0 < n && k0 + seg_len > n) ckpt += el[n].d;  // the last, shorter segment ends at n
        }
        part[tid] = ckpt;
        __syncthreads();
        for (int half = kBoundThreads / 2; half >= 1; half >>= 1) {
            if (tid < half) part[tid] += part[tid + half];
            __syncthreads();
        }
        const int64_t ckpt_all = part[0];
        __syncthreads();
        part[tid] = seg_max;
        __syncthreads();
        for (int half = kBoundThreads / 2; half >= 1; half >>= 1) {
            if (tid < half) part[tid] = part[tid + half] > part[tid] ? part[tid + half] : part[tid];
            __syncthreads();
        }
        const int64_t sqrt_set = ckpt_all + part[0];
        __syncthreads();
        part[tid] = greedy;
        __syncthreads();
        for (int half = kBoundThreads / 2; half >= 1; half >>= 1) {
            if (tid < half) part[tid] = part[tid + half] < part[tid] ? part[tid + half] : part[tid];
            __syncthreads();
        }
        if (tid == 0) part[0] = sqrt_set < part[0] ? sqrt_set : part[0];
        __syncthreads();
    } else {
        const int64_t wpc = waves_per_chain(n);
        const int64_t launched = (blocks_per_chain + tile_stride - 1) / tile_stride;
        for (int64_t t = tid; t < launched * waves_per_tile; t += kBoundThreads) {
            const int64_t wave = (t / waves_per_tile) * tile_stride * waves_per_tile + t % waves_per_tile;
            if (wave < wpc) {
                const int64_t cost = w.partial[c * wpc + wave].cost;
                best = cost < best ? cost : best;
            }
        }
        part[tid] = best;
        __syncthreads();
        for (int half = kBoundThreads / 2; half >= 1; half >>= 1) {
            if (tid < half) part[tid] = part[tid + half] < part[tid] ? part[tid + half] : part[tid];
            __syncthreads();
        }
    }
    // The search below reads the running sums W a few hundred times, one read after the other:
    // from LDS (the sorted sizes are no longer needed), not from the workspace.
    __syncthreads();
    for (int t = tid; t <= m_int; t += kBoundThreads) srt[t] = W[t];
    __syncthreads();
    if (tid != 0) return;
    const int32_t *Wl = srt;
    // UB: this stage's, or the earlier stage's if that was better
    int64_t room = part[0] == kInf ? (int64_t)INT32_MAX : part[0] - el[0].d - el[n].d;  // UB - d_0 - d_n
    if (stage == 1 && (int64_t)w.prune[c] < room) room = w.prune[c];
    if (room >= INT32_MAX) return;
    w.prune[c] = (int32_t)room;
    // the smallest s with LB(s) <= room (LB(room) <= room holds: m = 0 gives at most sum - s ... or the
    // search ends at room + 1, which prunes nothing that the upper bound leaves)
    const int64_t sum_int = Wl[m_int];
    auto lower = [&](int64_t sv) -> int64_t {
        int lo = 0, hi = m_int;  // smallest m with W(m) >= sum - (m+1) s
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if ((int64_t)Wl[mid] >= sum_int - (int64_t)(mid + 1) * sv) hi = mid; else lo = mid + 1;
        }
        const int64_t a = Wl[lo];
        const int64_t b = sum_int - (int64_t)lo * sv;  // the max at m - 1 (for m = 0: no smaller m, a = 0 wins)
        return lo == 0 ? a : (a < b ? a : b);
    };
    int64_t lo = 0, hi = room + 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (lower(mid) <= room) hi = mid; else lo = mid + 1;
    }
    w.prune_lo[c] = (int32_t)(lo < INT32_MAX ? lo : INT32_MAX);
    if (stage == 0) {
        // About n (room - s_lo) / mean ranges have their sum between the bounds (n starts, and as many
        // lengths as mean sizes fit the gap).  If that is a small part of all budgets, running them all
        // costs less than a sample that would only tighten the bounds further.
        const int64_t mean = sum_int / (m_int > 0 ? m_int : 1) + 1;
        const int64_t inside = (int64_t)n * ((room - lo) / mean + 1);
        w.skip_sample[c] = inside <= num_budgets(n) / kSkipSampleBelow ? 1 : 0;
    }
}

// All waves with a ring of RING entries per lane (for a pruned call: a sample of them, the
// bound that the sample gives, then the waves that the bound leaves); then the waves in which
// the ring was too small again with REDO_RING entries; lanes flagged after that are left to
// the wave-per-budget kernel.
template <int RING, int BLOCK, int REDO_RING>
void launch_shared(int n, int64_t batch, bool pruned, CubicWs w, hipStream_t stream)
{
    const int64_t blocks_per_chain = (num_budgets(n) + BLOCK - 1) / BLOCK;
    if (pruned) {  // the first bounds (stage 0 of cubic_bound_kernel) have been launched by the caller
        const int64_t sampled = (blocks_per_chain + kSampleStride - 1) / kSampleStride;
        hipLaunchKernelGGL((cubic_shared_kernel<RING, BLOCK, false>), dim3((unsigned)(sampled * batch)), dim3(BLOCK),
                           0, stream, n, blocks_per_chain, kSampleStride, kSharedPrune, w);
        hipLaunchKernelGGL(cubic_bound_kernel, dim3((unsigned)batch), dim3(kBoundThreads), 0, stream, n,
                           blocks_per_chain, kSampleStride, BLOCK / kWave, 1, w);
    }
    hipLaunchKernelGGL((cubic_shared_kernel<RING, BLOCK, false>), dim3((unsigned)(blocks_per_chain * batch)),
                       dim3(BLOCK), 0, stream, n, blocks_per_chain, 1, pruned ? kSharedPrune : kSharedAll, w);
    const int64_t waves = waves_per_chain(n) * batch;
    hipLaunchKernelGGL((cubic_shared_kernel<REDO_RING, kWave, true>),
                       dim3((unsigned)(waves < kRedoBlocks ? waves : kRedoBlocks)), dim3(kWave), 0, stream, n,
                       blocks_per_chain, 1, kSharedAll, w);
}

// ---- one budget per wave ---------------------------------------------------------

// F_s(0..n) into LDS array F by a wave reduction over each window; returns
// F_s(n).  With pred != nullptr also records, for every j, the smallest h in
// the window with minimal F (lane 0 writes).  Must be called by a full wave
// that is the whole workgroup.
template <typename V>
__device__ V wave_budget_table(const PD<V> *__restrict__ pd, int n, V s, V *F, int32_t *pred)
{
    const int lane = threadIdx.x;
    if (lane == 0) F[0] = pd[0].d;
    __syncthreads();
    int l = 0;  // window start, uniform
    V last = pd[0].d;
    for (int j = 1; j <= n; ++j) {
        const V Pj1 = pd[j].P;
        while (Pj1 - pd[l + 1].P > s) ++l;  // P[j-1] - P[l] > s
        int64_t bv = kInf, bh = kInf;
        for (int h = l + lane; h <= j - 1; h += kWave) {
            const int64_t v = (int64_t)F[h];
            if (v < bv) { bv = v; bh = h; }
        }
        wave_min_pair(bv, bh);
        last = pd[j].d + (V)bv;
        if (lane == 0) {
            F[j] = last;
            if (pred) pred[j] = (int32_t)bh;
        }
        __syncthreads();
    }
    return last;
}

// Bytes of LDS that queue_budget_pred needs for a chain of n layers.
template <typename V>
__host__ __device__ inline size_t queue_pred_bytes(int n) { return ((size_t)n + 1) * (2 * sizeof(V) + 4); }

// Predecessors for one budget by Algorithm 4's queue itself, run as a single
// sequential pass (every lane carries the same state, held in scalar registers;
// lane 0 does the stores).
// Only strictly larger tails are dropped, so among equal minima the oldest
// stays at the head: pred16[j] is the smallest h in the window with minimal F.
// The queue has full capacity n+1 in LDS: entry (F, P[h] + s, h).
template <typename V>
__device__ void queue_budget_pred(const PD<V> *__restrict__ pd, int n, V s_in, unsigned char *lds,
                                  uint16_t *&pred16)
{
    const V s = uniform(s_in);
    const int n1 = n + 1;
    V *qF = (V *)lds;
    V *qK = qF + n1;
    uint16_t *qH = (uint16_t *)(qK + n1);
    pred16 = qH + n1;
    const bool writer = threadIdx.x == 0;
    int hd = 0, tl = 0;
    V hF = pd[0].d, tF = hF, hK = pd[1].P + s;
    int hH = 0;
    if (writer) {
        qF[0] = hF;
        qK[0] = hK;
        qH[0] = 0;
        pred16[1] = 0;
    }
    V Fprev = pd[1].d + hF;
    PD<V> cur[kCells], ahead[kCells];
#pragma unroll
    for (int u = 0; u < kCells; ++u) cur[u] = pd[u];
    for (int j0 = 0; j0 <= n; j0 += kCells) {
#pragma unroll
        for (int u = 0; u < kCells; ++u) ahead[u] = pd[j0 + kCells + u];
#pragma unroll
        for (int u = 0; u < kCells; ++u) {
            const int j = j0 + u;
            if (j < 2 || j > n) continue;
            const V Pj1 = cur[u].P;
            while (tF > Fprev) {  // the head is smaller than F(j-1), so this stops at it
                --tl;
                tF = uniform(qF[tl]);
            }
            ++tl;
            const V key = Pj1 + s;
            if (writer) {
                qF[tl] = Fprev;
                qK[tl] = key;
                qH[tl] = (uint16_t)(j - 1);
            }
            tF = Fprev;
            if (hd == tl - 1 && hK < Pj1) {  // the entry just stored becomes the head
                hd = tl;
                hF = Fprev; hK = key; hH = j - 1;
            }
            while (hK < Pj1) {
                ++hd;
                hF = uniform(qF[hd]);
                hK = uniform(qK[hd]);
                hH = uniform((int32_t)qH[hd]);
            }
            if (writer) pred16[j] = (uint16_t)hH;
            Fprev = cur[u].d + hF;
        }
#pragma unroll
        for (int u = 0; u < kCells; ++u) cur[u] = ahead[u];
    }
    __syncthreads();
}

// Bytes of LDS that epoch_budget_pred needs for a chain of n layers, without and
// with its own copy of the (P, d) table.
template <typename V>
__host__ __device__ inline size_t epoch_pred_bytes(int n, bool staged)
{
    return ((size_t)n + 2) * (sizeof(V) + 2 + (staged ? 2 * sizeof(V) : 0));
}

// Predecessors for one budget, a whole wave working on it.  While the head h of
// the window stays inside it, F(j) = d_j + F(h) and the predecessor of j is h,
// for every j at once; only when h leaves (cell e) is the new head looked for,
// as the smallest index with minimal F in the window of e.  That is the
// smallest minimal predecessor for every j until it leaves in turn: what
// enters the window later is larger than the minimum, and what lies before it
// is larger or gone.  STAGED: the (P, d) table is copied to LDS first, which
// takes the memory latency out of the steps from one head to the next.  Gives
// up (returns false) after `max_heads` heads; pred16[1..n] is then unset.
template <typename V, bool STAGED>
__device__ bool epoch_budget_pred(const PD<V> *__restrict__ pd, int n, V s_in, unsigned char *lds, int max_heads,
                                  uint16_t *&pred16)
{
    const V s = uniform(s_in);
    const int lane = threadIdx.x;
    const int n1 = n + 1;
    V *F = (V *)lds;                         // [n1]
    V *Pl = F + n1;                          // [n1 + 1]: Pl[j] = P[j-1]
    V *dl = Pl + n1 + 1;                     // [n1]
    pred16 = STAGED ? (uint16_t *)(dl + n1) : (uint16_t *)(F + n1);
    if (STAGED) {
        // eight loads in flight per lane (the table is padded past n+1, so a clamped index is enough)
        constexpr int kAhead = 8;
        for (int j0 = lane; j0 <= n1; j0 += kWave * kAhead) {
            PD<V> x[kAhead];
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int j = j0 + u * kWave;
                x[u] = pd[j <= n1 ? j : n1];
            }
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int j = j0 + u * kWave;
                if (j <= n1) Pl[j] = x[u].P;
                if (j < n1) dl[j] = x[u].d;
            }
        }
        __syncthreads();
    }
    auto P_at = [&](int j) -> V { return STAGED ? Pl[j] : pd[j].P; };  // P[j-1]
    auto d_at = [&](int j) -> V { return STAGED ? dl[j] : pd[j].d; };
    if (lane == 0) F[0] = d_at(0);
    int h = 0, heads = 1;
    V m = d_at(0);          // F(h)
    V limit = P_at(1) + s;  // cells j with P[j-1] above this no longer see h
    int t = 1;
    while (t <= n) {
        // cells t.. up to the first one that no longer sees h
        int e = n1;
        for (int j0 = t; j0 <= n; j0 += kWave) {
            const int j = j0 + lane;
            const int jc = j < n1 ? j : n;
            const V xP = P_at(jc), xd = d_at(jc);
            const uint64_t out = __builtin_amdgcn_ballot_w64(j <= n && xP > limit);
            const int first = out ? j0 + (__ffsll((unsigned long long)out) - 1) : n1;
            if (j <= n && j < first) {
                F[j] = xd + m;
                pred16[j] = (uint16_t)h;
            }
            if (out) {
                e = first;
                break;
            }
        }
        if (e > n) break;
        if (++heads > max_heads) return false;
        __syncthreads();
        // window of e: indices i in (h, e-1] with P[e-1] - P[i] <= s; its start is near h
        const V Pe = P_at(e);
        {
            // Usual case, the window is shorter than a wave: the lanes take i = e-1, e-2, .. (the
            // window is a prefix of them), one reduction gives the minimum, and the highest lane
            // that holds it is the smallest index; its P[i] is the new head's key.
            const int i = e - 1 - lane;
            const bool valid = i > h;
            const int ic = valid ? i : e - 1;
            const V pi = P_at(ic + 1);  // P[ic]
            const V fi = F[ic];
            const bool in = valid && Pe - pi <= s;
            if (__builtin_amdgcn_ballot_w64(in) != ~0ull) {
                const V vmax = std::numeric_limits<V>::max();
                const V v = in ? fi : vmax;  // (values are positive: they order as unsigned)
                V mn;
                if constexpr (sizeof(V) == 4)
                    mn = (V)wave_min_u32((uint32_t)v);
                else
                    mn = (V)wave_min_u64((uint64_t)v);
                const uint64_t eq = __builtin_amdgcn_ballot_w64(in && v == mn);
                const int sel = 63 - __clzll((unsigned long long)eq);
                h = e - 1 - sel;
                m = mn;
                if constexpr (sizeof(V) == 4)
                    limit = (V)__builtin_amdgcn_readlane((int)pi, sel) + s;
                else
                    limit = (V)shfl_i64((int64_t)pi, sel) + s;
                t = e;
                continue;
            }
        }
        int l = e - 1;
        for (int i0 = h + 1; i0 <= e - 1; i0 += kWave) {
            const int i = i0 + lane;
            const uint64_t in = __builtin_amdgcn_ballot_w64(i <= e - 1 && Pe - P_at((i < n ? i : n) + 1) <= s);
            if (in) {
                l = i0 + (__ffsll((unsigned long long)in) - 1);
                break;
            }
        }
        int64_t bv = kInf, bh = kInf;
        for (int i = l + lane; i <= e - 1; i += kWave) {
            const int64_t v = (int64_t)F[i];
            if (v < bv) { bv = v; bh = i; }
        }
        wave_min_pair(bv, bh);
        h = (int)bh;
        m = (V)bv;
        limit = P_at(h + 1) + s;
        t = e;
    }
    __syncthreads();
    return true;
}

// Tries the forms of the predecessor pass that fit the LDS granted to the kernel, fastest first.
// Returns with pred16 (in LDS) set, or nullptr when the predecessors are in pred (in the workspace).
template <typename V>
__device__ void budget_pred(const PD<V> *__restrict__ pd, int n, V s, unsigned char *lds, size_t lds_bytes,
                            int32_t *pred, uint16_t *&pred16)
{
    if (epoch_pred_bytes<V>(n, true) <= lds_bytes) {
        if (epoch_budget_pred<V, true>(pd, n, s, lds, n / 16 + 8, pred16)) return;
    } else if (epoch_pred_bytes<V>(n, false) <= lds_bytes) {
        if (epoch_budget_pred<V, false>(pd, n, s, lds, n / 16 + 8, pred16)) return;
    }
    if (queue_pred_bytes<V>(n) <= lds_bytes) {
        queue_budget_pred<V>(pd, n, s, lds, pred16);
        return;
    }
    pred16 = nullptr;
    wave_budget_table<V>(pd, n, s, (V *)lds, pred);
}

__global__ __launch_bounds__(kWave) void cubic_overflow_kernel(int n, int64_t n_words, CubicWs w)
{
    const int64_t wpc = waves_per_chain(n);
    const int lane = threadIdx.x;
    // 64 flag words are looked at per step, one per lane; flagged ones are then
    // taken one at a time by the whole wave
    for (int64_t w0 = (int64_t)blockIdx.x * kWave; w0 < n_words; w0 += (int64_t)gridDim.x * kWave) {
        uint64_t mine = 0;
        if (w0 + lane < n_words && w.meta[(w0 + lane) / wpc].status == CKPT_OK) mine = w.flags[w0 + lane];
        uint64_t pending = __builtin_amdgcn_ballot_w64(mine != 0);  // chains in error never wrote their words
        while (pending) {
            const int src = __ffsll((unsigned long long)pending) - 1;
            pending &= pending - 1;
            const int64_t word = w0 + src;
            uint64_t flag = (uint64_t)shfl_i64((int64_t)mine, src);
            const int64_t c = word / wpc;
            const int64_t base = (word % wpc) * kWave;
            const ChainMeta meta = w.meta[c];
            Partial best = w.partial[word];
            while (flag) {
                const int bit = __ffsll((unsigned long long)flag) - 1;
                flag &= flag - 1;
                int64_t s64, cost;
                if (meta.mode32) {
                    const PD<int32_t> *pd = chain_table<int32_t>(w, c, n);
                    const int32_t s = w.sorted[c * num_budgets(n) + base + bit];
                    s64 = s;
                    cost = s64 + wave_budget_table<int32_t>(pd, n, s, (int32_t *)dyn_lds, nullptr);
                } else {
                    const PD<int64_t> *pd = chain_table<int64_t>(w, c, n);
                    s64 = budget_value<int64_t>(pd, base + bit, n);
                    cost = s64 + wave_budget_table<int64_t>(pd, n, s64, (int64_t *)dyn_lds, nullptr);
                }
                if (cost < best.cost || (cost == best.cost && s64 < best.s)) best = Partial{cost, s64};
                if (w.trace_s && lane == 0) w.trace_cost[word * kWave + bit] = (int64_t)((uint64_t)cost << meta.shift);
                __syncthreads();
            }
            if (lane == 0) w.partial[word] = best;
        }
    }
}

// ---- second-level reduction for long chains ------------------------------------------

// A chain of n = 4096 layers leaves 131,073 per-wave results; one wave reading
// them one after the other would take longer than the budgets kernel's tail, so
// kReduceBlocks workgroups per chain fold them first.
__global__ __launch_bounds__(256) void cubic_reduce_kernel(int n, CubicWs w)
{
    __shared__ Partial part[4];
    const int64_t c = blockIdx.y;
    if (w.meta[c].status != CKPT_OK) return;
    const int64_t wpc = waves_per_chain(n);
    const int64_t per = (wpc + kReduceBlocks - 1) / kReduceBlocks;
    const int64_t lo = (int64_t)blockIdx.x * per;
    const int64_t hi = lo + per < wpc ? lo + per : wpc;
    const Partial *src = w.partial + c * wpc;
    int64_t cost = kInf, s = kInf;
#pragma unroll 4
    for (int64_t t = lo + threadIdx.x; t < hi; t += 256) {
        const Partial p = src[t];
        if (p.cost < cost || (p.cost == cost && p.s < s)) { cost = p.cost; s = p.s; }
    }
    wave_min_pair(cost, s);
    if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = Partial{cost, s};
    __syncthreads();
    if (threadIdx.x == 0) {
        Partial best = part[0];
        for (int k = 1; k < 4; ++k)
            if (part[k].cost < best.cost || (part[k].cost == best.cost && part[k].s < best.s)) best = part[k];
        w.partial2[c * kReduceBlocks + blockIdx.x] = best;
    }
}

// ---- epilogue --------------------------------------------------------------------

__global__ __launch_bounds__(kWave) void cubic_epilogue_kernel(int n, size_t lds_bytes, int64_t cstride,
                                                               int64_t pstride, uint8_t *__restrict__ mask_out,
                                                               int64_t *__restrict__ peak_out,
                                                               int64_t *__restrict__ budget_out,
                                                               int32_t *__restrict__ status_out,
                                                               int64_t *__restrict__ evaluated_out, bool pruned,
                                                               CubicWs w)
{
    const int64_t c = blockIdx.x;
    const int lane = threadIdx.x;
    const int n1 = n + 1;
    const ChainMeta meta = w.meta[c];
    uint8_t *mp = mask_out + c * cstride;
    if (lane == 0 && status_out) status_out[c] = meta.status;
    if (lane == 0 && evaluated_out)  // only the 32-bit path prunes
        evaluated_out[c] = meta.status != CKPT_OK ? 0
                           : (pruned && meta.mode32) ? (int64_t)w.evaluated[c] : num_budgets(n);
    if (meta.status != CKPT_OK) {
        for (int k = lane; k < n1; k += kWave) mp[(int64_t)k * pstride] = 0;
        if (lane == 0) {
            peak_out[c] = -1;
            if (budget_out) budget_out[c] = -1;
        }
        return;
    }
    const int64_t wpc = waves_per_chain(n);
    const bool folded = wpc > kReduceFrom;
    const Partial *src = folded ? w.partial2 + c * kReduceBlocks : w.partial + c * wpc;
    const int64_t count = folded ? kReduceBlocks : wpc;
    int64_t cost = kInf, s = kInf;
    for (int64_t t = lane; t < count; t += kWave) {
        const Partial p = src[t];
        if (p.cost < cost || (p.cost == cost && p.s < s)) { cost = p.cost; s = p.s; }
    }
    wave_min_pair(cost, s);

    // predecessors: the sequential queue when its arrays fit the LDS granted to
    // the kernel, else the wave-per-window table
    int32_t *pred = w.pred + c * n1;
    uint16_t *pred16 = nullptr;
    if (meta.mode32)
        budget_pred<int32_t>(chain_table<int32_t>(w, c, n), n, (int32_t)s, dyn_lds, lds_bytes, pred, pred16);
    else
        budget_pred<int64_t>(chain_table<int64_t>(w, c, n), n, s, dyn_lds, lds_bytes, pred, pred16);

    // the value table is no longer needed: its LDS (the first n+1 bytes, below
    // pred16) becomes the mark array
    uint8_t *mark = dyn_lds;
    __syncthreads();
    for (int k = lane; k < n1; k += kWave) mark[k] = 0;
    __syncthreads();
    if (lane == 0) {
        int j = n;
        mark[n] = 1;
        while (j > 0) {
            j = pred16 ? (int)pred16[j] : pred[j];
            mark[j] = 1;
        }
        peak_out[c] = cost << meta.shift;
        if (budget_out) budget_out[c] = s << meta.shift;
    }
    __syncthreads();
    for (int k = lane; k < n1; k += kWave) mp[(int64_t)k * pstride] = mark[k];
}

}  // namespace

size_t cubic_workspace_bytes(int64_t batch, int n)
{
    const size_t n1 = (size_t)n + 1, B = (size_t)batch, wpc = (size_t)waves_per_chain(n);
    return align_up(B * sizeof(ChainMeta)) + align_up(B * table_len(n) * sizeof(PD<int64_t>)) +
           align_up(B * table_len(n) * sizeof(El)) + align_up(B * table_len(n) * sizeof(Snap)) +
           align_up(B * step_len(n) * sizeof(Step)) + align_up(B * group_len(n) * sizeof(Group)) + align_up(B * (size_t)num_budgets(n) * 4) + 256 + align_up(B * wpc * 8) +
           align_up(B * wpc * sizeof(Partial)) + align_up(B * wpc * 8) +
           align_up(B * kReduceBlocks * sizeof(Partial)) + align_up(B * n1 * 4) + 3 * align_up(B * 4) +
           align_up(B * n1 * 4) + align_up(B * 8) + 256;
}

int64_t cubic_trace_len(int n) { return waves_per_chain(n) * kWave; }

namespace {

// Once per device: the links kernel of long chains needs more dynamic LDS than the default limit.
constexpr int kMaxDevices = 64;
std::atomic<bool> links_lds_raised[kMaxDevices];

hipError_t raise_links_lds_limit()
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (links_lds_raised[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute((const void *)cubic_links_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)links_lds_bytes(CKPT_CUBIC_MAX_LAYERS));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)cubic_prepare_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)links_lds_bytes(CKPT_CUBIC_MAX_LAYERS));
    if (e == hipSuccess) links_lds_raised[dev].store(true, std::memory_order_release);
    return e;
}

}  // namespace

hipError_t launch_solve_cubic(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                              int64_t *peak_out, int64_t *budget_out, int32_t *status_out, bool pruned,
                              int64_t *evaluated_out, int64_t *trace_s, int64_t *trace_cost, void *ws,
                              hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    pruned = pruned && n >= kPruneFromLayers;
    CubicWs w = carve_cubic(ws, batch, n);
    const int64_t K = num_budgets(n);
    const int64_t total_blocks = (K + kWave - 1) / kWave * batch;  // the largest grid: one wave per workgroup
    const int64_t n_words = waves_per_chain(n) * batch;
    if (total_blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    {
        // The shared kernel's loop reads group summaries up to three pairs past the last group it uses
        // and (d, depth) pairs up to 15 positions past n - 1: the tables are padded for that.
        const int last_full = n / 8 * 8;
        const int rounds = last_full - 8 >= 32 ? (last_full - 8) / 32 : 0;
        if (group_slot(1) + 4 * (size_t)rounds + 2 > group_len(n) || (size_t)n + 15 > step_len(n) ||
            (size_t)n + 1 + kSnap > table_len(n))
            return hipErrorInvalidValue;
    }
    const size_t table_lds = ((size_t)n + 1) * 8;
    w.trace_s = trace_s;
    w.trace_cost = trace_cost;

    hipLaunchKernelGGL(cubic_prologue_kernel, dim3((unsigned)batch), dim3(kWave), 0, stream, d, batch, n,
                       st.chain, st.pos, w);
    if (links_lds_bytes(n) > 65536) {  // beyond the default limit for dynamic LDS
        const hipError_t e = raise_links_lds_limit();
        if (e != hipSuccess) return e;
    }
    // Everything runs on the caller's stream: the tables of the size stack and the budgets grouped by
    // value (one launch for long chains, two for short ones), then the first bounds of a pruned call
    // (they need those tables only).
    if (n >= kSliceLongFrom) {
        const int64_t blocks = (slice_groups(n) + 1) * batch;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL(cubic_prepare_kernel, dim3((unsigned)blocks), dim3(kLinksBlock), links_lds_bytes(n), stream,
                           n, batch, w);
    } else {
        hipLaunchKernelGGL(cubic_links_kernel, dim3((unsigned)batch), dim3(kLinksShortBlock), links_lds_bytes(n), stream,
                           n, w);
        if (n <= kSliceShortUpTo)
            hipLaunchKernelGGL((cubic_slice_kernel<64, 2>), dim3((unsigned)(slice_groups(n) * batch)), dim3(64),
                               ((size_t)n + 1) * 4, stream, n, w);
        else
            hipLaunchKernelGGL((cubic_slice_kernel<256, 8>), dim3((unsigned)(slice_groups(n) * batch)), dim3(256),
                               ((size_t)n + 1) * 4, stream, n, w);
    }
    if (pruned)
        hipLaunchKernelGGL(cubic_bound_kernel, dim3((unsigned)batch), dim3(kBoundThreads), 0, stream, n,
                           (num_budgets(n) + kWave - 1) / kWave, kSampleStride, 1, 0, w);
    launch_shared<16, 64, 64>(n, batch, pruned, w, stream);
    launch_budgets<int64_t, 16, 64>(n, batch, w, stream);
    const int64_t word_groups = (n_words + kWave - 1) / kWave;
    const unsigned over_grid = (unsigned)(word_groups < 4096 ? word_groups : 4096);
    hipLaunchKernelGGL(cubic_overflow_kernel, dim3(over_grid), dim3(kWave), table_lds, stream, n, n_words, w);
    if (waves_per_chain(n) > kReduceFrom)
        hipLaunchKernelGGL(cubic_reduce_kernel, dim3(kReduceBlocks, (unsigned)batch), dim3(256), 0, stream, n, w);
    // the epilogue takes as much LDS as the largest form of the predecessor pass that fits 64 KiB wants
    size_t epi_lds = table_lds;
    const size_t wishes[] = {queue_pred_bytes<int32_t>(n), queue_pred_bytes<int64_t>(n),
                             epoch_pred_bytes<int32_t>(n, false), epoch_pred_bytes<int64_t>(n, false),
                             epoch_pred_bytes<int32_t>(n, true), epoch_pred_bytes<int64_t>(n, true)};
    for (const size_t wish : wishes)
        if (wish <= 65536 && wish > epi_lds) epi_lds = wish;
    hipLaunchKernelGGL(cubic_epilogue_kernel, dim3((unsigned)batch), dim3(kWave), epi_lds, stream, n, epi_lds,
                       st.chain, st.pos, mask_out, peak_out, budget_out, status_out, evaluated_out, pruned, w);
    return hipGetLastError();
}

}  // namespace ckpt
