// Memory per training phase index for a given checkpoint set (Section 5.1,
// "training phase index": 0 before training, 1..n the forward stage of layer
// i, n+1..2n the backward stages of layers n..1, 2n+1 after training), under
// the memory behaviour of Algorithm 2 (static objective) or Algorithm 3
// (dynamic objective), one lane per chain.
//
// A stage's value is the live memory after the stage's allocations and before
// the release at its end:
//   forward stage i     sum_{c in C, c <= i-1} d_c + d_i + [i-1 not in C] d_{i-1}
//   backward stage of layer i, with h the last checkpoint below i and nx the
//   first checkpoint at or above i:
//     Algorithm 3       sum_{c in C, c <= h} d_c + sum_{k=h+1}^{i} d_k + max_{h<=k<nx} d_k
//                       (Equation (memory) for i = nx, Equation (iprime) otherwise)
//     Algorithm 2       sum_{c in C} d_c + sum_{h<k<nx} d_k
//   index 0 and 2n+1    d_0
// so the largest backward stage is the peak that ckpt_eval_peak returns.
//
// A backward stage needs something from each side of position i: the part of
// its segment below i (running sums from the pass itself) and the part above,
// max or sum of d_i..d_{nx-1}.  The kernel walks the chain once, upwards, in
// chunks of kChunk rows held in registers, with the next chunk already loaded
// and the one after it in flight.  For a chunk it first finds what lies above
// the chunk's last row (it scans the next chunk's registers up to the first
// checkpoint; while some lane of the wave has found none, the wave goes on
// with the rows in flight and then with eight further rows at a time),
// then sweeps the chunk downwards in registers to get the part above every
// row, then upwards to write both stages of every row.  Algorithm 3's stages
// need nothing else, so that objective reads 9(n+1) bytes and writes 16(n+1)
// per chain, which is what the method itself has to move.  Algorithm 2's
// stages all contain the sum of ALL checkpoints, which is only known at the
// end of the chain, so that objective passes over the chain once more
// beforehand; chains of up to 160 layers whose sizes fit 31 bits are left in
// LDS by that pass, and the walk reads them from there.
#include "ckpt_internal.h"

namespace ckpt {
namespace {

constexpr int kBlock = 64;
constexpr int kChunk = 8;
// Under Algorithm 2 the chains of up to this many layers are kept in LDS between the two passes
// (256 bytes per row and wave: 40 KB at most, so that four waves still fit a CU; with fewer the
// kernel is slower than reading the chain twice: 2.8 ms against 2.0 ms at n = 256).
constexpr int kLdsRowsMaxLayers = 160;

// The walk up the chain that writes both stages of every row.  ld(r) and lm(r) give the size and
// the mask byte of row r, 1 <= r <= n (from memory, or from the copy the first pass left in LDS).
template <int OBJ, class LD, class LM>
__device__ __forceinline__ void timeline_walk(const LD ld, const LM lm, const int n, const int64_t x0,
                                              const bool bad_mask, const uint64_t ckpt_all,
                                              int64_t *__restrict__ op, const int64_t opstride,
                                              int32_t *__restrict__ status_out, const int64_t c)
{
    const int64_t last = 2 * (int64_t)n + 1;
    // the part of a segment above a row: its largest size (Algorithm 3) or its sum (Algorithm 2).
    // Sums are unsigned so that an invalid chain cannot trip signed overflow.
    auto join = [](uint64_t acc, int64_t x) -> uint64_t {
        return OBJ == CKPT_OBJ_STATIC ? acc + (uint64_t)x : ((uint64_t)x > acc ? (uint64_t)x : acc);
    };

    // rows beyond n re-read row n and are not used
    // the masks of a chunk that has arrived are kept as one bit per row
    int64_t cur_d[kChunk], nxt_d[kChunk];
    uint32_t cur_m = 0, nxt_m = 0;
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
        const int a = min(1 + u, n), b = min(1 + kChunk + u, n);
        cur_d[u] = ld(a); cur_m |= (uint32_t)(lm(a) != 0) << u;
        nxt_d[u] = ld(b); nxt_m |= (uint32_t)(lm(b) != 0) << u;
    }

    bool bad_size = x0 <= 0, ovf = false;
    uint64_t total = (uint64_t)x0;
    int64_t dmax = x0;

    op[0] = x0;
    uint64_t below = (uint64_t)x0;  // checkpoints up to the last one below the row
    uint64_t seg = 0;               // non-checkpoints since then
    int64_t segmax = x0;            // largest size from that checkpoint up to the row before
    int64_t prev = 0;               // the row before, if it is no checkpoint, else 0

    for (int k0 = 1; k0 <= n; k0 += kChunk) {
        int64_t far_d[kChunk];
        uint8_t far_m[kChunk];
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const int a = min(k0 + 2 * kChunk + u, n);
            far_d[u] = ld(a); far_m[u] = lm(a);
        }

        // what lies above the chunk's last row: d from the next chunk's first row up to (not
        // including) the first checkpoint.  Most lanes find it among the next chunk's rows; as
        // long as some lane of the wave has not, the whole wave looks at eight more rows: first
        // the ones already requested for the chunk after next, then further ones, eight loads
        // at a time (one memory latency per round instead of one per row).
        uint64_t acc = 0;
        bool found = false;
        auto bits = [](const uint8_t(&mm)[kChunk]) -> uint32_t {
            uint32_t b = 0;
#pragma unroll
            for (int u = 0; u < kChunk; ++u) b |= (uint32_t)(mm[u] != 0) << u;
            return b;
        };
        auto scan = [&](const int64_t(&dd)[kChunk], const uint32_t mm, const int first_row) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                const bool ck = (mm >> u) & 1u;
                const bool open = !found && (first_row + u) <= n;
                found |= (first_row + u) > n || ck;
                if (open && !ck) acc = join(acc, dd[u]);
            }
        };
        scan(nxt_d, nxt_m, k0 + kChunk);
        if (__builtin_amdgcn_ballot_w64(!found) != 0) {
            scan(far_d, bits(far_m), k0 + 2 * kChunk);
            for (int kb = k0 + 3 * kChunk; __builtin_amdgcn_ballot_w64(!found) != 0; kb += kChunk) {
                int64_t more_d[kChunk];
                uint8_t more_m[kChunk];
#pragma unroll
                for (int u = 0; u < kChunk; ++u) {
                    const int a = min(kb + u, n);
                    more_d[u] = ld(a); more_m[u] = lm(a);
                }
                scan(more_d, bits(more_m), kb);
            }
        }

        // downwards: the part above each row of the chunk (the row itself included)
        uint64_t above[kChunk];
#pragma unroll
        for (int u = kChunk - 1; u >= 0; --u) {
            if (k0 + u <= n) acc = ((cur_m >> u) & 1u) ? 0 : join(acc, cur_d[u]);
            above[u] = acc;
        }

        // upwards: both stages of each row
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const int i = k0 + u;
            if (i > n) break;
            const int64_t x = cur_d[u];
            bad_size |= x <= 0;
            total += (uint64_t)x;
            ovf |= total > (uint64_t)INT64_MAX;
            dmax = x > dmax ? x : dmax;
            __builtin_nontemporal_store((int64_t)(below + (uint64_t)x + (uint64_t)prev), op + (int64_t)i * opstride);
            uint64_t b;
            if (OBJ == CKPT_OBJ_STATIC)
                b = ckpt_all + seg + above[u];
            else
                b = below + seg + (uint64_t)x + ((uint64_t)segmax > above[u] ? (uint64_t)segmax : above[u]);
            __builtin_nontemporal_store((int64_t)b, op + (last - i) * opstride);
            if ((cur_m >> u) & 1u) {
                below += (uint64_t)x;
                seg = 0;
                segmax = x;
                prev = 0;
            } else {
                seg += (uint64_t)x;
                segmax = x > segmax ? x : segmax;
                prev = x;
            }
        }
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            cur_d[u] = nxt_d[u];
            nxt_d[u] = far_d[u];
        }
        cur_m = nxt_m;
        nxt_m = bits(far_m);
    }
    op[last * opstride] = x0;
    ovf |= (total + (uint64_t)dmax) > (uint64_t)INT64_MAX;

    int32_t status = CKPT_OK;
    if (bad_size) status = CKPT_ERR_SIZE;
    else if (ovf) status = CKPT_ERR_OVERFLOW;
    else if (bad_mask) status = CKPT_ERR_MASK;
    if (status_out) status_out[c] = status;
    if (status != CKPT_OK)
        for (int64_t t = 0; t <= last; ++t) op[t * opstride] = -1;
}

// The timeline of chain c of a batch laid out by the strides (the lanes of a wave call it together).
// LDS_ROWS (Algorithm 2 only; `rows` is LDS for n x 64 words): the pass that adds up the checkpoints
// leaves row r >= 1 of each lane's chain in rows[r-1][lane] as size | mask << 31, and if every size
// of every chain of the wave is below 2^31 the walk reads the chain from there instead of from
// memory a second time.
template <int OBJ, bool LDS_ROWS>
__device__ __forceinline__ void eval_timeline_chain(const int64_t *__restrict__ d, const uint8_t *__restrict__ mask,
                                                    int64_t batch, int n, int64_t cstride, int64_t pstride,
                                                    int64_t *__restrict__ out, int64_t ocstride, int64_t opstride,
                                                    int32_t *__restrict__ status_out, const int64_t c, uint32_t *rows)
{
    static_assert(!LDS_ROWS || OBJ == CKPT_OBJ_STATIC, "only Algorithm 2 reads the chain twice");
    if (c >= batch) return;
    const int64_t *dp = d + c * cstride;
    const uint8_t *mp = mask + c * cstride;
    int64_t *op = out + c * ocstride;
    const int lane = threadIdx.x % kBlock;

    const int64_t x0 = dp[0];
    uint64_t ckpt_all = 0;  // sum of all checkpoints (Algorithm 2 only)
    bool narrow = true;
    if (OBJ == CKPT_OBJ_STATIC) {
        // both loads of a row are issued whatever the mask says, so that sixteen rows are in flight
#pragma unroll 16
        for (int k = 0; k <= n; ++k) {
            const uint8_t on = mp[(int64_t)k * pstride];
            const int64_t x = dp[(int64_t)k * pstride];
            ckpt_all += on ? (uint64_t)x : 0;
            if (LDS_ROWS && k >= 1) {
                rows[(k - 1) * kBlock + lane] = (uint32_t)x | (on ? 0x80000000u : 0u);
                narrow &= ((uint64_t)x >> 31) == 0;
            }
        }
    }
    const bool bad_mask = mp[0] == 0 || mp[(int64_t)n * pstride] == 0;
    auto ld_mem = [&](int r) -> int64_t { return dp[(int64_t)r * pstride]; };
    auto lm_mem = [&](int r) -> uint8_t { return mp[(int64_t)r * pstride]; };
    if (LDS_ROWS) {
        if (__builtin_amdgcn_ballot_w64(!narrow) == 0) {
            auto ld_lds = [&](int r) -> int64_t { return (int64_t)(rows[(r - 1) * kBlock + lane] & 0x7fffffffu); };
            auto lm_lds = [&](int r) -> uint8_t { return (uint8_t)(rows[(r - 1) * kBlock + lane] >> 31); };
            timeline_walk<OBJ>(ld_lds, lm_lds, n, x0, bad_mask, ckpt_all, op, opstride, status_out, c);
            return;
        }
    }
    timeline_walk<OBJ>(ld_mem, lm_mem, n, x0, bad_mask, ckpt_all, op, opstride, status_out, c);
}

template <int OBJ>
__global__ __launch_bounds__(kBlock) void eval_timeline_kernel(const int64_t *__restrict__ d,
                                                               const uint8_t *__restrict__ mask, int64_t batch,
                                                               int n, int64_t cstride, int64_t pstride,
                                                               int64_t *__restrict__ out, int64_t ocstride,
                                                               int64_t opstride, int32_t *__restrict__ status_out)
{
    const int64_t c = (int64_t)xcd_paired_block(blockIdx.x, gridDim.x) * kBlock + threadIdx.x;
    eval_timeline_chain<OBJ, false>(d, mask, batch, n, cstride, pstride, out, ocstride, opstride, status_out, c,
                                    nullptr);
}

// Algorithm 2 for chains short enough that a wave's 64 chains fit in LDS four times per CU (n words
// per lane, launched with n * 256 bytes of dynamic LDS): the chain is read from memory once.
extern __shared__ __align__(16) uint32_t timeline_rows[];
__global__ __launch_bounds__(kBlock) void eval_timeline_static_lds_kernel(const int64_t *__restrict__ d,
                                                                          const uint8_t *__restrict__ mask,
                                                                          int64_t batch, int n, int64_t cstride,
                                                                          int64_t pstride, int64_t *__restrict__ out,
                                                                          int64_t ocstride, int64_t opstride,
                                                                          int32_t *__restrict__ status_out)
{
    const int64_t c = (int64_t)xcd_paired_block(blockIdx.x, gridDim.x) * kBlock + threadIdx.x;
    eval_timeline_chain<CKPT_OBJ_STATIC, true>(d, mask, batch, n, cstride, pstride, out, ocstride, opstride, status_out,
                                               c, timeline_rows);
}

// Every group of a ragged call in one launch: a wave looks up the group its 64 chains belong to and
// writes their timelines (2n+2 rows, position-major) where the group's share of the wide staging
// lies, which is twice as far in as in the staging of the sizes.
template <int OBJ>
__global__ __launch_bounds__(kBlock) void eval_timeline_ragged_kernel(const int64_t *__restrict__ d_stage,
                                                                      const uint8_t *__restrict__ mask_stage,
                                                                      const RaggedGroupDev *__restrict__ groups,
                                                                      int n_groups, int64_t *__restrict__ wide_stage,
                                                                      int32_t *__restrict__ status_stage)
{
    const RaggedGroupDev g = groups[ragged_group_of_wave(groups, n_groups, blockIdx.x)];
    const int64_t c = ((int64_t)blockIdx.x - g.wave_first) * kBlock + threadIdx.x;
    eval_timeline_chain<OBJ, false>(d_stage + g.stage_off, mask_stage + g.stage_off, g.count, g.n, 1, g.pitch,
                                    wide_stage + 2 * g.stage_off, 1, g.pitch, status_stage + g.first, c, nullptr);
}

// Checkpoint sets that do not depend on the sizes: the two ends only, every
// position, or segments of ceil(sqrt(n)) layers (the sqrt(n) rule of Section
// 2.1 as Section 5 applies it: n = 24 gives {5,10,15,20,24}).  The byte of a
// position is the same for every chain, so with chains next to each other in
// memory (chain stride 1) a lane writes the bytes of PACK chains as one word.
template <int PACK>
__global__ __launch_bounds__(kBlock) void select_baseline_kernel(int64_t batch, int n, int64_t cstride,
                                                                 int64_t pstride, int kind, int seg_len,
                                                                 uint8_t *__restrict__ mask_out)
{
    const int64_t c = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * PACK;
    if (c >= batch) return;
    uint8_t *mp = mask_out + c * cstride;
    int next_multiple = 0;
    for (int k = 0; k <= n; ++k) {
        bool on = k == 0 || k == n || kind == CKPT_SELECT_ALL;
        if (k == next_multiple) {
            on |= kind == CKPT_SELECT_SQRT;
            next_multiple += seg_len;
        }
        if (PACK == 8)
            __builtin_nontemporal_store(on ? 0x0101010101010101ull : 0ull, (uint64_t *)(mp + (int64_t)k * pstride));
        else
            mp[(int64_t)k * pstride] = on ? 1 : 0;
    }
}

}  // namespace

hipError_t launch_eval_timeline(const int64_t *d, const uint8_t *mask, int64_t batch, int n, Strides st,
                                int objective, int64_t *out, Strides out_st, int32_t *status_out,
                                hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    const unsigned grid = (unsigned)((batch + kBlock - 1) / kBlock);
    if (objective == CKPT_OBJ_STATIC && n <= kLdsRowsMaxLayers)
        hipLaunchKernelGGL(eval_timeline_static_lds_kernel, dim3(grid), dim3(kBlock), (size_t)n * kBlock * 4, stream, d,
                           mask, batch, n, st.chain, st.pos, out, out_st.chain, out_st.pos, status_out);
    else if (objective == CKPT_OBJ_STATIC)
        hipLaunchKernelGGL(eval_timeline_kernel<CKPT_OBJ_STATIC>, dim3(grid), dim3(kBlock), 0, stream, d, mask,
                           batch, n, st.chain, st.pos, out, out_st.chain, out_st.pos, status_out);
    else
        hipLaunchKernelGGL(eval_timeline_kernel<CKPT_OBJ_DYNAMIC>, dim3(grid), dim3(kBlock), 0, stream, d, mask,
                           batch, n, st.chain, st.pos, out, out_st.chain, out_st.pos, status_out);
    return hipGetLastError();
}

hipError_t launch_eval_timeline_ragged(const int64_t *d_stage, const uint8_t *mask_stage,
                                       const RaggedGroupDev *groups, int n_groups, int64_t waves, int objective,
                                       int64_t *wide_stage, int32_t *status_stage, hipStream_t stream)
{
    if (waves == 0) return hipSuccess;
    static_assert(kBlock == kWave, "a workgroup is one of the groups' waves");
    if (objective == CKPT_OBJ_STATIC)
        hipLaunchKernelGGL(eval_timeline_ragged_kernel<CKPT_OBJ_STATIC>, dim3((unsigned)waves), dim3(kBlock), 0, stream,
                           d_stage, mask_stage, groups, n_groups, wide_stage, status_stage);
    else
        hipLaunchKernelGGL(eval_timeline_ragged_kernel<CKPT_OBJ_DYNAMIC>, dim3((unsigned)waves), dim3(kBlock), 0, stream,
                           d_stage, mask_stage, groups, n_groups, wide_stage, status_stage);
    return hipGetLastError();
}

hipError_t launch_select_baseline(int64_t batch, int n, Strides st, int kind, uint8_t *mask_out,
                                  hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    int seg_len = 1;  // ceil(sqrt(n))
    while ((int64_t)seg_len * seg_len < n) ++seg_len;
    // eight chains per lane when every row of eight bytes is contiguous and 8-byte aligned
    const bool packed = st.chain == 1 && batch % 8 == 0 && st.pos % 8 == 0 && ((uintptr_t)mask_out & 7u) == 0;
    if (packed) {
        const unsigned grid = (unsigned)((batch / 8 + kBlock - 1) / kBlock);
        hipLaunchKernelGGL(select_baseline_kernel<8>, dim3(grid), dim3(kBlock), 0, stream, batch, n, st.chain, st.pos,
                           kind, seg_len, mask_out);
    } else {
        const unsigned grid = (unsigned)((batch + kBlock - 1) / kBlock);
        hipLaunchKernelGGL(select_baseline_kernel<1>, dim3(grid), dim3(kBlock), 0, stream, batch, n, st.chain, st.pos,
                           kind, seg_len, mask_out);
    }
    return hipGetLastError();
}

}  // namespace ckpt
