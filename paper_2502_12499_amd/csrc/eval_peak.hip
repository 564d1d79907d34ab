// Peak memory of a given checkpoint set (Equation (cost), Section 3.1, and
// Equation (memory), Section 4), one lane per chain.
//
// The kernel is a single streaming pass: per chain it reads 8(n+1) bytes of
// sizes and (n+1) bytes of mask and writes 8 bytes.  With the position-major
// layout the 64 lanes of a wave read 512 contiguous bytes of sizes and 64 of
// mask per position; the loop is unrolled so that several rows are in flight
// per wave.  All state is a handful of 64-bit registers per lane.
#include "ckpt_internal.h"

namespace ckpt {
namespace {

constexpr int kBlock = 64;

// The evaluation of chain c of a batch laid out by (cstride, pstride).  OBJ = CKPT_OBJ_BOTH keeps
// the running values of both objectives and writes the dynamic peak `second` values after the
// static one.
template <int OBJ>
__device__ __forceinline__ void eval_peak_chain(const int64_t *__restrict__ d, const uint8_t *__restrict__ mask,
                                       int64_t batch, int n, int64_t cstride, int64_t pstride,
                                       int64_t *__restrict__ peak_out, int32_t *__restrict__ status_out,
                                       const int64_t c, const int64_t second)
{
    if (c >= batch) return;
    const int64_t *dp = d + c * cstride;
    const uint8_t *mp = mask + c * cstride;

    // Position 0 is the input: always resident, start of the first segment.
    int64_t x0 = dp[0];
    bool bad_size = x0 <= 0;
    bool bad_mask = mp[0] == 0;
    uint64_t total = (uint64_t)x0;
    bool ovf = false;
    int64_t dmax = x0;

    int64_t ckpt_sum = x0;  // sum of checkpoints seen so far
    int64_t seg_sum = 0;    // sum of non-checkpoints since the last checkpoint
    int64_t seg_max = x0;   // max over d_h..d_{k-1}, h the last checkpoint (Equation (memory))
    int64_t best = 0;       // Equation (cost): largest segment, else Equation (memory): largest m(i)
    int64_t best_dyn = 0;   // the latter when both are wanted
    uint8_t last_mask = 1;
    constexpr bool kStatic = OBJ == CKPT_OBJ_STATIC || OBJ == CKPT_OBJ_BOTH;
    constexpr bool kDynamic = OBJ == CKPT_OBJ_DYNAMIC || OBJ == CKPT_OBJ_BOTH;

#pragma unroll 16
    for (int k = 1; k <= n; ++k) {
        const int64_t x = __builtin_nontemporal_load(dp + (int64_t)k * pstride);
        const uint8_t m = __builtin_nontemporal_load(mp + (int64_t)k * pstride);
        bad_size |= x <= 0;
        total += (uint64_t)x;
        ovf |= total > (uint64_t)INT64_MAX;
        dmax = x > dmax ? x : dmax;
        last_mask = m;
        if (m) {
            ckpt_sum += x;
            if (kStatic) best = seg_sum > best ? seg_sum : best;
            if (kDynamic) {
                const int64_t mi = ckpt_sum + seg_sum + seg_max;
                if (OBJ == CKPT_OBJ_BOTH)
                    best_dyn = mi > best_dyn ? mi : best_dyn;
                else
                    best = mi > best ? mi : best;
                seg_max = x;
            }
            seg_sum = 0;
        } else {
            seg_sum += x;
            if (kDynamic) seg_max = x > seg_max ? x : seg_max;
        }
    }
    bad_mask |= last_mask == 0;
    ovf |= (total + (uint64_t)dmax) > (uint64_t)INT64_MAX;

    int32_t status = CKPT_OK;
    if (bad_size) status = CKPT_ERR_SIZE;
    else if (ovf) status = CKPT_ERR_OVERFLOW;
    else if (bad_mask) status = CKPT_ERR_MASK;

    int64_t peak = kStatic ? ckpt_sum + best : best;
    peak_out[c] = status == CKPT_OK ? peak : -1;
    if (OBJ == CKPT_OBJ_BOTH) peak_out[second + c] = status == CKPT_OK ? best_dyn : -1;
    if (status_out) status_out[c] = status;
}

template <int OBJ>
__global__ __launch_bounds__(kBlock) void eval_peak_kernel(const int64_t *__restrict__ d,
                                                           const uint8_t *__restrict__ mask,
                                                           int64_t batch, int n, int64_t cstride,
                                                           int64_t pstride,
                                                           int64_t *__restrict__ peak_out,
                                                           int32_t *__restrict__ status_out)
{
    const int64_t c = (int64_t)xcd_paired_block(blockIdx.x, gridDim.x) * kBlock + threadIdx.x;
    eval_peak_chain<OBJ>(d, mask, batch, n, cstride, pstride, peak_out, status_out, c, batch);
}

// Every group of a ragged call in one launch: a wave looks up the group its 64 chains belong to
// and evaluates them where that group is staged; results go to the chains' places (with both
// objectives the dynamic peaks `batch` values, the number of chains of all groups, further on).
template <int OBJ>
__global__ __launch_bounds__(kBlock) void eval_peak_ragged_kernel(const int64_t *__restrict__ d_stage,
                                                                  const uint8_t *__restrict__ mask_stage,
                                                                  const RaggedGroupDev *__restrict__ groups,
                                                                  int n_groups, int64_t batch,
                                                                  int64_t *__restrict__ peak_stage,
                                                                  int32_t *__restrict__ status_stage)
{
    const RaggedGroupDev g = groups[ragged_group_of_wave(groups, n_groups, blockIdx.x)];
    const int64_t c = ((int64_t)blockIdx.x - g.wave_first) * kBlock + threadIdx.x;
    eval_peak_chain<OBJ>(d_stage + g.stage_off, mask_stage + g.stage_off, g.count, g.n, 1, g.pitch,
                         peak_stage + g.first, status_stage + g.first, c, batch);
}

}  // namespace

hipError_t launch_eval_peak(const int64_t *d, const uint8_t *mask, int64_t batch, int n, Strides st,
                            int objective, int64_t *peak_out, int32_t *status_out, hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    const unsigned grid = (unsigned)((batch + kBlock - 1) / kBlock);
    if (objective == CKPT_OBJ_STATIC)
        hipLaunchKernelGGL(eval_peak_kernel<CKPT_OBJ_STATIC>, dim3(grid), dim3(kBlock), 0, stream, d, mask,
                           batch, n, st.chain, st.pos, peak_out, status_out);
    else if (objective == CKPT_OBJ_DYNAMIC)
        hipLaunchKernelGGL(eval_peak_kernel<CKPT_OBJ_DYNAMIC>, dim3(grid), dim3(kBlock), 0, stream, d, mask,
                           batch, n, st.chain, st.pos, peak_out, status_out);
    else
        hipLaunchKernelGGL(eval_peak_kernel<CKPT_OBJ_BOTH>, dim3(grid), dim3(kBlock), 0, stream, d, mask,
                           batch, n, st.chain, st.pos, peak_out, status_out);
    return hipGetLastError();
}

hipError_t launch_eval_peak_ragged(const int64_t *d_stage, const uint8_t *mask_stage, const RaggedGroupDev *groups,
                                   int n_groups, int64_t waves, int64_t batch, int objective, int64_t *peak_stage,
                                   int32_t *status_stage, hipStream_t stream)
{
    if (waves == 0) return hipSuccess;
    static_assert(kBlock == kWave, "a workgroup is one of the groups' waves");
    if (objective == CKPT_OBJ_STATIC)
        hipLaunchKernelGGL(eval_peak_ragged_kernel<CKPT_OBJ_STATIC>, dim3((unsigned)waves), dim3(kBlock), 0, stream,
                           d_stage, mask_stage, groups, n_groups, batch, peak_stage, status_stage);
    else if (objective == CKPT_OBJ_DYNAMIC)
        hipLaunchKernelGGL(eval_peak_ragged_kernel<CKPT_OBJ_DYNAMIC>, dim3((unsigned)waves), dim3(kBlock), 0, stream,
                           d_stage, mask_stage, groups, n_groups, batch, peak_stage, status_stage);
    else
        hipLaunchKernelGGL(eval_peak_ragged_kernel<CKPT_OBJ_BOTH>, dim3((unsigned)waves), dim3(kBlock), 0, stream,
                           d_stage, mask_stage, groups, n_groups, batch, peak_stage, status_stage);
    return hipGetLastError();
}

}  // namespace ckpt
