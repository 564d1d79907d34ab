// Quadratic-time dynamic checkpoint selection (Section 4.1: Equation (T-rec),
// Algorithm 5, Theorem 2), one wave per chain:
//
//   M(n) = d_n,   M(i) = d_i + min_{i<j<=n} max(M(j), U(i,j)),
//   U(i,j) = P[j] - P[i] + R(i,j),  P the prefix sums,  R(i,j) = max_{i<=k<j} d_k.
//
// The recurrence is sequential in i; for one i the candidates j are
// independent, so the 64 lanes take j = i+1+lane, i+65+lane, ...  Each lane
// keeps the best of its own candidates (ascending j, strict "<", so the
// smallest j among equals), then the wave takes the minimum value with row
// shifts and row broadcasts (DPP) and, among the lanes that hold it, the
// smallest j: that is the canonical next(i) of the linear-time solver, which
// this kernel cross-checks with none of its machinery (no queue, no crossover
// pointer).  R(i,j) is kept per j and raised to max(R, d_i) as i moves down,
// which is Algorithm 5's accumulation of s(i,j) turned around.
//
// State per chain in LDS: P, M, R (int64) and next (uint16) over 0..n, i.e.
// 26(n+1) bytes, which bounds n (CKPT_QUADRATIC_MAX_LAYERS).  Work per chain
// is n(n+1)/2 candidate evaluations on one wave: the kernel suits single
// chains and small batches, where a lane-per-chain kernel leaves the machine
// idle; on large batches the linear-time kernel is far ahead.
#include "ckpt_internal.h"

namespace ckpt {
namespace {

extern __shared__ __align__(16) unsigned char quad_lds[];

// UNROLL: candidates per lane loaded together (1 for short chains, whose lanes have at most
// a couple of candidates each; 4 hides the LDS latency on long ones).
template <int UNROLL>
__global__ __launch_bounds__(kWave) void quadratic_kernel(const int64_t *__restrict__ d, int64_t batch, int n,
                                                          int64_t cstride, int64_t pstride,
                                                          uint8_t *__restrict__ mask_out,
                                                          int64_t *__restrict__ peak_out,
                                                          int64_t *__restrict__ value_out,
                                                          int32_t *__restrict__ status_out)
{
    const int lane = threadIdx.x;
    const int n1 = n + 1;
    uint64_t *P = (uint64_t *)quad_lds;
    uint64_t *M = P + n1;
    uint64_t *R = M + n1;
    uint16_t *nxt = (uint16_t *)(R + n1);

    for (int64_t c = blockIdx.x; c < batch; c += gridDim.x) {
        const int64_t *dp = d + c * cstride;
        uint8_t *mp = mask_out + c * cstride;

        // prefix sums 64 positions at a time (inclusive scan by row shifts, carry in `base`),
        // validation on the way; R starts empty
        uint64_t base = 0, dmax = 0;
        bool bad_size = false, ovf = false;
        for (int k0 = 0; k0 < n1; k0 += kWave) {
            const int k = k0 + lane;
            const int64_t x = k < n1 ? dp[(int64_t)k * pstride] : 0;
            bad_size |= k < n1 && x <= 0;
            dmax = (uint64_t)x > dmax && x > 0 ? (uint64_t)x : dmax;
            uint64_t incl = x > 0 ? (uint64_t)x : 0;
#pragma unroll
            for (int dlt = 1; dlt < kWave; dlt <<= 1) {
                const uint64_t o = (uint64_t)__shfl_up((long long)incl, dlt, kWave);
                const bool oo = __shfl_up((int)ovf, dlt, kWave);
                if (lane >= dlt) {
                    incl += o;
                    ovf |= oo | (incl > (uint64_t)INT64_MAX);
                }
            }
            incl += base;
            ovf |= incl > (uint64_t)INT64_MAX;  // all terms positive: a wrap shows as > INT64_MAX first
            if (k < n1) {
                P[k] = incl;
                R[k] = 0;
            }
            base = (uint64_t)__shfl((long long)incl, kWave - 1, kWave);
            ovf = __shfl((int)ovf, kWave - 1, kWave);
        }
        dmax = ~wave_min_u64(~dmax);
        ovf |= (base + dmax) > (uint64_t)INT64_MAX;
        bad_size = __builtin_amdgcn_ballot_w64(bad_size) != 0;
        ovf = __builtin_amdgcn_ballot_w64(ovf) != 0;

        int32_t status = CKPT_OK;
        if (bad_size) status = CKPT_ERR_SIZE;
        else if (ovf) status = CKPT_ERR_OVERFLOW;
        if (status != CKPT_OK) {
            for (int k = lane; k < n1; k += kWave) {
                mp[(int64_t)k * pstride] = 0;
                if (value_out) value_out[c * cstride + (int64_t)k * pstride] = -1;
            }
            if (lane == 0) {
                peak_out[c] = -1;
                if (status_out) status_out[c] = status;
            }
            continue;
        }

        __syncthreads();
        if (lane == 0) {
            M[n] = P[n] - (n > 0 ? P[n - 1] : 0);
            nxt[n] = (uint16_t)n;
        }
        __syncthreads();
        uint64_t Pi = P[n - 1 >= 0 ? n - 1 : 0];
        for (int i = n - 1; i >= 0; --i) {
            const uint64_t Pbelow = i > 0 ? P[i - 1] : 0;  // also the next step's P[i]
            const uint64_t di = Pi - Pbelow;
            uint64_t best = ~0ull;
            uint32_t bestj = 0xffffffffu;
            // UNROLL candidates per lane at a time, all loads before the first store
            constexpr int kUnroll = UNROLL;
            for (int j0 = i + 1 + lane; j0 <= n; j0 += kUnroll * kWave) {
                uint64_t r[kUnroll], pj[kUnroll], m[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int j = min(j0 + u * kWave, n);  // beyond n: row n again, not used
                    r[u] = R[j];
                    pj[u] = P[j];
                    m[u] = M[j];
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int j = j0 + u * kWave;
                    if (j > n) break;
                    const uint64_t rr = di > r[u] ? di : r[u];
                    R[j] = rr;
                    const uint64_t uij = pj[u] - Pi + rr;  // U(i, j)
                    const uint64_t v = m[u] > uij ? m[u] : uij;
                    if (v < best) {
                        best = v;
                        bestj = (uint32_t)j;
                    }
                }
            }
            const uint64_t vmin = wave_min_u64(best);
            const uint32_t jmin = wave_min_u32(best == vmin ? bestj : 0xffffffffu);
            if (lane == 0) {
                M[i] = di + vmin;
                nxt[i] = (uint16_t)jmin;
            }
            Pi = Pbelow;
            __syncthreads();  // one wave per block: orders the lane's write before the others' reads
        }

        // outputs: the value function, and the set by following next from 0 (marked in LDS by
        // one lane over the no longer needed R, then written out by all)
        uint8_t *on = (uint8_t *)R;
        for (int k = lane; k < n1; k += kWave) {
            if (value_out) value_out[c * cstride + (int64_t)k * pstride] = (int64_t)M[k];
            on[k] = 0;
        }
        __syncthreads();
        if (lane == 0) {
            peak_out[c] = (int64_t)M[0];
            if (status_out) status_out[c] = CKPT_OK;
            int i = 0;
            on[0] = 1;
            while (i < n) {
                i = nxt[i];
                on[i] = 1;
            }
        }
        __syncthreads();
        for (int k = lane; k < n1; k += kWave) mp[(int64_t)k * pstride] = on[k];
        __syncthreads();  // the next chain reuses the arrays
    }
}

}  // namespace

size_t quadratic_lds_bytes(int n) { return ((size_t)n + 1) * 26 + 16; }

hipError_t launch_solve_quadratic(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                                  int64_t *peak_out, int64_t *value_out, int32_t *status_out, hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    const size_t lds = quadratic_lds_bytes(n);
    if (lds > 65536) {  // beyond the default limit for dynamic LDS
        const hipError_t e = hipFuncSetAttribute((const void *)quadratic_kernel<4>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    // enough waves to fill the machine several times over; each walks its share of the batch
    const int64_t cap = 256 * 32;
    const dim3 grid((unsigned)(batch < cap ? batch : cap));
    if (n <= 2 * kWave)
        hipLaunchKernelGGL(quadratic_kernel<1>, grid, dim3(kWave), lds, stream, d, batch, n, st.chain, st.pos,
                           mask_out, peak_out, value_out, status_out);
    else
        hipLaunchKernelGGL(quadratic_kernel<4>, grid, dim3(kWave), lds, stream, d, batch, n, st.chain, st.pos,
                           mask_out, peak_out, value_out, status_out);
    return hipGetLastError();
}

}  // namespace ckpt
