// Linear-time dynamic checkpoint selection (Section 4.2: Equation (TU),
// Lemmas 1-4, Algorithm 6), one lane per chain.
//
//   M(n) = d_n,   M(i) = d_i + min_{i<j<=n} max(M(j), U(i,j)),
//   U(i,j) = T(i) - T(j) + R(i,j),  T(k) = sum_{t>k} d_t,  R(i,j) = max_{i<=k<j} d_k.
//
// State per chain while i runs from n-1 down to 0:
//   Q    the monotone queue of Lemma 2 as a stack (pushes and pops happen at
//        the low-index end): entries (j, M(j), T(j)), M strictly decreasing
//        with j.  Slot 0 holds j = n.
//   pt   the crossover entry: the lowest-index entry of Q with U(i,j) >= M(j).
//        U(i,.) increases with j and M decreases along Q, so the entries at or
//        beyond pt satisfy the inequality and the ones before it do not; by
//        U(i-1,j) > U(i,j) (Lemma 4) pt only ever moves towards the low-index
//        end, and the entry at pt is never popped because M(i) > U(i,j_pt) >=
//        M(j_pt).  The minimum of Equation (TU) is at pt (value U(i,j_pt)) or
//        at the entry just before it (value M); ties go to the lower index.
//   rec  the prefix-maximum records of d_i, d_{i+1}, ...: positions k with d_k
//        larger than everything between i and k, as a stack (top = i).  R(i,j)
//        is the value of the record with the largest k < j; rp is that record
//        for j = j_pt.  This is what makes "U(i,j') from U(i,j)" exact when j
//        moves left: a range maximum cannot be undone, the record walk can.
//   nxt  the chosen j for every i; the set is read off by following nxt from 0.
//
// Every entry enters and leaves each stack once and pt, rp only move one way
// between pushes, so the work per chain is O(n).
//
// This kernel keeps the stacks in the caller's workspace (slot-major, chain
// contiguous, so that lanes at equal depth coalesce) with full capacity n+1:
// it is correct for any input.
#include "ckpt_internal.h"

namespace ckpt {
namespace {

constexpr int kBlock = 64;

struct LinearWs {
    int64_t *qM;
    int64_t *qT;
    int64_t *recD;
    int32_t *qJ;
    int32_t *recK;
    int32_t *nxt;
};

__host__ __device__ inline size_t linear_slots(int64_t batch, int n) { return (size_t)batch * ((size_t)n + 1); }

__host__ LinearWs carve_linear(void *ws, int64_t batch, int n)
{
    char *p = (char *)ws;
    const size_t slots = linear_slots(batch, n);
    LinearWs w;
    w.qM = (int64_t *)p;   p += align_up(slots * 8);
    w.qT = (int64_t *)p;   p += align_up(slots * 8);
    w.recD = (int64_t *)p; p += align_up(slots * 8);
    w.qJ = (int32_t *)p;   p += align_up(slots * 4);
    w.recK = (int32_t *)p; p += align_up(slots * 4);
    w.nxt = (int32_t *)p;
    return w;
}

__global__ __launch_bounds__(kBlock) void linear_general_kernel(const int64_t *__restrict__ d, int64_t batch,
                                                                int n, int64_t cstride, int64_t pstride,
                                                                uint8_t *__restrict__ mask_out,
                                                                int64_t *__restrict__ peak_out,
                                                                int32_t *__restrict__ status_out, LinearWs w)
{
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c >= batch) return;
    const int64_t *dp = d + c * cstride;
    uint8_t *mp = mask_out + c * cstride;
    // stack slot s of this chain
    auto at = [&](int s) -> int64_t { return (int64_t)s * batch + c; };

    int64_t x = dp[(int64_t)n * pstride];
    bool bad_size = x <= 0;
    bool ovf = false;
    int64_t dmax = x;

    // Q = {n}
    w.qJ[at(0)] = n;
    w.qM[at(0)] = x;
    w.qT[at(0)] = 0;
    int hd = 0, pt = 0;   // Q occupies slots 0..hd, crossover at pt
    int top = -1, rp = 0; // records occupy slots 0..top
    uint64_t T = 0;       // T(i)
    int64_t dnext = x;    // d_{i+1}
    int64_t Mi = x;

    for (int i = n - 1; i >= 0; --i) {
        const int64_t di = dp[(int64_t)i * pstride];
        bad_size |= di <= 0;
        dmax = di > dmax ? di : dmax;
        T += (uint64_t)dnext;
        ovf |= T > (uint64_t)INT64_MAX;
        dnext = di;
        if (bad_size | ovf) continue;  // keep scanning for errors, skip the work
        const int64_t Ti = (int64_t)T;

        // records: d_i hides every record not larger than it
        while (top >= 0 && w.recD[at(top)] <= di) --top;
        ++top;
        w.recD[at(top)] = di;
        w.recK[at(top)] = i;
        if (rp > top) rp = top;

        // move the crossover towards the low-index end while U(i,j) >= M(j)
        while (pt < hd) {
            const int e = pt + 1;
            const int je = w.qJ[at(e)];
            int r = rp;
            while (w.recK[at(r)] >= je) ++r;  // the top record has k = i < je
            const int64_t Ue = Ti - w.qT[at(e)] + w.recD[at(r)];
            if (Ue < w.qM[at(e)]) break;
            pt = e;
            rp = r;
        }
        int64_t best = Ti - w.qT[at(pt)] + w.recD[at(rp)];  // U(i, j_pt)
        int nx = w.qJ[at(pt)];
        if (pt < hd) {
            const int64_t Mp = w.qM[at(pt + 1)];
            if (Mp <= best) {
                best = Mp;
                nx = w.qJ[at(pt + 1)];
            }
        }
        Mi = di + best;
        w.nxt[at(i)] = nx;

        // Q: drop the entries that M(i) dominates, then push i
        while (hd > pt && w.qM[at(hd)] >= Mi) --hd;
        ++hd;
        w.qJ[at(hd)] = i;
        w.qM[at(hd)] = Mi;
        w.qT[at(hd)] = Ti;
    }
    // sum(d) + max(d) must be representable: T(0) + d_0 is sum(d)
    ovf |= (T + (uint64_t)dnext) > (uint64_t)INT64_MAX;
    ovf |= (T + (uint64_t)dnext + (uint64_t)dmax) > (uint64_t)INT64_MAX;

    int32_t status = CKPT_OK;
    if (bad_size) status = CKPT_ERR_SIZE;
    else if (ovf) status = CKPT_ERR_OVERFLOW;
    if (status_out) status_out[c] = status;
    peak_out[c] = status == CKPT_OK ? Mi : -1;

    if (status != CKPT_OK) {
        for (int k = 0; k <= n; ++k) mp[(int64_t)k * pstride] = 0;
        return;
    }
    int cur = 0;
    for (int k = 0; k <= n; ++k) {
        const bool on = k == cur;
        mp[(int64_t)k * pstride] = on ? 1 : 0;
        if (on && k < n) cur = w.nxt[at(k)];
    }
}

}  // namespace

size_t linear_workspace_bytes(int64_t batch, int n)
{
    const size_t slots = linear_slots(batch, n);
    return 3 * align_up(slots * 8) + 3 * align_up(slots * 4) + 256;
}

hipError_t launch_solve_linear(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                               int64_t *peak_out, int32_t *status_out, void *ws, hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    LinearWs w = carve_linear(ws, batch, n);
    const unsigned grid = (unsigned)((batch + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(linear_general_kernel, dim3(grid), dim3(kBlock), 0, stream, d, batch, n, st.chain,
                       st.pos, mask_out, peak_out, status_out, w);
    return hipGetLastError();
}

}  // namespace ckpt
