// Linear-time dynamic checkpoint selection (Section 4.2: Equation (TU),
// Lemmas 1-4, Algorithm 6).
//
//   M(n) = d_n,   M(i) = d_i + min_{i<j<=n} max(M(j), U(i,j)),
//   U(i,j) = T(i) - T(j) + R(i,j),  T(k) = sum_{t>k} d_t,  R(i,j) = max_{i<=k<j} d_k.
//
// State per chain while i runs from n-1 down to 0:
//   Q    the monotone queue of Lemma 2 as a stack (pushes and pops happen at
//        the low-index end, the "head"): entries j with M(j) strictly
//        decreasing in j.  An entry keeps M(j) and A(j) = M(j) + T(j), so the
//        crossover test U(i,j) >= M(j) reads T(i) + R(i,j) >= A(j).
//   pt   the crossover entry: the lowest-index entry of Q with U(i,j) >= M(j).
//        U(i,.) increases with j (Lemma 1) and M decreases along Q, so the
//        entries from pt to the far end satisfy the test and the ones between
//        the head and pt do not; since U(i-1,j) > U(i,j) (Lemma 4) pt only
//        moves towards the head, and the entry at pt is never popped because
//        M(i) > U(i,j_pt) >= M(j_pt).  Entries beyond pt are dead.  The
//        minimum of Equation (TU) is at pt (value U(i,j_pt)) or at the entry
//        just before it, the "candidate" (value M); ties go to the lower index.
//   rec  the prefix-maximum records of d_i, d_{i+1}, ..: positions k whose d_k
//        exceeds everything between i and k, as a stack (top = i).  R(i,j) is
//        the value of the record with the largest k < j.  R for the pt entry
//        and for the candidate are kept in registers (R <- max(R, d_i) each
//        step); the stack is walked only when pt moves and a new candidate
//        needs its R: a range maximum cannot be undone when j moves left, the
//        walk over records can.  Records at or beyond j_pt are dead.
//   nxt  the chosen j for every i; the set is read off by following nxt from 0.
// Every entry enters and leaves each stack once and the pointers move one way
// between pushes, so the work per chain is O(n).
//
// Kernels:
//   ring kernel     one lane per chain, every chain of the batch.  Only the live
//        parts of the two stacks are kept, as 16-slot rings in LDS laid out
//        [slot][lane] (bank = lane).  Values are held as 32-bit multiples of
//        2^sh, sh the number of trailing zero bits common to the sizes read so
//        far (stored values are shifted left when a size with fewer trailing
//        zeros arrives).  nxt(i) - i - 1 is parked as a byte in the chain's
//        mask_out slot i and replaced by the mask in a final forward sweep.
//        A lane defers its chain to the list kernel when a ring fills, the
//        values outgrow 30 bits, a step exceeds 255 positions, or a size is not
//        positive: it appends the chain to a list in the workspace.
//   list kernel     one wave per deferred chain (lane 0 works), 64-bit values,
//        stacks of full capacity n+1 in LDS (n <= 2047) or in the workspace.
//        Correct for any input, and the only writer of error statuses.
#include "ckpt_internal.h"

namespace ckpt {
namespace {

constexpr int kRing = 16;        // slots per lane in each ring
constexpr int kChunk = 8;        // rows in flight per lane
constexpr int kListBlocks = 1024;
constexpr int kLdsStackMaxN = 2047;

struct LinearWs {
    int32_t *count;   // [1] number of deferred chains (first 256 bytes)
    int32_t *list;    // [batch]
    char *scratch;    // kListBlocks * stack_bytes(n)
};

// Full-capacity state of one chain: qM, qT, recD (int64), qJ, recK, nxt (int32), padded to 256 bytes.
__host__ __device__ inline size_t stack_bytes(int n) { return (((size_t)n + 1) * 36 + 255) / 256 * 256; }
__host__ __device__ inline size_t lds_stack_bytes(int n) { return ((size_t)n + 1) * 32; }

__host__ LinearWs carve_linear(void *ws, int64_t batch, int n)
{
    char *p = (char *)ws;
    LinearWs w;
    w.count = (int32_t *)p; p += 256;
    w.list = (int32_t *)p;  p += align_up((size_t)batch * 4);
    w.scratch = p;
    return w;
}

__global__ void linear_reset_kernel(LinearWs w) { *w.count = 0; }

// ---------------------------------------------------------------------------
// ring kernel
// ---------------------------------------------------------------------------

__global__ __launch_bounds__(kWave) void linear_ring_kernel(const int64_t *__restrict__ d, int64_t batch, int n,
                                                            int64_t cstride, int64_t pstride,
                                                            uint8_t *__restrict__ mask_out,
                                                            int64_t *__restrict__ peak_out,
                                                            int32_t *__restrict__ status_out, LinearWs w)
{
    __shared__ uint32_t qM[kRing][kWave];
    __shared__ uint32_t qA[kRing][kWave];
    __shared__ uint32_t recD[kRing][kWave];
    __shared__ uint16_t qJ[kRing][kWave];
    __shared__ uint16_t recK[kRing][kWave];

    const int lane = threadIdx.x;
    const int64_t c = (int64_t)blockIdx.x * kWave + lane;
    const bool live = c < batch;
    const int64_t cc = live ? c : batch - 1;  // idle lanes shadow the last chain and write nothing
    const int64_t *dp = d + cc * cstride;
    uint8_t *mp = mask_out + cc * cstride;
    constexpr int kMsk = kRing - 1;
    constexpr uint32_t kLimit = 1u << 30;

    const int64_t xn = dp[(int64_t)n * pstride];
    bool defer = xn <= 0;
    int sh = defer ? 0 : __ffsll((unsigned long long)xn) - 1;
    uint64_t xs = (uint64_t)xn >> sh;
    defer |= xs >= kLimit;

    // Q = {n}: it is the crossover entry (U(i,n) > d_n = M(n) for every i)
    int hd = 0, pt = 0;
    uint32_t Mhd = (uint32_t)xs;   // M of the head entry
    uint32_t Tpt = 0, Jpt = n;     // T(j_pt), j_pt
    uint32_t Rp = 0;               // R(i, j_pt)
    bool cand = false;             // is there an entry between pt and the head side, i.e. pt < hd
    uint32_t Mc = 0, Ac = 0, Jc = 0, Rc = 0;  // the candidate (entry pt+1): M, A, j, R(i, j)
    int top = -1;                  // records occupy rp..top
    int rp = 0x3fffffff, rc = 0x3fffffff;  // lowest record index with k < j_pt / k < j_c (clamped to top)
    uint32_t Ti = 0;               // T(i) / 2^sh
    uint32_t dnext = (uint32_t)xs; // d_{i+1} / 2^sh
    uint32_t dmax = dnext;
    uint32_t Mi = dnext;
    qM[0][lane] = Mhd;
    qA[0][lane] = Mhd;  // T(n) = 0
    qJ[0][lane] = (uint16_t)n;

    // One step of the recurrence for position i, whose size x is already in a register.
    auto step_fn = [&](const int i, const int64_t x) {
        defer |= x <= 0;
        // common trailing zeros: rescale everything held so far if this size has fewer
        const int tz = x > 0 ? __ffsll((unsigned long long)x) - 1 : sh;
        if (__any(tz < sh)) {
            if (tz < sh) {
                const int k = sh - tz;
                const bool fits = k < 30 && ((Ti + dnext + dmax) >> (30 - k)) == 0;
                defer |= !fits;
                const int kk = fits ? k : 0;
#pragma unroll
                for (int s = 0; s < kRing; ++s) {
                    qM[s][lane] <<= kk;
                    qA[s][lane] <<= kk;
                    recD[s][lane] <<= kk;
                }
                Mhd <<= kk; Tpt <<= kk; Rp <<= kk; Mc <<= kk; Ac <<= kk; Rc <<= kk;
                Ti <<= kk; dnext <<= kk; dmax <<= kk;
                sh = tz;
            }
        }
        xs = (uint64_t)x >> sh;
        defer |= xs >= kLimit;
        const uint32_t di = (uint32_t)xs;
        Ti += dnext;
        dmax = di > dmax ? di : dmax;
        defer |= (Ti + di + dmax) >= kLimit;  // bounds M(i) and every U(i,j)

        // records: d_i hides every record not larger than it; the top record is d_{i+1}
        if (top >= 0 && dnext <= di) {
            --top;
            while (top >= rp && (uint32_t)recD[top & kMsk][lane] <= di) --top;
        }
        ++top;
        recD[top & kMsk][lane] = di;
        recK[top & kMsk][lane] = (uint16_t)i;
        rp = rp < top ? rp : top;
        rc = rc < top ? rc : top;
        Rp = di > Rp ? di : Rp;
        Rc = di > Rc ? di : Rc;
        defer |= (top - rp) >= kRing;

        // move the crossover towards the head while the candidate satisfies U(i,j) >= M(j)
        while (cand && Ti + Rc >= Ac) {
            ++pt;
            Tpt = Ac - Mc; Jpt = Jc; Rp = Rc; rp = rc;
            cand = pt < hd;
            if (cand) {
                const int e = (pt + 1) & kMsk;
                Mc = (uint32_t)qM[e][lane];
                Ac = (uint32_t)qA[e][lane];
                Jc = qJ[e][lane];
                int r = rc;
                while (r < top && recK[r & kMsk][lane] >= Jc) ++r;  // the top record has k = i < j_c
                rc = r;
                Rc = (uint32_t)recD[r & kMsk][lane];
            }
        }
        const uint32_t Upt = Ti + Rp - Tpt;  // U(i, j_pt)
        const bool take_cand = cand && Mc <= Upt;
        const uint32_t best = take_cand ? Mc : Upt;
        const uint32_t nx = take_cand ? Jc : Jpt;
        Mi = di + best;
        const uint32_t step = nx - (uint32_t)i - 1u;
        defer |= step > 255u;
        if (live) mp[(int64_t)i * pstride] = (uint8_t)step;

        // Q: drop the entries that M(i) dominates (never the crossover entry), then push i
        if (hd > pt && Mhd >= Mi) {
            --hd;
            while (hd > pt && (uint32_t)qM[hd & kMsk][lane] >= Mi) --hd;
        }
        ++hd;
        qM[hd & kMsk][lane] = Mi;
        qA[hd & kMsk][lane] = Mi + Ti;
        qJ[hd & kMsk][lane] = (uint16_t)i;
        Mhd = Mi;
        defer |= (hd - pt) >= kRing;
        if (hd == pt + 1) {  // the new entry is the candidate; no record has k < i yet
            cand = true;
            Mc = Mi; Ac = Mi + Ti; Jc = (uint32_t)i; Rc = 0; rc = 0x3fffffff;
        }
        dnext = di;
    };

    // Rows are fetched kChunk positions ahead of their use, so that the HBM
    // latency of a row overlaps the work on the rows before it.
    int64_t rows[kChunk], ahead[kChunk];
#pragma unroll
    for (int u = 0; u < kChunk; ++u) rows[u] = (n - 1 - u) >= 0 ? dp[(int64_t)(n - 1 - u) * pstride] : 1;
    for (int ihi = n - 1; ihi >= 0; ihi -= kChunk) {
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const int k = ihi - kChunk - u;
            ahead[u] = k >= 0 ? dp[(int64_t)k * pstride] : 1;
        }
#pragma unroll
        for (int u = 0; u < kChunk; ++u)
            if (ihi - u >= 0) step_fn(ihi - u, rows[u]);
#pragma unroll
        for (int u = 0; u < kChunk; ++u) rows[u] = ahead[u];
    }
    defer |= sh > 32;  // results must fit 64 bits after shifting back

    if (!live) return;
    if (defer) {
        const int slot = atomicAdd(w.count, 1);
        w.list[slot] = (int32_t)c;
        return;
    }
    peak_out[c] = (int64_t)((uint64_t)Mi << sh);
    if (status_out) status_out[c] = CKPT_OK;
    // forward sweep: replace the parked steps by the mask
    int cur = 0;
    for (int k0 = 0; k0 <= n; k0 += kChunk) {
        uint8_t b[kChunk];
#pragma unroll
        for (int u = 0; u < kChunk; ++u) b[u] = (k0 + u) <= n ? mp[(int64_t)(k0 + u) * pstride] : 0;
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const int k = k0 + u;
            const bool on = k == cur;
            if (on) cur = k + 1 + b[u];
            b[u] = on ? 1 : 0;
        }
#pragma unroll
        for (int u = 0; u < kChunk; ++u)
            if ((k0 + u) <= n) mp[(int64_t)(k0 + u) * pstride] = b[u];
    }
}

// ---------------------------------------------------------------------------
// list kernel: one wave per deferred chain, full-capacity stacks, 64-bit
// ---------------------------------------------------------------------------

extern __shared__ __align__(16) unsigned char lin_lds[];

template <bool LDS_STACKS>
__global__ __launch_bounds__(kWave) void linear_list_kernel(const int64_t *__restrict__ d, int n, int64_t cstride,
                                                            int64_t pstride, uint8_t *__restrict__ mask_out,
                                                            int64_t *__restrict__ peak_out,
                                                            int32_t *__restrict__ status_out, LinearWs w)
{
    const int count = *w.count;
    const size_t n1 = (size_t)n + 1;
    char *base = w.scratch + (size_t)blockIdx.x * stack_bytes(n);
    int32_t *nxt = (int32_t *)(base + n1 * 32);
    if (LDS_STACKS) base = (char *)lin_lds;
    int64_t *qM = (int64_t *)base;
    int64_t *qT = qM + n1;
    int64_t *recD = qT + n1;
    int32_t *qJ = (int32_t *)(recD + n1);
    int32_t *recK = qJ + n1;

    for (int item = blockIdx.x; item < count; item += gridDim.x) {
        if (threadIdx.x != 0) continue;
        const int64_t c = w.list[item];
        const int64_t *dp = d + c * cstride;
        uint8_t *mp = mask_out + c * cstride;

        int64_t x = dp[(int64_t)n * pstride];
        bool bad_size = x <= 0;
        bool ovf = false;
        int64_t dmax = x;
        qJ[0] = n;
        qM[0] = x;
        qT[0] = 0;
        int hd = 0, pt = 0;    // Q occupies slots 0..hd, crossover at pt
        int top = -1, rp = 0;  // records occupy slots 0..top
        uint64_t T = 0;        // T(i)
        int64_t dnext = x;     // d_{i+1}
        int64_t Mi = x;

        for (int i = n - 1; i >= 0; --i) {
            const int64_t di = dp[(int64_t)i * pstride];
            bad_size |= di <= 0;
            dmax = di > dmax ? di : dmax;
            T += (uint64_t)dnext;
            ovf |= T > (uint64_t)INT64_MAX;
            dnext = di;
            if (bad_size | ovf) continue;  // keep scanning for errors, skip the work
            ovf |= (T + (uint64_t)di + (uint64_t)dmax) > (uint64_t)INT64_MAX;  // bounds M(i) and every U(i,j)
            if (ovf) continue;
            const int64_t Ti = (int64_t)T;

            while (top >= 0 && recD[top] <= di) --top;
            ++top;
            recD[top] = di;
            recK[top] = i;
            if (rp > top) rp = top;

            while (pt < hd) {
                const int e = pt + 1;
                const int je = qJ[e];
                int r = rp;
                while (recK[r] >= je) ++r;  // the top record has k = i < je
                if (Ti - qT[e] + recD[r] < qM[e]) break;
                pt = e;
                rp = r;
            }
            int64_t best = Ti - qT[pt] + recD[rp];  // U(i, j_pt)
            int nx = qJ[pt];
            if (pt < hd) {
                const int64_t Mp = qM[pt + 1];
                if (Mp <= best) {
                    best = Mp;
                    nx = qJ[pt + 1];
                }
            }
            Mi = di + best;
            nxt[i] = nx;

            while (hd > pt && qM[hd] >= Mi) --hd;
            ++hd;
            qJ[hd] = i;
            qM[hd] = Mi;
            qT[hd] = Ti;
        }
        ovf |= (T + (uint64_t)dnext + (uint64_t)dmax) > (uint64_t)INT64_MAX;  // sum(d) + max(d)

        int32_t status = CKPT_OK;
        if (bad_size) status = CKPT_ERR_SIZE;
        else if (ovf) status = CKPT_ERR_OVERFLOW;
        if (status_out) status_out[c] = status;
        peak_out[c] = status == CKPT_OK ? Mi : -1;
        if (status != CKPT_OK) {
            for (int k = 0; k <= n; ++k) mp[(int64_t)k * pstride] = 0;
            continue;
        }
        int cur = 0;
        for (int k = 0; k <= n; ++k) {
            const bool on = k == cur;
            mp[(int64_t)k * pstride] = on ? 1 : 0;
            if (on && k < n) cur = nxt[k];
        }
    }
}

}  // namespace

size_t linear_workspace_bytes(int64_t batch, int n)
{
    return 256 + align_up((size_t)batch * 4) + (size_t)kListBlocks * stack_bytes(n) + 256;
}

hipError_t launch_solve_linear(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                               int64_t *peak_out, int32_t *status_out, void *ws, hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    LinearWs w = carve_linear(ws, batch, n);
    const unsigned grid = (unsigned)((batch + kWave - 1) / kWave);
    hipLaunchKernelGGL(linear_reset_kernel, dim3(1), dim3(1), 0, stream, w);
    hipLaunchKernelGGL(linear_ring_kernel, dim3(grid), dim3(kWave), 0, stream, d, batch, n, st.chain, st.pos,
                       mask_out, peak_out, status_out, w);
    const unsigned lgrid = (unsigned)(batch < kListBlocks ? batch : kListBlocks);
    if (n <= kLdsStackMaxN)
        hipLaunchKernelGGL(linear_list_kernel<true>, dim3(lgrid), dim3(kWave), lds_stack_bytes(n), stream, d, n,
                           st.chain, st.pos, mask_out, peak_out, status_out, w);
    else
        hipLaunchKernelGGL(linear_list_kernel<false>, dim3(lgrid), dim3(kWave), 0, stream, d, n, st.chain, st.pos,
                           mask_out, peak_out, status_out, w);
    return hipGetLastError();
}

}  // namespace ckpt
