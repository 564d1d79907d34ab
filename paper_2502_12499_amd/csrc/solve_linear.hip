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
//   R    the range maximum cannot be undone when j moves left (the paper's
//        "U(i,j') from U(i,j)"), so it is kept exactly in another form: every
//        entry carries G = max of d from its own position up to the next entry
//        towards the far end (fixed when the entry is pushed: the front maximum
//        joined with the G of the entries it replaced), and R(i,j) of an entry
//        is the maximum of d since the head was pushed ("front") joined with
//        the G of the entries above it.  R of the pt entry and of the candidate
//        live in registers (R <- max(R, d_i) each step); the join over the
//        entries above is only taken when pt moves and a new candidate needs
//        its R.  (The general kernel below uses the stack of prefix-maximum
//        records of d_i, d_{i+1}, .. for the same purpose.)
//   nxt  the chosen j for every i; the set is read off by following nxt from 0.
// Every entry enters and leaves each stack once and the pointers move one way
// between pushes, so the work per chain is O(n).
//
// Kernels:
//   ring kernel     one lane per chain, every chain of the batch.  Only the live
//        part of the stack is kept, as a 16-slot ring in LDS laid out
//        [slot][lane].  Values are held as 32-bit multiples of
//        2^sh, sh the number of trailing zero bits common to the sizes read so
//        far (stored values are shifted left when a size with fewer trailing
//        zeros arrives).  nxt(i) - i - 1 is a byte: chains of up to 256 layers
//        keep these bytes in vector registers (the same register for every
//        lane, indexed by the wave-uniform position); longer chains park them in
//        the chain's mask_out slot i.  A final forward sweep turns them into the mask.
//        A lane defers its chain when a ring fills, the values outgrow 30 bits,
//        a step exceeds 255 positions, or a size is not positive: it appends
//        the chain to a list in the workspace.
//   wide kernel     one lane per chain on that list: the same algorithm in
//        64-bit arithmetic with plain loops (sizes that are not multiples of a
//        large power of two end up here).  Chains it cannot take either (ring
//        full, step beyond 255, sizes not positive, sums beyond 64 bits) go on
//        a second list.
//   list kernel     one wave per chain of the second list (lane 0 works),
//        64-bit values, stacks of full capacity n+1 in LDS (n <= 2047) or in
//        the workspace.  Correct for any input, and the only writer of error
//        statuses.
#include "ckpt_internal.h"

#include <atomic>

namespace ckpt {
namespace {

constexpr int kRing = 16;        // slots per lane in each ring
constexpr int kChunk = 8;        // rows in flight per lane
constexpr int kListBlocks = 1024;
constexpr int kLdsStackMaxN = 2047;

struct LinearWs {
    int32_t *count;   // [2] chains deferred by the ring kernel, chains deferred again by the wide kernel
                      // (first 256 bytes)
    int32_t *list;    // [batch] the former
    int32_t *list2;   // [batch] the latter
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
    w.list2 = (int32_t *)p; p += align_up((size_t)batch * 4);
    w.scratch = p;
    return w;
}

__global__ void linear_reset_kernel(LinearWs w) { w.count[0] = 0; w.count[1] = 0; }

// Puts every chain on the first deferred list (layouts the ring kernel does not address).
__global__ void linear_defer_all_kernel(int64_t batch, LinearWs w)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c < batch) w.list[c] = (int32_t)c;
    if (c == 0) w.count[0] = (int32_t)batch;
}

// Largest chain stride (elements) for which 63 strides of 8-byte elements fit a 32-bit offset.
constexpr int64_t kRingMaxChainStride = (int64_t)1 << 22;

// ---------------------------------------------------------------------------
// ring kernel
// ---------------------------------------------------------------------------

// A ring entry is three words, each in a plane of its own laid out [slot][lane]
// (so the 64 lanes of a wave always hit 64 different words of a plane, whatever
// slot each of them is at: no bank conflicts):
//   M    M(j)
//   A    M(j) + T(j)
//   GJ   G << 8 | (j & 255), G = max of d over [j, j'), j' the next entry towards the
//        far end.  A maximum over such words orders by G first, which is all the
//        folds below need; the low byte of j is enough because a step is at most
//        255 positions (checked per chunk), and a byte is what gets stored of it.
constexpr int kPlaneM = 0, kPlaneA = 1, kPlaneGJ = 2, kPlanes = 3;

// LOG_REGS (chains of at most kLogMaxLayers layers): the chosen step of every position is kept as a
// byte in 64 vector registers per lane (two per chunk of eight positions, written and read with a
// wave-uniform register index) instead of being parked in the caller's mask array: nothing but
// the sizes is read and nothing but the mask written.
constexpr int kLogMaxLayers = 256;
typedef uint32_t u32x32 __attribute__((ext_vector_type(32)));

// `block` of `grid`: which 64 chains of the batch the wave takes; `list_base` is added to a
// chain's number when it goes on the deferred list (the place of the batch's first chain among
// all chains of a ragged call, else 0); `ring`: the wave's 12 KB of LDS.
template <bool LOG_REGS>
__device__ __forceinline__ void linear_ring_wave(const int64_t *__restrict__ d, int64_t batch, int n, int64_t cstride,
                                        int64_t pstride, uint8_t *__restrict__ mask_out,
                                        int64_t *__restrict__ peak_out, int32_t *__restrict__ status_out,
                                        const LinearWs &w, const unsigned block, const unsigned grid,
                                        const int64_t list_base, uint32_t (&ring)[kPlanes][kRing][kWave])
{
    // Ring positions are kept pre-multiplied by the byte stride of a slot, so
    // the LDS address of a position is one AND-OR away (the ring is aligned to
    // its own size; the kernel declares it, aligned to 4096 bytes, and hands it in).
    constexpr uint32_t kStep = (uint32_t)(kWave * sizeof(uint32_t));  // bytes from a slot to the next
    constexpr uint32_t kSlotMask = (uint32_t)(kRing - 1) * kStep;
    constexpr uint32_t kPlane = (uint32_t)kRing * kStep;              // bytes from a plane to the next
    constexpr int kA = kPlaneA * (int)(kPlane / 4), kGJ = kPlaneGJ * (int)(kPlane / 4);  // in words
    constexpr uint32_t kNone = 0xffffffffu;  // "no candidate": never passes a test
    static_assert(kPlane == 4096, "plane size and alignment");
    // What the assembly hard-codes: the literal plane offsets 4096 and 8192 of its LDS reads, a
    // ring aligned to a plane so that an address is (position & mask) | lane base, steps and
    // positions that fit the low byte of a GJ word, and lane offsets of the rows that fit 31 bits.
    static_assert(kPlanes == 3 && kRing == 16 && kWave == 64 && kStep == 256, "ring geometry in the assembly");
    static_assert(sizeof(ring) == 3 * 4096 && (kSlotMask & (kStep - 1)) == 0, "ring size and slot mask");
    static_assert(63 * kRingMaxChainStride * 8 < ((int64_t)1 << 31), "32-bit lane offsets");

    const int lane = threadIdx.x;
    const int64_t c0 = (int64_t)xcd_paired_block(block, grid) * kWave;
    const int64_t c = c0 + lane;
    const bool live = c < batch;
    const int64_t cc = live ? c : batch - 1;  // idle lanes shadow the last chain and write nothing
    // Addresses are a wave-uniform base (scalar registers) plus a 32-bit lane offset: the
    // launcher only takes this kernel when 63 chain strides fit 31 bits.
    const char *dbase = (const char *)(d + c0 * cstride);
    uint8_t *mbase = mask_out + c0 * cstride;
    const uint32_t doff = (uint32_t)((cc - c0) * cstride) * 8u;
    const uint32_t moff = (uint32_t)((cc - c0) * cstride);
    // a wave-uniform 64-bit value, moved to scalar registers
    auto scalar = [](uint64_t a) -> uint64_t {
        return ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32)) << 32) |
               (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    };
    auto row = [&](int k) -> int64_t {  // k is the same in every lane: the row's base stays scalar
        const int ks = __builtin_amdgcn_readfirstlane(k);
        return *(const int64_t *)(dbase + (int64_t)ks * pstride * 8 + doff);
    };
    uint8_t *mp = mask_out + cc * cstride;
    constexpr uint32_t kLimit = 1u << 30;       // bound on T(i) + d_i + max d, hence on every M(i) and U(i,j)
    constexpr uint32_t kChunkLimit = 1u << 24;  // bound on a single size (it shares a word with a byte of j)

    typedef __attribute__((address_space(3))) uint32_t *LdsPtr;
    const uint32_t lane_base = (uint32_t)(uintptr_t)(LdsPtr)&ring[kPlaneM][0][lane];
    auto entry = [&](uint32_t pos) -> LdsPtr { return (LdsPtr)(uintptr_t)((pos & kSlotMask) | lane_base); };

    const int64_t xn = row(n);
    bool defer = xn <= 0;
    int sh = defer ? 0 : __ffsll((unsigned long long)xn) - 1;
    sh = sh < 31 ? sh : 31;  // so that a size's low word alone says whether it is a multiple of 2^sh
    uint64_t xs = (uint64_t)xn >> sh;
    defer |= xs >= kChunkLimit;

    // Q = {n}: it is the crossover entry (U(i,n) > d_n = M(n) for every i)
    uint32_t hd = 0, pt = 0;                   // ring positions of the head and of the crossover entry
    uint32_t Mhd = (uint32_t)xs, Ghd = 0;      // M and GJ of the head entry
    // (M, GJ) of the three entries under the head, read back after every push so
    // that the steps that follow find them in registers (what lies beyond the
    // crossover entry is never looked at, so it does not matter what they hold there)
    uint32_t M1 = 0, G1 = 0, M2 = 0, G2 = 0, M3 = 0, G3 = 0, M4 = 0, G4 = 0;
    uint32_t Tpt = 0, Jpt = n, Rp = 0;         // crossover entry: T(j), j (only its low byte is kept up), R(i, j)
    uint32_t Jfull = n;                        // its position in full, as of the last chunk check
    uint32_t Mc = kNone, Ac = kNone, Jc = 0, Rc = 0;  // candidate (the entry before pt): M, A, j, R(i, j)
    uint32_t Ti = 0;                           // T(i) / 2^sh
    uint32_t dnext = (uint32_t)xs;             // d_{i+1} / 2^sh
    uint32_t dmax = dnext;                     // a bound on the sizes so far (below twice the largest)
    uint32_t Mi = dnext;
    {
        LdsPtr e = entry(0);
        e[0] = Mhd; e[kA] = Mhd; e[kGJ] = (uint32_t)n & 255u;  // T(n) = 0, nothing beyond n
    }

    // Range and alignment are settled for kChunk rows at a time, before their steps, and a
    // lane that cannot go on is switched off for good (its chain goes on the deferred list):
    // the lanes that run a step hold exact values, which is what ends the loops below and
    // keeps the stack's entries in order.
    // `all` is the OR of the rows (so its trailing zeros are the fewest of theirs and its
    // magnitude bounds each of them; a negative size shows as a huge one), `zero` says that
    // one of them is 0, `ilow` is the lowest position of the chunk.
    auto chunk_check = [&](const uint64_t all, const bool zero, const int ilow) {
        const uint32_t low = (uint32_t)all & ((1u << sh) - 1u);
        if (__builtin_amdgcn_ballot_w64(low != 0) != 0) {
            if (low != 0) {
                // fewer common trailing zeros: rescale everything held so far
                const int tz = __ffs(low) - 1;
                const int k = sh - tz;
                const bool fits = k < 30 && ((Ti + dnext + dmax) >> (30 - k)) == 0;
                defer |= !fits;
                const int kk = fits ? k : 0;
                auto scale_gj = [kk](uint32_t gj) -> uint32_t { return ((gj & ~255u) << kk) | (gj & 255u); };
#pragma unroll
                for (int t = 0; t < kRing; ++t) {
                    LdsPtr e = entry((uint32_t)t * kStep);
                    e[0] <<= kk; e[kA] <<= kk; e[kGJ] = scale_gj(e[kGJ]);
                }
                Mhd <<= kk; Ghd = scale_gj(Ghd); Tpt <<= kk; Rp <<= kk; Rc <<= kk;
                M1 <<= kk; G1 = scale_gj(G1); M2 <<= kk; G2 = scale_gj(G2); M3 <<= kk; G3 = scale_gj(G3);
                M4 <<= kk; G4 = scale_gj(G4);
                Mc = Mc == kNone ? kNone : Mc << kk;
                Ac = Ac == kNone ? kNone : Ac << kk;
                Ti <<= kk; dnext <<= kk; dmax <<= kk;
                sh = tz;
            }
        }
        // sizes positive and below 2^24, T(i) + d + max d below 2^30 now: no sum of this chunk wraps
        const uint64_t scaled = all >> sh;
        defer |= zero | (scaled >= kChunkLimit);
        dmax = (uint32_t)scaled > dmax ? (uint32_t)scaled : dmax;
        defer |= (Ti + dnext + dmax) >= kLimit;
        // The crossover entry's position in full from its low byte: it has not moved up since the
        // last check and lies above the last chunk's lowest position, fewer than 256 places in all.
        // Every step of this chunk is at most j_pt - i - 1 of its lowest position: one byte holds it.
        Jfull -= (Jfull - Jpt) & 255u;
        defer |= (Jfull - (uint32_t)ilow) > 248u;
    };

    u32x32 logA = {}, logB = {};   // LOG_REGS: the steps of chunk k as bytes of logA[k] (u = 0..3) and logB[k] (u = 4..7)
    uint32_t acc0 = 0, acc1 = 0;   // ... of the chunk under way
    // One step of the recurrence for position i = ihi - u, whose size x is already in a register.
    auto step_fn = [&](const int i, const int64_t x, const int u) {
        const uint32_t di = __builtin_amdgcn_alignbit((uint32_t)((uint64_t)x >> 32), (uint32_t)x, (uint32_t)sh);
        const uint32_t di8 = di << 8;  // as a GJ word
        Ti += dnext;
        Rp = di > Rp ? di : Rp;
        Rc = di > Rc ? di : Rc;

        // Move the crossover towards the head while the candidate satisfies
        // U(i,j) >= M(j).  A new candidate's R is the front maximum joined with the
        // G of the entries above it.  Runs while ANY lane has to move; lanes that
        // are done sit out under the exec mask.  (In assembly: the compiler's
        // lowering of this doubly nested divergent loop is several times longer.)
        {
            uint32_t ad, e, t0;
            uint64_t sv, sv2, sv3;
            asm volatile(
                "Lw_%=:\n\t"
                "v_add_u32 %[t0], %[Ti], %[Rc]\n\t"
                "v_cmp_ge_u32 vcc, %[t0], %[Ac]\n\t"
                "s_cbranch_vccz Lw_done_%=\n\t"
                "s_and_saveexec_b64 %[sv], vcc\n\t"
                "v_add_u32 %[pt], %[step], %[pt]\n\t"
                "v_sub_u32 %[Tpt], %[Ac], %[Mc]\n\t"
                "v_mov_b32 %[Jpt], %[Jc]\n\t"
                "v_mov_b32 %[Rp], %[Rc]\n\t"
                "v_mov_b32 %[Ac], -1\n\t"
                "v_mov_b32 %[Mc], -1\n\t"
                "v_cmp_ne_u32 vcc, %[pt], %[hd]\n\t"
                "s_and_saveexec_b64 %[sv2], vcc\n\t"
                // the new candidate, and its R from the G of the entries above it
                // (as GJ words; the shift at the end takes the byte of j off again):
                // the head's and the three under it are in registers
                "s_mov_b64 %[sv3], exec\n\t"
                "v_add_u32 %[e], %[step], %[pt]\n\t"
                "v_and_or_b32 %[ad], %[e], %[mask], %[lo]\n\t"
                "ds_read_b32 %[Mc], %[ad]\n\t"
                "ds_read_b32 %[Ac], %[ad] offset:4096\n\t"
                "ds_read_b32 %[Jc], %[ad] offset:8192\n\t"
                "v_sub_u32 %[t0], %[hd], %[e]\n\t"
                "v_mov_b32 %[Rc], %[di8]\n\t"
                "v_cmp_le_u32 vcc, %[step], %[t0]\n\t"
                "s_and_b64 exec, exec, vcc\n\t"
                "v_max_u32 %[Rc], %[Rc], %[Ghd]\n\t"
                "v_cmp_le_u32 vcc, 2*%[step], %[t0]\n\t"
                "s_and_b64 exec, exec, vcc\n\t"
                "v_max_u32 %[Rc], %[Rc], %[G1]\n\t"
                "v_cmp_le_u32 vcc, 3*%[step], %[t0]\n\t"
                "s_and_b64 exec, exec, vcc\n\t"
                "v_max_u32 %[Rc], %[Rc], %[G2]\n\t"
                "v_cmp_le_u32 vcc, 4*%[step], %[t0]\n\t"
                "s_and_b64 exec, exec, vcc\n\t"
                "v_max_u32 %[Rc], %[Rc], %[G3]\n\t"
                // more than four entries above it (rare: one test for the whole wave): the rest from the ring
                "v_cmp_le_u32 vcc, 5*%[step], %[t0]\n\t"
                "s_cbranch_vccz Lg_done_%=\n\t"
                "v_subrev_u32 %[e], 3*%[step], %[hd]\n\t"
                "Lg_%=:\n\t"
                "v_subrev_u32 %[e], %[step], %[e]\n\t"
                "v_sub_u32 %[t0], %[e], %[pt]\n\t"
                "v_cmp_lt_u32 vcc, %[step], %[t0]\n\t"
                "s_and_b64 exec, exec, vcc\n\t"
                "s_cbranch_execz Lg_done_%=\n\t"
                "v_and_or_b32 %[ad], %[e], %[mask], %[lo]\n\t"
                "ds_read_b32 %[t0], %[ad] offset:8192\n\t"
                "s_waitcnt lgkmcnt(0)\n\t"
                "v_max_u32 %[Rc], %[Rc], %[t0]\n\t"
                "s_branch Lg_%=\n\t"
                "Lg_done_%=:\n\t"
                "s_mov_b64 exec, %[sv3]\n\t"
                "v_lshrrev_b32 %[Rc], 8, %[Rc]\n\t"
                "s_mov_b64 exec, %[sv2]\n\t"
                "s_waitcnt lgkmcnt(0)\n\t"
                "s_mov_b64 exec, %[sv]\n\t"
                "s_branch Lw_%=\n\t"
                "Lw_done_%=:\n\t"
                : [pt] "+v"(pt), [Tpt] "+v"(Tpt), [Jpt] "+v"(Jpt), [Rp] "+v"(Rp), [Mc] "+v"(Mc), [Ac] "+v"(Ac),
                  [Jc] "+v"(Jc), [Rc] "+v"(Rc), [ad] "=&v"(ad), [e] "=&v"(e), [t0] "=&v"(t0), [sv] "=&s"(sv),
                  [sv2] "=&s"(sv2), [sv3] "=&s"(sv3)
                : [Ti] "v"(Ti), [hd] "v"(hd), [di8] "v"(di8), [Ghd] "v"(Ghd), [G1] "v"(G1), [G2] "v"(G2), [G3] "v"(G3),
                  [lo] "v"(lane_base), [mask] "s"(kSlotMask), [step] "i"(kStep)
                : "vcc", "scc", "memory");  // (s_and_saveexec writes SCC)
        }
        const uint32_t Upt = Ti + Rp - Tpt;  // U(i, j_pt)
        const bool take_cand = Mc <= Upt;    // ties go to the lower index; kNone never wins
        const uint32_t best = take_cand ? Mc : Upt;
        const uint32_t nx = take_cand ? Jc : Jpt;
        Mi = di + best;
        const uint32_t step = nx - (uint32_t)i - 1u;
        // Parked with a store the compiler does not count, so that its waits on the
        // rows fetched ahead stay partial (a counted store would make it wait for
        // everything in flight; an uncounted one can only lengthen a wait).
        if constexpr (LOG_REGS) {
            // the step's low byte into byte u % 4 of the chunk's word (u is a literal once unrolled)
            const uint32_t sel = 0x03020100u ^ ((0x04u ^ (uint32_t)(u & 3)) << (8 * (u & 3)));
            if (u < 4)
                acc0 = __builtin_amdgcn_perm(step, acc0, sel);
            else
                acc1 = __builtin_amdgcn_perm(step, acc1, sel);
        } else if (live) {
            const uint64_t rowbase = scalar((uint64_t)(uintptr_t)(mbase + (int64_t)i * pstride));
            // The compiler may form the scalar base with v_readfirstlane right before this
            // statement; a vector memory instruction must not read such a register within five
            // wait states, and the compiler does not look inside the statement: wait here.
            asm volatile("s_nop 4\n\tglobal_store_byte %0, %1, %2" : : "v"(moff), "v"(step), "s"(rowbase) : "memory");
        }

        // Q: drop the entries that M(i) dominates (never the crossover entry),
        // folding their G into the new entry's, then push i
        uint32_t Gacc = di8;  // a GJ word: only its G part is used
        {
            // up to three drops are decided on the mirrors.  The crossover entry is never
            // dropped, M(i) being above its value, and the tests are nested, so what the
            // mirrors hold beyond it is never looked at.
            const bool p0 = Mhd >= Mi;
            const bool p1 = p0 & (M1 >= Mi);
            const bool p2 = p1 & (M2 >= Mi);
            const bool p3 = p2 & (M3 >= Mi);
            Gacc = p0 ? (Ghd > Gacc ? Ghd : Gacc) : Gacc;
            Gacc = p1 ? (G1 > Gacc ? G1 : Gacc) : Gacc;
            Gacc = p2 ? (G2 > Gacc ? G2 : Gacc) : Gacc;
            hd -= p0 ? kStep : 0u;
            hd -= p1 ? kStep : 0u;
            hd -= p2 ? kStep : 0u;
            if (__builtin_amdgcn_ballot_w64(p3) != 0) {
                // more: the third mirror goes too, and the lanes concerned go on with the fourth (the
                // others fail the first test), then from the ring, one at a time, down to the
                // crossover entry at the latest.
                Gacc = p3 ? (G3 > Gacc ? G3 : Gacc) : Gacc;
                hd -= p3 ? kStep : 0u;
                Mhd = p3 ? M4 : 0u;
                Ghd = G4;
                uint32_t ad;
                uint64_t sv;
                asm volatile(
                    "Lq_%=:\n\t"
                    "v_cmp_ge_u32 vcc, %[Mhd], %[Mi]\n\t"
                    "s_cbranch_vccz Lq_done_%=\n\t"
                    "s_and_saveexec_b64 %[sv], vcc\n\t"
                    "v_max_u32 %[G], %[G], %[Ghd]\n\t"
                    "v_subrev_u32 %[hd], %[step], %[hd]\n\t"
                    "v_and_or_b32 %[ad], %[hd], %[mask], %[lo]\n\t"
                    "ds_read_b32 %[Mhd], %[ad]\n\t"
                    "ds_read_b32 %[Ghd], %[ad] offset:8192\n\t"
                    "s_waitcnt lgkmcnt(0)\n\t"
                    "s_mov_b64 exec, %[sv]\n\t"
                    "s_branch Lq_%=\n\t"
                    "Lq_done_%=:\n\t"
                    : [hd] "+v"(hd), [Mhd] "+v"(Mhd), [Ghd] "+v"(Ghd), [G] "+v"(Gacc), [ad] "=&v"(ad), [sv] "=&s"(sv)
                    : [Mi] "v"(Mi), [lo] "v"(lane_base), [mask] "s"(kSlotMask), [step] "i"(kStep)
                    : "vcc", "scc", "memory");  // (s_and_saveexec writes SCC)
            }
        }
        // a ring that is full keeps its entries: the chain is deferred and the new entry
        // takes the head's slot, so that the lane's stack stays in order for the rest of the chunk
        const bool full = (hd - pt) >= (uint32_t)(kRing - 1) * kStep;
        defer |= full;
        hd += full ? 0u : kStep;
        {
            Gacc = (Gacc & ~255u) | ((uint32_t)i & 255u);
            LdsPtr e = entry(hd);
            e[0] = Mi; e[kA] = Mi + Ti; e[kGJ] = Gacc;
        }
        Mhd = Mi;
        Ghd = Gacc;
        {
            LdsPtr e1 = entry(hd - kStep), e2 = entry(hd - 2 * kStep), e3 = entry(hd - 3 * kStep);
            M1 = e1[0]; G1 = e1[kGJ];
            M2 = e2[0]; G2 = e2[kGJ];
            M3 = e3[0]; G3 = e3[kGJ];
            LdsPtr e4 = entry(hd - 4 * kStep);
            M4 = e4[0]; G4 = e4[kGJ];
        }
        const bool fresh = hd == pt + kStep;  // the new entry is the candidate; R(i', i) starts empty
        Mc = fresh ? Mi : Mc;
        Ac = fresh ? Mi + Ti : Ac;
        Jc = fresh ? (uint32_t)i : Jc;
        Rc = fresh ? 0u : Rc;
        dnext = di;
    };

    // Rows are fetched kChunk positions ahead of their use, so that the HBM
    // latency of a row overlaps the work on the rows before it.
    int64_t rows[kChunk], ahead[kChunk];
#pragma unroll
    for (int u = 0; u < kChunk; ++u) rows[u] = row(max(n - 1 - u, 0));
    int chunk = 0;
    for (int ihi = n - 1; ihi >= 0; ihi -= kChunk, ++chunk) {
#pragma unroll
        for (int u = 0; u < kChunk; ++u)  // rows below 0 re-read row 0 and are not used
            ahead[u] = row(max(ihi - kChunk - u, 0));
        uint64_t all = 0;
        bool zero = false;
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const uint64_t x = (uint64_t)rows[u];  // a row below 0 holds row 0 again: harmless here
            all |= x;
            zero |= x == 0;
        }
        if (!defer) chunk_check(all, zero, max(ihi - kChunk + 1, 0));
        if (!defer) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u)
                if (ihi - u >= 0) step_fn(ihi - u, rows[u], u);
            if constexpr (LOG_REGS) {
                const int k = __builtin_amdgcn_readfirstlane(chunk);
                logA[k] = acc0;
                logB[k] = acc1;
                acc0 = 0;
                acc1 = 0;
            }
        }
#pragma unroll
        for (int u = 0; u < kChunk; ++u) rows[u] = ahead[u];
    }

    if (!live) return;
    if (defer) {
        const int slot = atomicAdd(w.count, 1);
        w.list[slot] = (int32_t)(c + list_base);
        return;
    }
    peak_out[c] = (int64_t)((uint64_t)Mi << sh);
    if (status_out) status_out[c] = CKPT_OK;
    if constexpr (LOG_REGS) {
        // forward sweep over the steps in the registers: position i = n-1 - (8k + u), ascending.
        // Rows are addressed by a scalar base that moves up one row per position, plus the lane's
        // offset; only the first chunk taken (the last one filled) can reach below position 0.
        int cur = 0;
        auto sweep_chunk = [&](const int ks, const bool guarded) {
            const uint32_t w0 = logA[ks], w1 = logB[ks];
            const int ilow = n - 1 - (kChunk * ks + kChunk - 1);  // the chunk's lowest position (below 0 if guarded)
            uint8_t *rowp = mbase + (int64_t)ilow * pstride;      // wave-uniform; one row up per position
#pragma unroll
            for (int u = kChunk - 1; u >= 0; --u, rowp += pstride) {
                const int i = ilow + (kChunk - 1 - u);
                if (guarded && i < 0) continue;
                const uint32_t step = ((u < 4 ? w0 : w1) >> (8 * (u & 3))) & 255u;
                const bool on = i == cur;
                cur = on ? i + 1 + (int)step : cur;
                rowp[moff] = on ? 1 : 0;
            }
        };
        int k = chunk - 1;
        if (k >= 0) sweep_chunk(__builtin_amdgcn_readfirstlane(k), true);
        for (--k; k >= 0; --k) sweep_chunk(__builtin_amdgcn_readfirstlane(k), false);
        mp[(int64_t)n * pstride] = 1;
        return;
    }
    // forward sweep: replace the parked steps by the mask (once they have all landed)
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
    int cur = 0;
    constexpr int kSweep = 32;  // rows in flight per lane in this sweep, which does nothing but wait for them
    for (int k0 = 0; k0 <= n; k0 += kSweep) {
        uint8_t b[kSweep];
#pragma unroll
        for (int u = 0; u < kSweep; ++u) b[u] = (k0 + u) <= n ? mp[(int64_t)(k0 + u) * pstride] : 0;
#pragma unroll
        for (int u = 0; u < kSweep; ++u) {
            const int k = k0 + u;
            const bool on = k == cur;
            if (on) cur = k + 1 + b[u];
            b[u] = on ? 1 : 0;
        }
#pragma unroll
        for (int u = 0; u < kSweep; ++u)
            if ((k0 + u) <= n) mp[(int64_t)(k0 + u) * pstride] = b[u];
    }
}

template <bool LOG_REGS>
__global__ __launch_bounds__(kWave) void linear_ring_kernel(const int64_t *__restrict__ d, int64_t batch, int n,
                                                            int64_t cstride, int64_t pstride,
                                                            uint8_t *__restrict__ mask_out,
                                                            int64_t *__restrict__ peak_out,
                                                            int32_t *__restrict__ status_out, LinearWs w)
{
    __shared__ __attribute__((aligned(4096))) uint32_t ring[kPlanes][kRing][kWave];
    linear_ring_wave<LOG_REGS>(d, batch, n, cstride, pstride, mask_out, peak_out, status_out, w, blockIdx.x,
                               gridDim.x, 0, ring);
}

// Every group of a ragged call in one launch: a wave looks up the group its 64 chains belong to
// and solves them where that group is staged, with the step log in registers if the group's
// chains have up to kLogMaxLayers layers (a wave-uniform branch: long and short groups run side by
// side on the chip).  Results go to the chains' places.
__global__ __launch_bounds__(kWave) void linear_ring_ragged_kernel(const int64_t *__restrict__ d_stage,
                                                                   const RaggedGroupDev *__restrict__ groups,
                                                                   int n_groups, uint8_t *__restrict__ mask_stage,
                                                                   int64_t *__restrict__ peak_stage,
                                                                   int32_t *__restrict__ status_stage, LinearWs w)
{
    __shared__ __attribute__((aligned(4096))) uint32_t ring[kPlanes][kRing][kWave];
    const RaggedGroupDev g = groups[ragged_group_of_wave(groups, n_groups, blockIdx.x)];
    const unsigned waves = (unsigned)((g.count + kWave - 1) / kWave);
    const unsigned block = blockIdx.x - (unsigned)g.wave_first;
    if (g.n <= kLogMaxLayers)
        linear_ring_wave<true>(d_stage + g.stage_off, g.count, g.n, 1, g.pitch, mask_stage + g.stage_off,
                               peak_stage + g.first, status_stage + g.first, w, block, waves, g.first, ring);
    else
        linear_ring_wave<false>(d_stage + g.stage_off, g.count, g.n, 1, g.pitch, mask_stage + g.stage_off,
                                peak_stage + g.first, status_stage + g.first, w, block, waves, g.first, ring);
}

// ---------------------------------------------------------------------------
// wide kernel: one lane per chain deferred by the ring kernel, 64-bit values
// ---------------------------------------------------------------------------

struct alignas(32) WideEntry {
    int64_t M;   // M(j)
    int64_t G;   // max of d over [j, j'), j' the next entry towards the far end
    int64_t A;   // M(j) + T(j)
    int32_t J;   // j
    int32_t pad;
};

constexpr int kWideBlocks = 2048;

// The ring kernel's algorithm again, in 64-bit arithmetic and with plain loops,
// for the chains whose values did not fit 32 bits there.  The lanes of a wave
// take listed chains and walk i together.  A chain with a size that is not
// positive, with sums beyond 64 bits, with more than kRing live entries or with
// a step beyond 255 positions goes on to the list kernel.
// With `groups` (a ragged call) a listed number is a chain's place among all chains: its group
// gives the length, where the chain is staged and where its results go, per lane.
__global__ __launch_bounds__(kWave) void linear_wide_kernel(const int64_t *__restrict__ d, int n_all,
                                                            int64_t cstride, int64_t pstride_all,
                                                            uint8_t *__restrict__ mask_out,
                                                            int64_t *__restrict__ peak_out,
                                                            int32_t *__restrict__ status_out, LinearWs w,
                                                            const RaggedGroupDev *__restrict__ groups, int n_groups)
{
    __shared__ WideEntry ring[kRing][kWave];
    const int lane = threadIdx.x;
    const int count = w.count[0];
    for (int item0 = blockIdx.x * kWave; item0 < count; item0 += gridDim.x * kWave) {
        const bool live = item0 + lane < count;
        const int64_t c = w.list[live ? item0 + lane : count - 1];  // the number results are filed under
        int n = n_all;
        int64_t pstride = pstride_all;
        const int64_t *dp = d + c * cstride;
        uint8_t *mp = mask_out + c * cstride;
        if (groups) {
            const RaggedGroupDev g = groups[ragged_group_of_place(groups, n_groups, c)];
            n = g.n;
            pstride = g.pitch;
            dp = d + g.stage_off + (c - g.first);
            mp = mask_out + g.stage_off + (c - g.first);
        }
        auto at = [&](int pos) -> WideEntry & { return ring[pos & (kRing - 1)][lane]; };

        int64_t x = dp[(int64_t)n * pstride];
        bool out = x <= 0;  // no longer this kernel's chain
        int64_t dmax = x, dnext = x, Mi = x;
        uint64_t T = 0;
        int hd = 0, pt = 0;
        at(0) = WideEntry{x, 0, x, n, 0};
        int64_t Tpt = 0, Rp = 0;
        int Jpt = n;
        bool has_c = false;
        int64_t Mc = 0, Ac = 0, Rc = 0;
        int Jc = 0;

        for (int i = n - 1; i >= 0; --i) {
            const int64_t di = dp[(int64_t)i * pstride];
            out |= di <= 0;
            dmax = di > dmax ? di : dmax;
            T += (uint64_t)dnext;
            dnext = di;
            out |= T > (uint64_t)INT64_MAX;
            if (!out) out |= (T + (uint64_t)di + (uint64_t)dmax) > (uint64_t)INT64_MAX;  // bounds M(i), every U(i,j)
            if (out) continue;
            const int64_t Ti = (int64_t)T;
            Rp = di > Rp ? di : Rp;
            Rc = di > Rc ? di : Rc;
            // the crossover moves towards the head while the candidate satisfies U(i,j) >= M(j)
            while (has_c && Ti + Rc >= Ac) {
                ++pt;
                Tpt = Ac - Mc;
                Jpt = Jc;
                Rp = Rc;
                has_c = pt != hd;
                if (has_c) {
                    const WideEntry e = at(pt + 1);
                    Mc = e.M; Ac = e.A; Jc = e.J;
                    Rc = di;  // joined with the G of the entries above the new candidate
                    for (int q = pt + 2; q <= hd; ++q) {
                        const int64_t g = at(q).G;
                        Rc = g > Rc ? g : Rc;
                    }
                }
            }
            const int64_t Upt = Ti + Rp - Tpt;  // U(i, j_pt)
            const bool take = has_c && Mc <= Upt;  // ties go to the lower index
            Mi = di + (take ? Mc : Upt);
            const int step = (take ? Jc : Jpt) - i - 1;
            out |= step > 255;
            if (live) mp[(int64_t)i * pstride] = (uint8_t)step;
            // Q: drop the entries that M(i) dominates (never the crossover entry), then push i
            int64_t Gacc = di;
            while (hd > pt && at(hd).M >= Mi) {
                const int64_t g = at(hd).G;
                Gacc = g > Gacc ? g : Gacc;
                --hd;
            }
            ++hd;
            out |= hd - pt >= kRing;
            at(hd) = WideEntry{Mi, Gacc, Mi + Ti, i, 0};
            if (hd == pt + 1) {
                has_c = true;
                Mc = Mi; Ac = Mi + Ti; Jc = i; Rc = 0;
            }
        }
        if (!live) continue;
        if (out) {
            w.list2[atomicAdd(w.count + 1, 1)] = (int32_t)c;
            continue;
        }
        peak_out[c] = Mi;
        if (status_out) status_out[c] = CKPT_OK;
        // forward sweep: replace the parked steps by the mask
        __threadfence_block();
        int cur = 0;
        for (int k = 0; k <= n; ++k) {
            uint8_t *q = mp + (int64_t)k * pstride;
            const bool on = k == cur;
            if (on) cur = k + 1 + *q;
            *q = on ? 1 : 0;
        }
    }
}

// ---------------------------------------------------------------------------
// list kernel: one wave per deferred chain, full-capacity stacks, 64-bit
// ---------------------------------------------------------------------------

extern __shared__ __align__(16) unsigned char lin_lds[];

// n_all: the chains' length, or in a ragged call (`groups`) the longest one, for which the stacks
// are laid out; a listed number is then a chain's place among all chains, as in the wide kernel.
template <bool LDS_STACKS>
__global__ __launch_bounds__(kWave) void linear_list_kernel(const int64_t *__restrict__ d, int n_all,
                                                            int64_t cstride, int64_t pstride_all,
                                                            uint8_t *__restrict__ mask_out,
                                                            int64_t *__restrict__ peak_out,
                                                            int32_t *__restrict__ status_out, LinearWs w,
                                                            const RaggedGroupDev *__restrict__ groups, int n_groups)
{
    const int count = w.count[1];
    const size_t n1 = (size_t)n_all + 1;
    char *base = w.scratch + (size_t)blockIdx.x * stack_bytes(n_all);
    int32_t *nxt = (int32_t *)(base + n1 * 32);
    if (LDS_STACKS) base = (char *)lin_lds;
    int64_t *qM = (int64_t *)base;
    int64_t *qT = qM + n1;
    int64_t *recD = qT + n1;
    int32_t *qJ = (int32_t *)(recD + n1);
    int32_t *recK = qJ + n1;

    for (int item = blockIdx.x; item < count; item += gridDim.x) {
        if (threadIdx.x != 0) continue;
        const int64_t c = w.list2[item];
        int n = n_all;
        int64_t pstride = pstride_all;
        const int64_t *dp = d + c * cstride;
        uint8_t *mp = mask_out + c * cstride;
        if (groups) {
            const RaggedGroupDev g = groups[ragged_group_of_place(groups, n_groups, c)];
            n = g.n;
            pstride = g.pitch;
            dp = d + g.stage_off + (c - g.first);
            mp = mask_out + g.stage_off + (c - g.first);
        }

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
    return 256 + 2 * align_up((size_t)batch * 4) + (size_t)kListBlocks * stack_bytes(n) + 256;
}

// ---------------------------------------------------------------------------
// the call that allocates nothing: the lists live in an array of the library's own
// ---------------------------------------------------------------------------

// Up to CKPT_NOALLOC_MAX_LAYERS layers the list kernel keeps its stacks in LDS, so the
// scratch is the two counters and the two lists of chain indices only.
constexpr size_t kNoallocScratchBytes = 256 + 2 * ((size_t)CKPT_NOALLOC_MAX_BATCH * 4) + 256;
static_assert(CKPT_NOALLOC_MAX_LAYERS <= kLdsStackMaxN, "the list kernel must not need scratch stacks");

namespace {
// One copy per GPU, at an address of its own on each; held until the process ends.
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_of_device[kMaxDevices];
}  // namespace

hipError_t launch_solve_linear_noalloc(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                                       int64_t *peak_out, int32_t *status_out, hipStream_t stream)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    // The array's name is a host-side stand-in; its device address is looked up once per
    // device, with that device current (two threads that race here store the same address).
    void *ptr = scratch_of_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        scratch_of_device[dev].store(ptr, std::memory_order_release);
    }
    return launch_solve_linear(d, batch, n, st, mask_out, peak_out, status_out, ptr, stream);
}

hipError_t launch_solve_linear(const int64_t *d, int64_t batch, int n, Strides st, uint8_t *mask_out,
                               int64_t *peak_out, int32_t *status_out, void *ws, hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    LinearWs w = carve_linear(ws, batch, n);
    const unsigned grid = (unsigned)((batch + kWave - 1) / kWave);
    hipLaunchKernelGGL(linear_reset_kernel, dim3(1), dim3(1), 0, stream, w);
    if (st.chain <= kRingMaxChainStride)
        if (n <= kLogMaxLayers)
            hipLaunchKernelGGL(linear_ring_kernel<true>, dim3(grid), dim3(kWave), 0, stream, d, batch, n, st.chain,
                               st.pos, mask_out, peak_out, status_out, w);
        else
            hipLaunchKernelGGL(linear_ring_kernel<false>, dim3(grid), dim3(kWave), 0, stream, d, batch, n, st.chain,
                               st.pos, mask_out, peak_out, status_out, w);
    else
        hipLaunchKernelGGL(linear_defer_all_kernel, dim3((unsigned)((batch + 255) / 256)), dim3(256), 0, stream,
                           batch, w);
    const int64_t wide_blocks = (batch + kWave - 1) / kWave;
    hipLaunchKernelGGL(linear_wide_kernel, dim3((unsigned)(wide_blocks < kWideBlocks ? wide_blocks : kWideBlocks)),
                       dim3(kWave), 0, stream, d, n, st.chain, st.pos, mask_out, peak_out, status_out, w,
                       (const RaggedGroupDev *)nullptr, 0);
    const unsigned lgrid = (unsigned)(batch < kListBlocks ? batch : kListBlocks);
    if (n <= kLdsStackMaxN)
        hipLaunchKernelGGL(linear_list_kernel<true>, dim3(lgrid), dim3(kWave), lds_stack_bytes(n), stream, d, n,
                           st.chain, st.pos, mask_out, peak_out, status_out, w, (const RaggedGroupDev *)nullptr, 0);
    else
        hipLaunchKernelGGL(linear_list_kernel<false>, dim3(lgrid), dim3(kWave), 0, stream, d, n, st.chain, st.pos,
                           mask_out, peak_out, status_out, w, (const RaggedGroupDev *)nullptr, 0);
    return hipGetLastError();
}

hipError_t launch_solve_linear_ragged(const int64_t *d_stage, const RaggedGroupDev *groups, int n_groups,
                                      int64_t waves, int64_t batch, int max_layers, uint8_t *mask_stage,
                                      int64_t *peak_stage, int32_t *status_stage, void *ws, hipStream_t stream)
{
    if (batch == 0) return hipSuccess;
    LinearWs w = carve_linear(ws, batch, max_layers);
    hipLaunchKernelGGL(linear_reset_kernel, dim3(1), dim3(1), 0, stream, w);
    hipLaunchKernelGGL(linear_ring_ragged_kernel, dim3((unsigned)waves), dim3(kWave), 0, stream, d_stage, groups,
                       n_groups, mask_stage, peak_stage, status_stage, w);
    const int64_t wide_blocks = (batch + kWave - 1) / kWave;
    hipLaunchKernelGGL(linear_wide_kernel, dim3((unsigned)(wide_blocks < kWideBlocks ? wide_blocks : kWideBlocks)),
                       dim3(kWave), 0, stream, d_stage, max_layers, 1, 0, mask_stage, peak_stage, status_stage, w,
                       groups, n_groups);
    const unsigned lgrid = (unsigned)(batch < kListBlocks ? batch : kListBlocks);
    if (max_layers <= kLdsStackMaxN)
        hipLaunchKernelGGL(linear_list_kernel<true>, dim3(lgrid), dim3(kWave), lds_stack_bytes(max_layers), stream,
                           d_stage, max_layers, 1, 0, mask_stage, peak_stage, status_stage, w, groups, n_groups);
    else
        hipLaunchKernelGGL(linear_list_kernel<false>, dim3(lgrid), dim3(kWave), 0, stream, d_stage, max_layers, 1, 0,
                           mask_stage, peak_stage, status_stage, w, groups, n_groups);
    return hipGetLastError();
}

}  // namespace ckpt
