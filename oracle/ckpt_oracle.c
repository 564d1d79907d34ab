/*
 * CPU oracle for checkpoint selection on a chain of n layers.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * tests, the smoke check and the benchmark's CPU-baseline leg compare the GPU
 * library against.  It shares no code with the GPU library and nothing in the
 * product path may call it.
 *
 * Conventions (paper, Section 3.1 "Problem Definition"): a chain of n layers is
 * the array d[0..n] of n+1 positive sizes; d[0] is the input, d[n] the output
 * and both are always checkpoints.  A checkpoint set is mask[0..n] of bytes
 * with mask[0] = mask[n] = 1.  All arithmetic is exact 64-bit integer.
 *
 * Every function follows the plain definition it cites, in the paper's
 * notation, with no blocking or reordering.
 *
 * Readings taken where the paper is silent or inconsistent:
 *  - Section 4 states its recurrences for d_1..d_n with answer M(1); here the
 *    same array d[0..n] is used for both objectives and the answer is M(0).
 *  - The recurrence for M(i) ranges over i < j <= n (Algorithm 5's loop
 *    bounds), not i < j < n as the displayed equations say.
 *  - Algorithm 4 reads the queue head before inserting i; Equation (T) lets
 *    j = i be a candidate, so i is inserted first here.
 *  - Algorithm 4 returns min_s (s + M(n,s)), which would let d_n sit in a
 *    trailing segment; since d_n is a checkpoint the cost of a budget s is
 *    s + d_n + M(n-1,s).
 *  - M(-1,s) = 0, so that position 0 contributes d_0.
 *  - Algorithm 3 recomputes a segment before it releases the previous output
 *    gradient buffer; Equation (memory) does not contain that transient, so
 *    the event simulator releases the old buffer first.
 *  - Optimal sets are not unique.  The canonical set is defined on the value
 *    functions: static objective - the smallest optimal budget s*, then from
 *    j = n the smallest feasible predecessor with minimal value; dynamic
 *    objective - from i = 0 the smallest j attaining M(i).
 *
 * Pinned by tests/test_oracle_*.py: brute force over all subsets (n <= 20),
 * closed forms for fixed sets and uniform chains, monotonicity and bounds,
 * hand-worked tiny chains, the paper's VGG-19 sets and memory gaps, the
 * event simulators of Algorithms 2 and 3 against the closed forms, the
 * per-phase timeline against the printed prediction curve of Section 5.2
 * (phase indices 0..36; the rest of that curve is not consistent with
 * Equation (memory), so the later backward stages are pinned by hand-worked
 * chains and closed forms only), and the sqrt(n) sets of the peak-memory table.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef int64_t i64;
#define ORC_INF INT64_MAX

/* ------------------------------------------------------------------------ */
/* Objective functions                                                       */
/* ------------------------------------------------------------------------ */

/* Equation (cost), Section 3.1: sum of all checkpoints plus the largest
 * segment, a segment being the non-checkpoints between two consecutive
 * checkpoints (possibly empty).  Returns -1 if an end is not a checkpoint. */
i64 orc_peak_static(const i64 *d, const uint8_t *mask, int n)
{
    if (!mask[0] || !mask[n]) return -1;
    i64 checkpoint_memory = 0;
    for (int i = 0; i <= n; i++)
        if (mask[i]) checkpoint_memory += d[i];
    i64 segment_memory = 0;
    int h = 0;                                   /* previous checkpoint */
    for (int i = 1; i <= n; i++) {
        if (!mask[i]) continue;
        i64 sum = 0;
        for (int j = h + 1; j <= i - 1; j++) sum += d[j];
        if (sum > segment_memory) segment_memory = sum;
        h = i;
    }
    return checkpoint_memory + segment_memory;
}

/* Equation (memory), Section 4: for a checkpoint i whose previous checkpoint
 * is h,  m(i) = sum_{c in C, c <= i} d_c + sum_{k=h+1}^{i-1} d_k
 *              + max_{h <= k < i} d_k ;  the peak is the largest m(i). */
i64 orc_peak_dynamic(const i64 *d, const uint8_t *mask, int n)
{
    if (!mask[0] || !mask[n]) return -1;
    i64 peak = 0;
    int h = 0;
    for (int i = 1; i <= n; i++) {
        if (!mask[i]) continue;
        i64 c_i = 0;                             /* checkpoints up to i */
        for (int c = 0; c <= i; c++) if (mask[c]) c_i += d[c];
        i64 seg = 0;
        for (int k = h + 1; k <= i - 1; k++) seg += d[k];
        i64 grad = 0;                            /* output gradient buffer */
        for (int k = h; k < i; k++) if (d[k] > grad) grad = d[k];
        i64 m = c_i + seg + grad;
        if (m > peak) peak = m;
        h = i;
    }
    return peak;
}

/* Algorithm 2 as an allocate/free event simulation: returns the largest
 * number of live bytes.  d_0 is resident from the start. */
i64 orc_sim_static(const i64 *d, const uint8_t *mask, int n)
{
    if (!mask[0] || !mask[n]) return -1;
    i64 live = d[0], peak = d[0];
    /* forward phase */
    for (int i = 1; i <= n; i++) {
        live += d[i];                            /* allocate d_i */
        if (live > peak) peak = live;
        if (!mask[i - 1]) live -= d[i - 1];      /* free a non-checkpoint */
    }
    /* backward phase */
    int seg_lo = 1, seg_hi = 0;                  /* live recomputed segment */
    for (int i = n; i >= 1; i--) {
        if (mask[i]) {
            for (int k = seg_lo; k <= seg_hi; k++) live -= d[k];
            int h = i - 1;
            while (!mask[h]) h--;
            seg_lo = h + 1; seg_hi = i - 1;
            for (int k = seg_lo; k <= seg_hi; k++) live += d[k];
            if (live > peak) peak = live;
        }
    }
    return peak;
}

/* Algorithm 3 as an event simulation (old gradient buffer released before the
 * segment is recomputed, see the header). */
i64 orc_sim_dynamic(const i64 *d, const uint8_t *mask, int n)
{
    if (!mask[0] || !mask[n]) return -1;
    i64 live = d[0], peak = d[0];
    for (int i = 1; i <= n; i++) {
        live += d[i];
        if (live > peak) peak = live;
        if (!mask[i - 1]) live -= d[i - 1];
    }
    i64 r = 0;                                   /* gradient buffer size */
    for (int i = n; i >= 1; i--) {
        if (mask[i]) {
            int h = i - 1;
            while (!mask[h]) h--;
            live -= r;                           /* release previous buffer */
            for (int k = h + 1; k <= i - 1; k++) live += d[k];
            r = 0;
            for (int k = h; k <= i - 1; k++) if (d[k] > r) r = d[k];
            live += r;
            if (live > peak) peak = live;
        }
        live -= d[i];                            /* release d_i */
    }
    return peak;
}

/* Memory per training phase index (Section 5.1, "Models and Definitions":
 * index 0 is the stage before training, 1..n the forward stage of layer i,
 * n+1..2n the backward stages of layers n..1, 2n+1 the stage after
 * training), read off the allocate/free events of Algorithm 2 (objective 0)
 * or Algorithm 3 (objective 1).  The value of a stage is the number of live
 * bytes once the stage has made its allocations and before it releases
 * anything at its end: in a forward stage d_i is allocated while d_{i-1} is
 * still there; a backward stage of Algorithm 3 is sampled before "release
 * the memory d_i" (so a checkpoint stage gives m(i) of Equation (memory) and
 * the other stages m(i') of Equation (iprime)); the old gradient buffer is
 * released before the segment is recomputed, as in orc_sim_dynamic.  Before
 * and after training only the input d_0 is resident.  out has 2n+2 entries;
 * they are all -1 if an end is not a checkpoint. */
void orc_timeline(const i64 *d, const uint8_t *mask, int n, int objective, i64 *out)
{
    if (!mask[0] || !mask[n]) {
        for (int t = 0; t <= 2 * n + 1; t++) out[t] = -1;
        return;
    }
    i64 live = d[0];
    out[0] = live;
    for (int i = 1; i <= n; i++) {               /* forward phase */
        live += d[i];                            /* allocate d_i */
        out[i] = live;
        if (!mask[i - 1]) live -= d[i - 1];      /* free a non-checkpoint */
    }
    if (objective == 0) {                        /* Algorithm 2 */
        int seg_lo = 1, seg_hi = 0;              /* live recomputed segment */
        for (int i = n; i >= 1; i--) {
            if (mask[i]) {
                for (int k = seg_lo; k <= seg_hi; k++) live -= d[k];
                int h = i - 1;
                while (!mask[h]) h--;
                seg_lo = h + 1; seg_hi = i - 1;
                for (int k = seg_lo; k <= seg_hi; k++) live += d[k];
            }
            out[2 * n + 1 - i] = live;
        }
    } else {                                     /* Algorithm 3 */
        i64 r = 0;                               /* gradient buffer size */
        for (int i = n; i >= 1; i--) {
            if (mask[i]) {
                int h = i - 1;
                while (!mask[h]) h--;
                live -= r;
                for (int k = h + 1; k <= i - 1; k++) live += d[k];
                r = 0;
                for (int k = h; k <= i - 1; k++) if (d[k] > r) r = d[k];
                live += r;
            }
            out[2 * n + 1 - i] = live;
            live -= d[i];                        /* release d_i */
        }
    }
    out[2 * n + 1] = d[0];
}

/* ------------------------------------------------------------------------ */
/* Checkpoint sets that do not look at the sizes (Section 2.1)               */
/* ------------------------------------------------------------------------ */

/* kind 0: no interior checkpoint (only d_0 and d_n);  kind 1: every position;
 * kind 2: Chen et al.'s sqrt(n) rule as the paper applies it in Section 5 -
 * segments of k = ceil(sqrt(n)) layers, i.e. checkpoints at the multiples of
 * k below n, plus the forced ends (n = 24 gives {5,10,15,20,24}, n = 15 gives
 * {4,8,12,15}, the sets of the peak-memory table). */
void orc_select_baseline(int n, int kind, uint8_t *mask_out)
{
    int k = 1;
    while ((i64)k * k < n) k++;
    for (int i = 0; i <= n; i++) {
        uint8_t on = (i == 0 || i == n);
        if (kind == 1) on = 1;
        if (kind == 2 && i % k == 0) on = 1;
        mask_out[i] = on;
    }
}

/* ------------------------------------------------------------------------ */
/* Brute force over all subsets (n <= 24)                                    */
/* ------------------------------------------------------------------------ */

/* Walks every bit pattern over positions 1..n (2^n of them), keeps those in
 * which position n is set (position 0 is always set; the others are not valid
 * sets), and evaluates the chosen objective (0: static, 1: dynamic).  Returns
 * the optimum; *n_optimal counts the optimal sets; min_maxseg receives
 * the smallest largest-segment sum among the optimal sets (static objective
 * only, used to pin the canonical budget). */
i64 orc_brute(const i64 *d, int n, int objective, i64 *n_optimal, i64 *min_maxseg)
{
    uint8_t mask[32];
    i64 best = ORC_INF, count = 0, best_seg = ORC_INF;
    for (uint32_t bits = 0; bits < (1u << n); bits++) {
        if (!((bits >> (n - 1)) & 1u)) continue; /* d_n must be a checkpoint */
        mask[0] = 1;
        for (int i = 1; i <= n; i++) mask[i] = (bits >> (i - 1)) & 1u;
        i64 v = objective ? orc_peak_dynamic(d, mask, n) : orc_peak_static(d, mask, n);
        i64 seg = 0, run = 0;
        for (int i = 0; i <= n; i++) {
            if (mask[i]) { if (run > seg) seg = run; run = 0; } else run += d[i];
        }
        if (v < best) { best = v; count = 1; best_seg = seg; }
        else if (v == best) { count++; if (seg < best_seg) best_seg = seg; }
    }
    if (n_optimal) *n_optimal = count;
    if (min_maxseg) *min_maxseg = best_seg;
    return best;
}

/* ------------------------------------------------------------------------ */
/* Static objective: Section 3.2                                             */
/* ------------------------------------------------------------------------ */

/* For one segment budget s, the table F(j) = d_j + M(j-1,s) by the literal
 * form of Equation (T): M(i,s) = min over l(i) <= j <= i of d_j + M(j-1,s),
 * where j ranges over positions whose trailing segment j+1..i fits in s.
 * F has n+1 entries; F(n) is the checkpoint memory c_s with d_n forced. */
static void static_table_literal(const i64 *d, int n, i64 s, i64 *F)
{
    F[0] = d[0];                                 /* d_0 + M(-1,s), M(-1,s) = 0 */
    for (int i = 0; i <= n - 1; i++) {
        /* M(i,s) */
        i64 M = ORC_INF;
        i64 seg = 0;                             /* sum_{k=j+1}^{i} d_k */
        for (int j = i; j >= 0; j--) {
            if (seg > s) break;                  /* Inequality (j) fails from here on */
            if (F[j] < M) M = F[j];
            seg += d[j];
        }
        F[i + 1] = d[i + 1] + M;
    }
}

/* Canonical set for a budget s from its table: from j = n take the smallest
 * feasible predecessor h with minimal F(h). */
static void static_backtrack(const i64 *d, int n, i64 s, const i64 *F, uint8_t *mask)
{
    memset(mask, 0, (size_t)n + 1);
    int j = n;
    mask[n] = 1;
    while (j > 0) {
        i64 target = F[j] - d[j];
        i64 seg = 0;
        int pred = -1;
        for (int h = j - 1; h >= 0; h--) {
            if (seg > s) break;
            if (F[h] == target) pred = h;        /* keeps the smallest */
            seg += d[h];
        }
        mask[pred] = 1;
        j = pred;
    }
}

/* Number of candidate budgets: the empty segment plus every contiguous range
 * inside d_1..d_{n-1} ("enumerating the start and end points"). */
i64 orc_num_budgets(int n) { return (i64)n * (n - 1) / 2 + 1; }

/* Writes the candidate budgets in the order: 0, then ranges by length and
 * start. */
void orc_budgets(const i64 *d, int n, i64 *out)
{
    i64 *P = (i64 *)malloc(sizeof(i64) * ((size_t)n + 1));   /* P[k] = d_0 + .. + d_k */
    P[0] = d[0];
    for (int k = 1; k <= n; k++) P[k] = P[k - 1] + d[k];
    i64 t = 0;
    out[t++] = 0;
    for (int len = 1; len <= n - 1; len++)
        for (int a = 1; a + len - 1 <= n - 1; a++)
            out[t++] = P[a + len - 1] - P[a - 1];            /* d_a + .. + d_{a+len-1} */
    free(P);
}

/* The two-step scheme with the literal recurrence.  O(n^4); small n only.
 * Returns min_s (s + c_s); mask_out the canonical set, s_out the smallest
 * optimal budget. */
i64 orc_solve_static_literal(const i64 *d, int n, uint8_t *mask_out, i64 *s_out)
{
    i64 K = orc_num_budgets(n);
    i64 *budgets = (i64 *)malloc(sizeof(i64) * (size_t)K);
    i64 *F = (i64 *)malloc(sizeof(i64) * ((size_t)n + 1));
    orc_budgets(d, n, budgets);
    i64 best = ORC_INF, best_s = ORC_INF;
    for (i64 t = 0; t < K; t++) {
        i64 s = budgets[t];
        static_table_literal(d, n, s, F);
        i64 cost = s + F[n];
        if (cost < best || (cost == best && s < best_s)) { best = cost; best_s = s; }
    }
    if (mask_out) {
        static_table_literal(d, n, best_s, F);
        static_backtrack(d, n, best_s, F, mask_out);
    }
    if (s_out) *s_out = best_s;
    free(F); free(budgets);
    return best;
}

/* Algorithm 4 for one budget: window start l(i) by a sliding window, and the
 * minimum of d_q + M(q-1,s) over the window from a monotone queue Q that
 * drops strictly larger tails.  Returns c_s = d_n + M(n-1,s).  Mq[] and Q[]
 * are caller scratch of n+1 entries each; if F_out is given it receives
 * F(j) = d_j + M(j-1,s). */
static i64 static_budget_queue(const i64 *d, int n, i64 s, i64 *key, int *Q, i64 *F_out)
{
    int head = 0, tail = 0;                      /* Q[head..tail-1] */
    int l = 0;                                   /* l(i) */
    i64 window = 0;                              /* sum_{k=l+1}^{i} d_k */
    i64 M_prev = 0;                              /* M(i-1,s), M(-1,s) = 0 */
    for (int i = 0; i <= n - 1; i++) {
        if (i > 0) window += d[i];
        while (window > s) { l++; window -= d[l]; }
        key[i] = d[i] + M_prev;                  /* d_i + M(i-1,s) */
        while (tail > head && key[Q[tail - 1]] > key[i]) tail--;
        Q[tail++] = i;
        while (Q[head] < l) head++;
        M_prev = key[Q[head]];                   /* M(i,s) */
    }
    key[n] = d[n] + M_prev;
    if (F_out) memcpy(F_out, key, sizeof(i64) * ((size_t)n + 1));
    return key[n];
}

/* Algorithm 4 over every budget, OpenMP over budgets.  Same result contract
 * as orc_solve_static_literal.  first_budget/num: evaluate only budgets
 * [first, first+num) of the list (num < 0: all), for bounded timing runs. */
i64 orc_solve_static_range(const i64 *d, int n, uint8_t *mask_out, i64 *s_out,
                           i64 first_budget, i64 num)
{
    i64 K = orc_num_budgets(n);
    i64 *budgets = (i64 *)malloc(sizeof(i64) * (size_t)K);
    orc_budgets(d, n, budgets);
    i64 lo = first_budget, hi = (num < 0) ? K : first_budget + num;
    if (hi > K) hi = K;
    i64 best = ORC_INF, best_s = ORC_INF;
#pragma omp parallel
    {
        i64 *key = (i64 *)malloc(sizeof(i64) * ((size_t)n + 1));
        int *Q = (int *)malloc(sizeof(int) * ((size_t)n + 1));
        i64 my_best = ORC_INF, my_s = ORC_INF;
#pragma omp for schedule(dynamic, 64)
        for (i64 t = lo; t < hi; t++) {
            i64 s = budgets[t];
            i64 cost = s + static_budget_queue(d, n, s, key, Q, NULL);
            if (cost < my_best || (cost == my_best && s < my_s)) { my_best = cost; my_s = s; }
        }
#pragma omp critical
        {
            if (my_best < best || (my_best == best && my_s < best_s)) { best = my_best; best_s = my_s; }
        }
        free(key); free(Q);
    }
    if (mask_out && best != ORC_INF) {
        i64 *F = (i64 *)malloc(sizeof(i64) * ((size_t)n + 1));
        i64 *key = (i64 *)malloc(sizeof(i64) * ((size_t)n + 1));
        int *Q = (int *)malloc(sizeof(int) * ((size_t)n + 1));
        static_budget_queue(d, n, best_s, key, Q, F);
        static_backtrack(d, n, best_s, F, mask_out);
        free(F); free(key); free(Q);
    }
    if (s_out) *s_out = best_s;
    free(budgets);
    return best;
}

i64 orc_solve_static(const i64 *d, int n, uint8_t *mask_out, i64 *s_out)
{
    return orc_solve_static_range(d, n, mask_out, s_out, 0, -1);
}

/* c_s for one budget, exposed for monotonicity tests (literal recurrence). */
i64 orc_static_cs(const i64 *d, int n, i64 s)
{
    i64 *F = (i64 *)malloc(sizeof(i64) * ((size_t)n + 1));
    static_table_literal(d, n, s, F);
    i64 c = F[n];
    free(F);
    return c;
}

/* ------------------------------------------------------------------------ */
/* Dynamic objective: Section 4.1                                            */
/* ------------------------------------------------------------------------ */

/* Equation (s): s(i,j) = sum_{k=i+1}^{j-1} d_k + max_{i <= k < j} d_k. */
static i64 s_ij(const i64 *d, int i, int j)
{
    i64 sum = 0, mx = 0;
    for (int k = i + 1; k <= j - 1; k++) sum += d[k];
    for (int k = i; k < j; k++) if (d[k] > mx) mx = d[k];
    return sum + mx;
}

/* Algorithm 5: M(n) = d_n; M(i) = min_{i<j<=n} max(d_i + M(j),
 * d_i + s(i,j) + d_j), with s(i,j) accumulated as j advances.  M_out (n+1
 * entries, may be NULL) receives the value function; mask_out the canonical
 * set (from i = 0, the smallest j attaining M(i)).  Returns M(0). */
i64 orc_solve_dynamic(const i64 *d, int n, uint8_t *mask_out, i64 *M_out)
{
    i64 *M = (i64 *)malloc(sizeof(i64) * ((size_t)n + 1));
    int *next = (int *)malloc(sizeof(int) * ((size_t)n + 1));
    M[n] = d[n];
    next[n] = n;
    for (int i = n - 1; i >= 0; i--) {
        M[i] = ORC_INF;
        i64 sum = 0, mx = d[i];                  /* s(i,i+1) = d_i */
        for (int j = i + 1; j <= n; j++) {
            i64 a = d[i] + M[j];
            i64 b = d[i] + (sum + mx) + d[j];
            i64 v = a > b ? a : b;
            if (v < M[i]) { M[i] = v; next[i] = j; }
            sum += d[j];
            if (d[j] > mx) mx = d[j];
        }
    }
    if (mask_out) {
        memset(mask_out, 0, (size_t)n + 1);
        int i = 0;
        mask_out[0] = 1;
        while (i < n) { i = next[i]; mask_out[i] = 1; }
    }
    if (M_out) memcpy(M_out, M, sizeof(i64) * ((size_t)n + 1));
    i64 r = M[0];
    free(M); free(next);
    return r;
}

/* Same recurrence with s(i,j) recomputed from Equation (s) for every pair:
 * O(n^3), for checking the accumulation above on small chains. */
i64 orc_solve_dynamic_literal(const i64 *d, int n, i64 *M_out)
{
    i64 *M = (i64 *)malloc(sizeof(i64) * ((size_t)n + 1));
    M[n] = d[n];
    for (int i = n - 1; i >= 0; i--) {
        M[i] = ORC_INF;
        for (int j = i + 1; j <= n; j++) {
            i64 a = d[i] + M[j];
            i64 b = d[i] + s_ij(d, i, j) + d[j];
            i64 v = a > b ? a : b;
            if (v < M[i]) M[i] = v;
        }
    }
    if (M_out) memcpy(M_out, M, sizeof(i64) * ((size_t)n + 1));
    i64 r = M[0];
    free(M);
    return r;
}

/* ------------------------------------------------------------------------ */
/* Batches: chain c occupies d[c*(n+1) .. c*(n+1)+n] (chain-major).          */
/* ------------------------------------------------------------------------ */

void orc_batch_peak(const i64 *d, const uint8_t *mask, i64 batch, int n, int objective, i64 *peak_out)
{
#pragma omp parallel for schedule(static)
    for (i64 c = 0; c < batch; c++) {
        const i64 *dc = d + c * ((i64)n + 1);
        const uint8_t *mc = mask + c * ((i64)n + 1);
        peak_out[c] = objective ? orc_peak_dynamic(dc, mc, n) : orc_peak_static(dc, mc, n);
    }
}

void orc_batch_timeline(const i64 *d, const uint8_t *mask, i64 batch, int n, int objective, i64 *out)
{
#pragma omp parallel for schedule(static)
    for (i64 c = 0; c < batch; c++)
        orc_timeline(d + c * ((i64)n + 1), mask + c * ((i64)n + 1), n, objective,
                     out + c * (2 * (i64)n + 2));
}

void orc_batch_solve_dynamic(const i64 *d, i64 batch, int n, uint8_t *mask_out, i64 *peak_out)
{
#pragma omp parallel for schedule(static)
    for (i64 c = 0; c < batch; c++)
        peak_out[c] = orc_solve_dynamic(d + c * ((i64)n + 1), n,
                                        mask_out ? mask_out + c * ((i64)n + 1) : NULL, NULL);
}

void orc_batch_solve_static(const i64 *d, i64 batch, int n, uint8_t *mask_out, i64 *peak_out, i64 *s_out)
{
    /* chains in sequence; each chain's budgets run in parallel */
    for (i64 c = 0; c < batch; c++)
        peak_out[c] = orc_solve_static(d + c * ((i64)n + 1), n,
                                       mask_out ? mask_out + c * ((i64)n + 1) : NULL,
                                       s_out ? s_out + c : NULL);
}

/* ------------------------------------------------------------------------ */
/* Ragged batches: chain c has n_c = off[c+1] - off[c] - 1 layers and         */
/* occupies d[off[c] .. off[c+1]-1]; masks use the same offsets, timelines   */
/* (2 n_c + 2 values) start at 2 off[c].  What cutting a network that is not  */
/* a chain into linear sub-chains produces (the paper's concluding remarks),  */
/* or one model in plain and in extended specs (Section 5.4).  Each chain is  */
/* solved on its own by the functions above.                                  */
/* ------------------------------------------------------------------------ */

void orc_ragged_peak(const i64 *d, const uint8_t *mask, const i64 *off, i64 batch, int objective, i64 *peak_out)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (i64 c = 0; c < batch; c++) {
        int n = (int)(off[c + 1] - off[c] - 1);
        peak_out[c] = objective ? orc_peak_dynamic(d + off[c], mask + off[c], n)
                                : orc_peak_static(d + off[c], mask + off[c], n);
    }
}

void orc_ragged_timeline(const i64 *d, const uint8_t *mask, const i64 *off, i64 batch, int objective, i64 *out)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (i64 c = 0; c < batch; c++)
        orc_timeline(d + off[c], mask + off[c], (int)(off[c + 1] - off[c] - 1), objective, out + 2 * off[c]);
}

void orc_ragged_solve_dynamic(const i64 *d, const i64 *off, i64 batch, uint8_t *mask_out, i64 *peak_out)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (i64 c = 0; c < batch; c++)
        peak_out[c] = orc_solve_dynamic(d + off[c], (int)(off[c + 1] - off[c] - 1),
                                        mask_out ? mask_out + off[c] : NULL, NULL);
}

void orc_ragged_solve_static(const i64 *d, const i64 *off, i64 batch, uint8_t *mask_out, i64 *peak_out, i64 *s_out)
{
    for (i64 c = 0; c < batch; c++)
        peak_out[c] = orc_solve_static(d + off[c], (int)(off[c + 1] - off[c] - 1),
                                       mask_out ? mask_out + off[c] : NULL, s_out ? s_out + c : NULL);
}

/* c_s of Equation (T) for each budget of a list, by the literal recurrence. */
void orc_static_cs_list(const i64 *d, int n, const i64 *s_list, i64 count, i64 *out)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (i64 t = 0; t < count; t++) out[t] = orc_static_cs(d, n, s_list[t]);
}

/* Number of threads the batch and budget loops use from now on (t < 1: the default again). */
void orc_set_threads(int t)
{
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    extern int omp_get_num_procs(void);
    omp_set_num_threads(t >= 1 ? t : omp_get_num_procs());
#else
    (void)t;
#endif
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
