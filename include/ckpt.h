/*
 * ckpt.h - C ABI of the MI355X (gfx950) checkpoint-selection library.
 *
 * Problem (paper, Section 3.1 "Problem Definition"): a chain of n layers is the
 * sequence of n+1 positive data sizes d_0..d_n (bytes); d_0 is the input, d_n
 * the output, and both are always checkpoints.  A checkpoint set C is a byte
 * mask over positions 0..n with mask[0] = mask[n] = 1.
 *
 * Memory and ownership.  Every pointer below, except the ckpt_layout itself
 * and the offsets_host of the ragged calls, is a DEVICE pointer owned by the
 * caller.  The library allocates no memory, keeps no data, streams or events
 * between calls and does not synchronise: each call validates its arguments on
 * the host, enqueues its kernels on `hip_stream` (a hipStream_t passed as
 * void*, NULL = the null stream) and returns.  (Two exceptions, stated where
 * they are declared: the ragged calls wait once for a small copy, and
 * ckpt_solve_linear_noalloc uses a device array of the library's own.)  Outputs are valid
 * once the stream has reached the end of the call's work.  `ws` is scratch of
 * at least ckpt_workspace_bytes() bytes, 256-byte aligned, private to the call
 * until it has finished on the stream; its contents need no initialisation.
 *
 * Layout.  A batch holds `batch` independent chains of the same n.  Element k
 * of chain c of an int64 array `a` is a[c*chain_stride + k*pos_stride]
 * (strides in elements, both > 0).  The fast layout is position-major
 * ("structure of arrays"): chain_stride = 1, pos_stride = batch, which makes
 * the 64 lanes of a wavefront read 512 contiguous bytes per position.  Masks
 * (input and output) use the same two strides in bytes.  Chain-major
 * (chain_stride = n+1, pos_stride = 1) is accepted and slower.
 *
 * Errors.  Host-detectable errors (null pointer, bad shape or stride, too
 * small a workspace) are returned and nothing is launched.  Data-dependent
 * errors are reported per chain in status_out[c] (may be NULL) as one of the
 * ckpt_status values; such a chain gets peak -1 and an all-zero mask, the
 * other chains are unaffected:
 *   CKPT_ERR_SIZE      some d_k <= 0 (Lemma 1 of Section 4.2 needs d > 0),
 *   CKPT_ERR_OVERFLOW  sum(d) + max(d) does not fit in a signed 64-bit value,
 *   CKPT_ERR_MASK      mask[0] or mask[n] is 0 (ckpt_eval_peak only).
 *
 * Results are exact integers.  Where several optimal sets exist the library
 * returns a canonical one, defined on the value functions (see each call).
 */
#ifndef CKPT_H
#define CKPT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CKPT_OK = 0,
    CKPT_ERR_NULL = 1,
    CKPT_ERR_SHAPE = 2,
    CKPT_ERR_SIZE = 3,
    CKPT_ERR_OVERFLOW = 4,
    CKPT_ERR_MASK = 5,
    CKPT_ERR_WORKSPACE = 6,
    CKPT_ERR_DEVICE = 7
} ckpt_status;

typedef enum {
    CKPT_OBJ_STATIC = 0,  /* Equation (cost), Section 3.1: all checkpoints + largest segment */
    CKPT_OBJ_DYNAMIC = 1, /* Equation (memory), Section 4: early release + output-gradient buffer */
    CKPT_OBJ_BOTH = 2     /* ckpt_eval_peak only: both of the above from one pass over the chains */
} ckpt_objective;

/* Checkpoint sets that do not look at the sizes (ckpt_select_baseline). */
typedef enum {
    CKPT_SELECT_ENDS = 0, /* only d_0 and d_n: everything is recomputed in one segment */
    CKPT_SELECT_ALL = 1,  /* every position: nothing is recomputed (Algorithm 1) */
    CKPT_SELECT_SQRT = 2  /* segments of ceil(sqrt(n)) layers (Section 2.1) */
} ckpt_baseline;

typedef enum {
    CKPT_CALL_EVAL_PEAK = 0,
    CKPT_CALL_SOLVE_CUBIC = 1,
    CKPT_CALL_SOLVE_LINEAR = 2,
    CKPT_CALL_EVAL_TIMELINE = 3
} ckpt_call;

/* Largest n accepted by ckpt_eval_peak and ckpt_solve_linear, and by
 * ckpt_solve_cubic (whose work grows as n^3). */
#define CKPT_MAX_LAYERS 65535
#define CKPT_CUBIC_MAX_LAYERS 8191
/* Largest n accepted by ckpt_solve_quadratic (its per-chain state lives in LDS). */
#define CKPT_QUADRATIC_MAX_LAYERS 4095

typedef struct {
    int64_t batch;        /* number of chains, 0 .. 2^31-1 (0: the call does nothing) */
    int32_t n_layers;     /* n >= 1; every chain has n+1 sizes */
    int64_t chain_stride; /* elements between the same position of consecutive chains */
    int64_t pos_stride;   /* elements between consecutive positions of one chain */
} ckpt_layout;

/* Bytes of scratch the call `which` (a ckpt_call) needs for this layout;
 * 0 if the layout is invalid.  Host-only, launches nothing. */
size_t ckpt_workspace_bytes(int which, const ckpt_layout *layout);

/* Peak memory of a given checkpoint set, per chain.
 *   CKPT_OBJ_STATIC : Equation (cost), the model of Algorithm 2 -
 *       sum_{i in C} d_i + max over segments of the segment's sum.
 *   CKPT_OBJ_DYNAMIC: Equation (memory), the model of Algorithm 3 - the
 *       largest, over checkpoints i with previous checkpoint h, of
 *       sum_{c in C, c <= i} d_c + sum_{h<k<i} d_k + max_{h<=k<i} d_k.
 *   CKPT_OBJ_BOTH   : both (Section 5 compares a set's memory under the two
 *       models): the chains are read once, peak_out receives 2 * batch values,
 *       the static peaks first (peak_out[c]), then the dynamic ones
 *       (peak_out[batch + c]); a chain's status is the same under either.
 * d [in] sizes, mask [in] checkpoint bytes (non-zero = checkpoint), both in
 * `layout`; peak_out [out] `batch` int64 (2 * batch with CKPT_OBJ_BOTH);
 * status_out [out] `batch` int32 or NULL. */
int ckpt_eval_peak(const int64_t *d, const uint8_t *mask, const ckpt_layout *layout,
                   int objective, int64_t *peak_out, int32_t *status_out,
                   void *ws, size_t ws_bytes, void *hip_stream);

/* Optimal checkpoint set under Equation (cost) by the two-step scheme of
 * Section 3.2 (Algorithm 4, Theorem 1): for every candidate segment budget s
 * (0 and every sum of a contiguous range inside d_1..d_{n-1}) the least
 * checkpoint memory c_s whose segments all fit in s, by the recurrence of
 * Equation (T); the answer is min_s (s + c_s) with d_0 and d_n checkpoints.
 * n <= CKPT_CUBIC_MAX_LAYERS.
 * Canonical result: budget_out[c] is the smallest optimal budget value s*;
 * the set is built from position n by taking, each time, the smallest
 * feasible predecessor of minimal value.
 * mask_out [out] bytes 0/1 in `layout`; peak_out [out] `batch` int64;
 * budget_out [out] `batch` int64 or NULL; status_out as above. */
int ckpt_solve_cubic(const int64_t *d, const ckpt_layout *layout, uint8_t *mask_out,
                     int64_t *peak_out, int64_t *budget_out, int32_t *status_out,
                     void *ws, size_t ws_bytes, void *hip_stream);

/* The same result as ckpt_solve_cubic, without running the recurrence for
 * budgets that cannot be optimal.  Any cost s + c_s that has been reached
 * bounds the optimum from above (UB).  From above: c_s >= d_0 + d_n for every
 * budget (both ends are checkpoints), so a budget s > UB - d_0 - d_n costs more
 * than UB.  From below: with m interior checkpoints the other interior layers
 * form at most m+1 segments of at most s each, so the checkpoints weigh at
 * least sum(interior) - (m+1) s, and at least the m smallest interior sizes
 * W(m); c_s - d_0 - d_n >= min_m max(W(m), sum(interior) - (m+1) s), which
 * does not grow with s, so the budgets for which it exceeds UB - d_0 - d_n are
 * the ones below some s_lo.  The call takes a first UB from feasible sets it
 * builds itself (a checkpoint every ceil(sqrt(n)) layers; greedy sets for a
 * grid of segment limits); if the bounds from that UB still leave more than an
 * eighth of the budgets it runs one tile in 64 of the budgets (ordered by value) inside
 * them and takes UB from those as well; then it runs the budgets inside the
 * bounds: the optimum, the smallest optimal budget and
 * the canonical set are unchanged (both comparisons are strict, so ties are
 * never cut).  Chains whose values need 64-bit arithmetic, and chains of
 * fewer than 3072 layers (where pruning costs more than it saves),
 * are solved without pruning.
 * evaluated_out [out] `batch` int64 or NULL: the number of budgets whose
 * recurrence was run (sampled ones counted again when they run a second time),
 * times n the recurrence cells actually evaluated; ckpt_solve_cubic always
 * runs n(n-1)/2 + 1.  Other arguments and workspace as for ckpt_solve_cubic. */
int ckpt_solve_cubic_pruned(const int64_t *d, const ckpt_layout *layout, uint8_t *mask_out,
                            int64_t *peak_out, int64_t *budget_out, int64_t *evaluated_out,
                            int32_t *status_out, void *ws, size_t ws_bytes, void *hip_stream);

/* ckpt_solve_cubic that also returns the curve whose minimum the two-step
 * scheme of Section 3.2 takes: for every candidate budget s of a chain its
 * cost s + c_s, c_s the least checkpoint memory with every segment within s
 * (Equation (T)).  budgets_out, costs_out [out]: `batch` x
 * ckpt_cubic_costs_len(n) int64 each, chain c at offset c x that length.  The
 * budgets come in the order the kernels take them (grouped by value, 64 to a
 * wavefront, not sorted), with -1 in both arrays in the unused places at the
 * end of a chain's list; a chain with a data error leaves its part unwritten.
 * The n(n-1)/2 + 1 budgets (as a multiset: equal sums of different ranges
 * appear once each) are 0 and every sum of a contiguous range inside
 * d_1..d_{n-1}.  Other arguments, results and workspace as ckpt_solve_cubic. */
int64_t ckpt_cubic_costs_len(int32_t n_layers);
int ckpt_solve_cubic_costs(const int64_t *d, const ckpt_layout *layout, uint8_t *mask_out,
                           int64_t *peak_out, int64_t *budget_out, int64_t *budgets_out,
                           int64_t *costs_out, int32_t *status_out,
                           void *ws, size_t ws_bytes, void *hip_stream);

/* Optimal checkpoint set under Equation (memory) by the linear-time method of
 * Section 4.2 (Equation (TU), Lemmas 1-4, Algorithm 6, Theorem 3):
 *   M(n) = d_n,  M(i) = d_i + min_{i<j<=n} max(M(j), U(i,j)),
 *   U(i,j) = sum_{k=i+1}^{j} d_k + max_{i<=k<j} d_k ;  peak_out[c] = M(0).
 * Canonical result: from i = 0 the set follows the smallest j attaining M(i).
 * Arguments as for ckpt_solve_cubic (no budget). */
int ckpt_solve_linear(const int64_t *d, const ckpt_layout *layout, uint8_t *mask_out,
                      int64_t *peak_out, int32_t *status_out,
                      void *ws, size_t ws_bytes, void *hip_stream);

/* ckpt_solve_linear for callers that cannot allocate device memory (code under
 * HIP graph capture, serving loops, harnesses that forbid hipMalloc): the same
 * kernels and the same results, with the scratch that ckpt_solve_linear takes
 * from `ws` held in an array of the library's own instead (about 8 MiB of
 * device memory per GPU, reserved when the library is loaded and kept until
 * the process ends).  The call allocates and frees nothing and calls no
 * allocating routine.  Limits: batch <= CKPT_NOALLOC_MAX_BATCH and n <=
 * CKPT_NOALLOC_MAX_LAYERS, beyond which CKPT_ERR_SHAPE is returned and nothing
 * is launched.  Every call on a GPU uses that GPU's one array: calls that
 * overlap on one GPU (two streams, two threads) race and must be ordered by
 * the caller; calls in a row on one stream are fine (the call clears what it
 * needs at its start).  Arguments as for ckpt_solve_linear, without ws. */
#define CKPT_NOALLOC_MAX_BATCH 1048576
#define CKPT_NOALLOC_MAX_LAYERS 2047
int ckpt_solve_linear_noalloc(const int64_t *d, const ckpt_layout *layout, uint8_t *mask_out,
                              int64_t *peak_out, int32_t *status_out, void *hip_stream);

/* Memory per training phase index of a given checkpoint set, per chain
 * (Section 5.1, "training phase index": 0 is the stage before training, 1..n
 * the forward stage of layer i, n+1..2n the backward stages of layers n..1,
 * 2n+1 the stage after training; the curves of Section 5 plot this).  A stage
 * is sampled after its allocations and before the release at its end:
 *   forward stage i: the checkpoints up to i-1, d_i, and d_{i-1} if it is no
 *       checkpoint (the forward loop of Algorithms 2 and 3);
 *   backward stage of layer i, h the last checkpoint below i, nx the first
 *       checkpoint at or above i:
 *     CKPT_OBJ_DYNAMIC (Algorithm 3): sum_{c in C, c <= h} d_c + sum_{k=h+1}^{i} d_k
 *       + max_{h<=k<nx} d_k, i.e. Equation (memory) at a checkpoint and
 *       Equation (iprime) between checkpoints;
 *     CKPT_OBJ_STATIC (Algorithm 2): sum_{c in C} d_c + sum_{h<k<nx} d_k;
 *   indices 0 and 2n+1: d_0.
 * The largest backward stage equals the peak of ckpt_eval_peak.
 * d, mask [in] as for ckpt_eval_peak.  timeline_out [out] int64, 2n+2 values
 * per chain: phase t of chain c at timeline_out[c*out_chain_stride +
 * t*out_phase_stride] (strides in elements, both > 0; the fast layout is
 * out_chain_stride = 1, out_phase_stride = batch); it must not overlap the
 * inputs.  status_out as above; a chain with a data error gets -1 in every
 * phase.  Needs no scratch. */
int ckpt_eval_timeline(const int64_t *d, const uint8_t *mask, const ckpt_layout *layout,
                       int objective, int64_t *timeline_out, int64_t out_chain_stride,
                       int64_t out_phase_stride, int32_t *status_out, void *hip_stream);

/* The size-independent checkpoint sets that the paper compares against
 * (Section 2.1 and the peak-memory table of Section 5), written for every
 * chain of the layout: `kind` is a ckpt_baseline.  CKPT_SELECT_SQRT puts a
 * checkpoint at every multiple of ceil(sqrt(n)) below n (n = 24: {5, 10, 15,
 * 20, 24}; n = 15: {4, 8, 12, 15}); positions 0 and n are always set.
 * mask_out [out] bytes 0/1 in `layout`.  Needs no sizes and no scratch;
 * evaluate the sets with ckpt_eval_peak or ckpt_eval_timeline. */
int ckpt_select_baseline(const ckpt_layout *layout, int kind, uint8_t *mask_out, void *hip_stream);

/* The same optimum and the same canonical set as ckpt_solve_linear, by the
 * quadratic-time recurrence of Section 4.1 (Equation (T-rec), Algorithm 5,
 * Theorem 2) evaluated directly: for every i all j > i are tried, one
 * wavefront per chain with the candidates j across its lanes.  It shares
 * nothing with the linear-time kernel (no queue, no crossover pointer) and so
 * cross-checks it on the device; it is also the quicker call for a single
 * chain or a small batch.  n <= CKPT_QUADRATIC_MAX_LAYERS.
 * mask_out, peak_out, status_out as for ckpt_solve_linear; value_out [out]
 * int64 in `layout`, M(i) for every position i (all -1 for a chain with a data
 * error), or NULL.  Needs no scratch. */
int ckpt_solve_quadratic(const int64_t *d, const ckpt_layout *layout, uint8_t *mask_out,
                         int64_t *peak_out, int64_t *value_out, int32_t *status_out,
                         void *hip_stream);

/* Ragged batches: chains of different n in one call.  Section 6 (Conclusion and
 * Future Work) proposes cutting an arbitrary computation graph into many
 * linear sub-models, which yields chains of many different lengths, and
 * Section 5.4 solves one network at two granularities of its specs (AlexNet
 * as a chain of 12 and of 15 layers); the networks of Section 5 range from
 * these to VGG-19's 24 layers.  A caller with such a set hands all
 * chains over at once.  Chain c has n_c = offsets[c+1] - offsets[c] - 1 layers
 * (1 <= n_c <= the call's limit) and its sizes d_0..d_{n_c} are the elements
 * offsets[c] .. offsets[c+1]-1 of the flat device array d; flat masks (input
 * or output) use the same offsets in bytes, and the flat timeline has the
 * 2 n_c + 2 phases of chain c from element 2 offsets[c] on.  peak_out,
 * budget_out and status_out hold one value per chain, as in the equal-length
 * calls, whose results each chain gets exactly (same equations, same canonical
 * sets, same per-chain errors); ckpt_ragged_eval_peak takes CKPT_OBJ_BOTH as
 * ckpt_eval_peak does (2 * batch peaks, the static ones first).
 *   offsets_host [in] batch + 1 ascending element offsets in HOST memory (the
 *       caller built the batch and knows them; the library plans its launches
 *       from them).  It is read during the call only.
 *   offsets_dev [in] the same offsets in DEVICE memory, or NULL.  With NULL the
 *       call counts the lengths on the host and copies offsets_host into the
 *       workspace itself (from pageable host memory these are the slowest
 *       steps of a call on a large batch).  With a device copy the lengths are
 *       counted and checked on the device and offsets_host is not read (it may
 *       be NULL), except by ckpt_ragged_solve_cubic, which launches length by
 *       length and always plans on the host.
 *   ws: ckpt_ragged_workspace_bytes(which, offsets_host, batch) bytes, 256-byte
 *       aligned; it receives the counts of the lengths, the table of groups
 *       (the chains of one length), the chains' places grouped by length
 *       (handed out on the device: the order inside a group differs from call
 *       to call, the results do not), a copy of the offsets, room to stage
 *       every group in the position-major layout and the solver's own
 *       workspace.
 * Unlike the other calls these wait once on the stream before they enqueue
 * their kernels: for the copy of the table of groups (and of the offsets) into
 * ws, or, with offsets_dev, for the totals of the device's count, which size
 * the launches that follow.  Work already on the stream finishes first, and the
 * calls cannot be captured into a HIP graph.  A bad offset (decreasing, negative
 * or beyond INT64_MAX / 64, n_c < 1 or beyond the limit) returns CKPT_ERR_SHAPE;
 * found on the host nothing has been launched then, found on the device only
 * the count, which writes to ws alone.  batch = 0 does nothing.
 * ckpt_ragged_workspace_bytes returns 0 for such input. */
size_t ckpt_ragged_workspace_bytes(int which, const int64_t *offsets_host, int64_t batch);
int ckpt_ragged_eval_peak(const int64_t *d, const uint8_t *mask, const int64_t *offsets_host,
                          const int64_t *offsets_dev, int64_t batch, int objective,
                          int64_t *peak_out, int32_t *status_out,
                          void *ws, size_t ws_bytes, void *hip_stream);
int ckpt_ragged_eval_timeline(const int64_t *d, const uint8_t *mask, const int64_t *offsets_host,
                              const int64_t *offsets_dev, int64_t batch, int objective,
                              int64_t *timeline_out, int32_t *status_out,
                              void *ws, size_t ws_bytes, void *hip_stream);
int ckpt_ragged_solve_linear(const int64_t *d, const int64_t *offsets_host,
                             const int64_t *offsets_dev, int64_t batch,
                             uint8_t *mask_out, int64_t *peak_out, int32_t *status_out,
                             void *ws, size_t ws_bytes, void *hip_stream);
int ckpt_ragged_solve_cubic(const int64_t *d, const int64_t *offsets_host,
                            const int64_t *offsets_dev, int64_t batch,
                            uint8_t *mask_out, int64_t *peak_out, int64_t *budget_out,
                            int32_t *status_out, void *ws, size_t ws_bytes, void *hip_stream);

/* Number of recurrence cells one ckpt_solve_cubic call evaluates per chain:
 * (n(n-1)/2 + 1) budgets times n positions.  Host-only. */
int64_t ckpt_cubic_cells(int32_t n_layers);

/* Static, human-readable name of a ckpt_status value. */
const char *ckpt_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CKPT_H */
