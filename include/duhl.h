/*
 * duhl.h -- C ABI of the DuHL hot path for AMD MI355X (gfx950).
 *
 * DuHL (Algorithm 2 of the paper) trains a generalized linear model
 *     min_alpha  f(A alpha) + sum_i g_i(alpha_i),     A = [a_1 .. a_n] in R^{d x n}   (eq. (1))
 * on a fast unit with limited memory: each round it picks the m coordinates with the
 * largest coordinate-wise duality gap (eq. (4), (11), (13)), keeps their columns in the
 * fast unit's memory and runs randomized coordinate descent on them against the shared
 * vector v (Section 4.1, Appendix D).  This library is that per-round work on one GPU:
 *
 *     duhl_gap       per-coordinate gaps  z_i            (eq. (4); Appendix E)
 *     duhl_select    top-m working set P, rho            (eq. (11)/(13); eq. (7))
 *     duhl_cd_epoch  one pass of exact coordinate steps   (Algorithm 3; Appendix D)
 *     column swap    host -> device copy of new columns   (Algorithm 2, the step that refreshes B's memory)
 *     duhl_objective O(alpha)                             (Appendix C (b), (c))
 *
 * Models.  DUHL_LASSO:  O = ||A alpha - b||^2/(2d) + lambda ||alpha||_1, shared vector
 * v = A alpha - b.  DUHL_SVM (hinge loss, dual): O = -(1/n) sum y_i alpha_i +
 * ||A alpha||^2/(2 lambda n^2) with y_i alpha_i in [0,1], shared vector v = A alpha; a column
 * of A is one sample.  DUHL_ELASTIC_NET (Appendix D): O = ||A alpha - b||^2/(2d) +
 * lambda (eta/2 ||alpha||^2 + (1-eta) ||alpha||_1) with 0 < eta <= 1, shared vector v = A alpha - b;
 * eta = 1 is the ridge regression of Appendix C (a).  All data and state are fp32; scalar results
 * are returned as double.
 *
 * General rules.  Every call returns a duhl_status and never throws or aborts.  On error
 * the out-parameters are untouched and duhl_last_error() describes the cause.  Arrays passed
 * in stay owned by the caller; "borrowed" arrays (the matrix and the target vector) must
 * outlive the context.  The library owns alpha, v, z, the column norms and the slot buffers
 * (hipMalloc).  Work is enqueued on the two streams given at creation; a call that returns a
 * scalar to the host waits for the compute stream.  A context is not thread-safe.
 * "device" / "host" below says in which memory a pointer must live.
 */
#ifndef DUHL_H
#define DUHL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct duhl_ctx duhl_ctx;

/* (Every enumeration of an argument ends in a *_ENUM_MAX member: it widens the type's range to all of
 * int, so that a caller's invalid value reaches the library's own check -- and is answered with
 * DUHL_EINVAL -- instead of being undefined behaviour in the C++ behind this header.) */
typedef enum { DUHL_LASSO = 0, DUHL_SVM = 1, DUHL_ELASTIC_NET = 2, DUHL_MODEL_ENUM_MAX = 0x7fffffff } duhl_model;

typedef enum {
    DUHL_OK = 0,
    DUHL_EINVAL = -1,   /* bad argument (null pointer, size, lambda, malformed CSR, label)   */
    DUHL_ENOMEM = -2,   /* device or host allocation failed                                  */
    DUHL_EHIP = -3,     /* a HIP runtime call failed                                         */
    DUHL_ESTATE = -4,   /* call out of order (no data yet, no working set, swap in flight)   */
    DUHL_EBUDGET = -5   /* m exceeds the column budget given at creation                     */
} duhl_status;

/* Where the matrix lives (Assumption 1: unit A holds everything, unit B a subset). */
typedef enum {
    DUHL_RESIDENT_DEVICE = 0, /* whole matrix in HBM; the working set is an index list        */
    DUHL_RESIDENT_HOST = 1,   /* matrix in pinned, device-mapped host memory; the library
                                 keeps budget_cols columns in device slots and swaps          */
    DUHL_RESIDENT_HOST_PAGEABLE = 2, /* matrix in ordinary host memory that the device cannot read (for
                                 machines that cannot pin all of it): as DUHL_RESIDENT_HOST, but
                                 every column that crosses the host link is first copied by host
                                 threads into pinned staging buffers (3 x 64 MB for the gap passes,
                                 3 x 64 MB for the column swap, owned by the library)           */
    DUHL_RESIDENCY_ENUM_MAX = 0x7fffffff
} duhl_residency;

typedef enum { DUHL_ALPHA = 0, DUHL_V = 1, DUHL_Z = 2, DUHL_P = 3, DUHL_SQNORM = 4, DUHL_WHAT_ENUM_MAX = 0x7fffffff } duhl_what;

/* Visiting scheme of duhl_cd_epoch. */
typedef enum {
    DUHL_CD_SEQUENTIAL = 0, /* one coordinate at a time, in the given order (Algorithm 3)     */
    DUHL_CD_ASYNC = 1,      /* many coordinates at once, the library's fastest scheme          */
    DUHL_CD_ATOMIC = 2,     /* many coordinates at once, one atomic update of v per step
                               (the thread-block-per-coordinate scheme of Appendix D)          */
    DUHL_CD_MODE_ENUM_MAX = 0x7fffffff
} duhl_cd_mode;

/* Create a context for a problem with columns of length d (1 <= d < 2^29) and n coordinates
 * (1 <= n < 2^31).
 * budget_cols: the memory of unit B in columns (Assumption 1 of Section 3: B holds at most m of the
 * n columns) -- the largest working set and, for DUHL_RESIDENT_HOST, the number of device
 * column slots; 1 <= budget_cols.  device: HIP device ordinal.  compute_stream / copy_stream:
 * hipStream_t handles (NULL = the default stream); both must have the default priority. */
duhl_status duhl_create(duhl_ctx **out, duhl_model model, int64_t d, int64_t n,
                        int64_t budget_cols, int device, void *compute_stream, void *copy_stream);

/* Mixing parameter eta of DUHL_ELASTIC_NET, 0 < eta <= 1 (default 1 = ridge).  Takes effect at the
 * next duhl_set_data_* call.  DUHL_EINVAL for other models or values. */
duhl_status duhl_set_eta(duhl_ctx *ctx, double eta);

/* Two kernels let workgroups wait for each other on the device: the selection (five barriers per
 * call) and the coordinate-descent workers that span several compute units (once per coordinate).
 * Every such wait gives up after `polls` polls (default 2^22: seconds, where the waits take
 * microseconds); the kernels then end early, alpha, v and the working set are undefined, and the next
 * call that returns a scalar fails with DUHL_EHIP until the data are set again
 * (duhl_set_data_* restores a usable context).  polls in [0, 2^31); 0 makes any wait that is not
 * satisfied at once fail, which is how the error path can be exercised from the host. */
duhl_status duhl_set_wait_limit(duhl_ctx *ctx, int64_t polls);

/* Dense data (Section 2: A in R^{d x n}, fp32 per Section 5.3).  A: column-major, column i at
 * A + i*ld, ld >= d (fastest when A is 16-byte aligned and ld is a multiple of 4: the kernels
 * then use 16-byte loads); a device pointer for DUHL_RESIDENT_DEVICE, a pinned host pointer that the
 * device can read for DUHL_RESIDENT_HOST, any host pointer for DUHL_RESIDENT_HOST_PAGEABLE; borrowed.
 * With DUHL_RESIDENT_HOST_PAGEABLE duhl_select reads the swap plan back (it waits for the compute
 * stream) and a library thread stages and copies the columns until duhl_commit_swap; duhl_gap over
 * an index list reads every listed column from host memory.  target (device, borrowed): b of length d
 * for the Lasso and the elastic net, labels y in {+1,-1} of length n for the SVM.  lambda: the lambda of the
 * objectives above, finite and > 0.  Resets alpha = 0, v = -b (Lasso) or 0 (SVM), computes the
 * column norms and a first full gap pass into z (one read of A).  Waits for completion.
 * DUHL_EINVAL for a NaN or an infinity in the target vector or the matrix, labels other than +-1,
 * a lambda that is not finite and positive; the context then holds no data. */
duhl_status duhl_set_data_dense(duhl_ctx *ctx, const float *A, int64_t ld, duhl_residency res,
                                const float *target, double lambda);

/* The same for a host-resident matrix (unit A's memory, Section 3) handed over in pieces, for
 * machines that limit the size of one pinned allocation: piece k holds the columns
 * [k*cols_per_chunk, min(n, (k+1)*cols_per_chunk)), column i of them at
 * chunks[k] + (i - k*cols_per_chunk)*ld.  chunks: host array of n_chunks pointers, read during the
 * call only; n_chunks == ceil(n / cols_per_chunk).  Each piece: pinned host memory that the device can
 * read, borrowed like A above.  Residency is DUHL_RESIDENT_HOST; everything else as for
 * duhl_set_data_dense.  DUHL_EINVAL for a NULL piece, a piece the device cannot read, or counts that do not fit n. */
duhl_status duhl_set_data_dense_chunks(duhl_ctx *ctx, const float *const *chunks, int64_t n_chunks,
                                       int64_t cols_per_chunk, int64_t ld, const float *target,
                                       double lambda);

/* Sparse data: CSR over coordinates, i.e. row i lists the non-zeros of column a_i (for the SVM
 * dual: CSR of the sample matrix).  rowptr (n+1, non-decreasing, rowptr[0] = 0), colidx (each
 * in [0,d), strictly increasing inside a row), val: device pointers, borrowed.  Only DUHL_RESIDENT_DEVICE.  Otherwise as above. */
duhl_status duhl_set_data_csr(duhl_ctx *ctx, const int64_t *rowptr, const int32_t *colidx,
                              const float *val, duhl_residency res, const float *target,
                              double lambda);

/* Coordinate-wise duality gaps (eq. (4)) at the current (alpha, v), written into the gap
 * memory z of Section 4.1:
 *   Lasso (Appendix E, Lipschitzing bound B = ||b||^2/(2 lambda d)), c_i = a_i^T v:
 *       z_i = (1/d) [ alpha_i c_i + B [|c_i| - lambda d]_+ + lambda d |alpha_i| ]
 *   SVM (Appendix E), s_i = a_i^T v / (lambda n):
 *       z_i = (1/n) [ alpha_i s_i + max(0, 1 - y_i s_i) - y_i alpha_i ]
 *   elastic net (eq. (4) with the conjugate of g_i; for eta = 1 the ridge gap of Appendix E), L = lambda d:
 *       z_i = (1/d) [ alpha_i c_i + L (eta/2 alpha_i^2 + (1-eta)|alpha_i|) + [|c_i| - L(1-eta)]_+^2 / (2 L eta) ]
 * clamped at 0.  idx (device, int32, each in [0,n) -- other values are skipped --, no
 * duplicates) lists the `count` coordinates to refresh; idx == NULL refreshes all n coordinates (device residency) or every
 * column currently held in a device slot (host residency), and count is then ignored.  Other
 * entries of z keep their (stale) values.  gap_sum (host, may be NULL): sum of the entries
 * written, the total gap when all were asked for; non-NULL makes the call wait.
 * Device residency, idx == NULL, and alpha, v, z untouched since duhl_set_data_* (no pass, no
 * duhl_set, no device pointer to them handed out): z still holds the gaps of set_data's own full
 * pass, and the call returns their sum without computing them again. */
duhl_status duhl_gap(duhl_ctx *ctx, const int32_t *idx, int64_t count, double *gap_sum);

/* duhl_gap for callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  No context: the caller passes every input and
 * output, and the per-workgroup partial sums of the pass (the only memory duhl_gap needs beyond
 * them) live in a static device array of DUHL_GAP_STATIC_MAX_GROUPS doubles (512 KB) that every GPU
 * the library runs on holds until the process ends.  The call allocates and frees nothing, waits
 * for nothing, and only enqueues kernels on `stream` (hipStream_t, NULL = the default stream).
 * Dense matrix in device memory only: A, ld, v (d floats), alpha (n floats), target (the labels y,
 * n floats, for DUHL_SVM; unused otherwise), idx / count as for duhl_gap (idx == NULL: all n).
 * lambda, eta (DUHL_ELASTIC_NET) as for duhl_set_data_dense / duhl_set_eta; bound: the Lasso's
 * B = ||b||^2 / (2 lambda d).  Outputs (device): z (n floats; entries not listed keep their values),
 * gap_sum (one double, may be NULL): the sum of the entries written.  All pointers are borrowed
 * for the duration of the enqueued work.
 * Limit: the pass may have at most DUHL_GAP_STATIC_MAX_GROUPS workgroups; a workgroup takes 4 to 32
 * coordinates (4 wavefronts of 1, 2, 4 or 8 columns each, by the rule duhl_create uses), so lists
 * of up to 262,144 coordinates always fit and up to 2,097,152 may; longer ones are refused with
 * DUHL_EINVAL.  err (host, err_len bytes, may be NULL) receives the text of an error.
 * Every call on a GPU uses that GPU's one array: calls that overlap on the same GPU (two streams,
 * two threads) race on it and their gap_sum is undefined; z is not affected.  The first call on a
 * device looks up the array's address (hipGetSymbolAddress): make it outside a graph capture. */
#define DUHL_GAP_STATIC_MAX_GROUPS 65536
duhl_status duhl_gap_dense_static(duhl_model model, int64_t d, int64_t n, const float *A, int64_t ld,
                                  const float *v, const float *alpha, const float *target,
                                  double lambda, double eta, double bound, const int32_t *idx,
                                  int64_t count, float *z, double *gap_sum, int device, void *stream,
                                  char *err, int64_t err_len);

/* Working-set selection (eq. (13)): the m coordinates with the largest z, ties to the smaller
 * index; 1 <= m <= min(n, budget_cols).  The set becomes the *pending* working set; with host
 * residency the columns it lacks are copied into free device slots on the copy stream while
 * the compute stream stays free for duhl_cd_epoch on the current set (Figure 2).  That overlap
 * needs budget_cols >= |current| + m; with fewer slots the copy first waits for the compute
 * stream and duhl_cd_epoch is refused (DUHL_ESTATE) until duhl_commit_swap.
 * P_out (device, m int32, may be NULL): the set in ascending order.  n_swapped (host, may be
 * NULL): columns that have to be copied (device residency: members that the current set lacks;
 * counted only when asked for).  rho (host, may be NULL): eq. (7) evaluated on z,
 * (mean of z over P)/(mean of z over all).  Non-NULL host outputs make the call wait for the
 * compute stream (not for the copies). */
duhl_status duhl_select(duhl_ctx *ctx, int64_t m, int32_t *P_out, int64_t *n_swapped,
                        double *rho);

/* Selection rules.  DUHL_SELECT_GAP is eq. (13) and what duhl_select does.  The other two are the
 * reference schemes the paper compares against: DUHL_SELECT_RANDOM draws a uniformly random
 * subset of size m (Section 5.1; arg = seed), DUHL_SELECT_BLOCK takes the arg-th contiguous block
 * of m coordinates, wrapping around at n (the sequential block scheme of Section 5.2). */
typedef enum { DUHL_SELECT_GAP = 0, DUHL_SELECT_RANDOM = 1, DUHL_SELECT_BLOCK = 2,
               DUHL_SELECT_RULE_ENUM_MAX = 0x7fffffff } duhl_select_rule;

/* duhl_select with a choice of rule; everything else (pending set, copies, outputs, rho of eq. (7)
 * evaluated on the gap memory z for the chosen set) as for duhl_select. */
duhl_status duhl_select_rule_apply(duhl_ctx *ctx, duhl_select_rule rule, uint64_t arg, int64_t m,
                                   int32_t *P_out, int64_t *n_swapped, double *rho);

/* Unit A's task in Algorithm 2 (for as long as unit B works on its block, A picks coordinates j and
 * stores their gaps at the round's starting point alpha^(t) in the gap memory, z_j = gap_j(alpha_j^(t))),
 * for a dense matrix with DUHL_RESIDENT_HOST.  duhl_host_sample_begin snapshots alpha and v at the
 * current point of the compute stream and starts nthreads host threads (1..256) that evaluate the
 * coordinate gaps of idx_host[0..count) (host, int32, each in [0,n)) from the matrix in host memory,
 * in list order, while the caller goes on enqueueing GPU work; the host link is not used.
 * duhl_host_sample_end stops them (wait_all == 0: after the column each is working on; != 0: after
 * the whole list), writes the refreshed entries into the gap memory z on the compute stream and
 * waits for that; n_done (host, may be NULL) = entries refreshed.  One round at a time per context;
 * the list must not repeat a coordinate. */
duhl_status duhl_host_sample_begin(duhl_ctx *ctx, const int32_t *idx_host, int64_t count, int nthreads);
duhl_status duhl_host_sample_end(duhl_ctx *ctx, int wait_all, int64_t *n_done);

/* The round boundary of Figure 2 (the point of Algorithm 2 where the refreshed memory of unit B
 * and the result of its update step meet): make the pending working set current.  The compute
 * stream waits (on the device, not the host) for the column copies, then later calls see the new set.  DUHL_ESTATE if nothing is
 * pending. */
duhl_status duhl_commit_swap(duhl_ctx *ctx);

/* One pass of exact coordinate steps over the current working set (Appendix D):
 *   Lasso:  gamma = alpha_j - a_j^T v/||a_j||^2,  alpha_j <- sign(gamma)[|gamma| - lambda d/||a_j||^2]_+
 *   SVM:    alpha_j <- y_j clip(y_j(alpha_j + (y_j - a_j^T v/(lambda n)) lambda n/||a_j||^2), 0, 1)
 *   e.net:  gamma = (alpha_j ||a_j||^2 - a_j^T v)/(||a_j||^2 + lambda eta d),
 *           alpha_j <- sign(gamma)[|gamma| - lambda d (1-eta)/(||a_j||^2 + lambda eta d)]_+
 *   both:   v <- v + a_j (alpha_j_new - alpha_j_old)
 * order (device, int32): the coordinates to visit, in visiting order; each must belong to the
 * current working set and, for the concurrent schemes, appear once (a repeated coordinate may be
 * solved by two workers at the same time, which leaves v inconsistent with alpha); values outside
 * [0,n) are skipped; n_order entries.
 * order == NULL: the whole set -- ascending for DUHL_CD_SEQUENTIAL, a pseudo-random permutation
 * drawn from (seed, pass counter) otherwise.
 * DUHL_CD_SEQUENTIAL solves one coordinate after the other and is reproducible.
 * The concurrent schemes solve up to max_inflight coordinates without seeing each other's update
 * of v -- the asynchrony of Appendix D, bounded.  max_inflight = 0 lets the library choose from
 * sigma(L), an estimate of the largest eigenvalue of an L-column Gram block made from the block
 * shape and the mean correlation of a column sample taken by duhl_set_data_*: the largest L with
 * sigma(L) <= 2 (concurrent exact steps still contract), or 2*count/sigma(count) capped at count/4
 * if that is more.  Strongly correlated columns tolerate fewer concurrent steps -- in particular
 * groups of near-duplicate columns that a selection by gap gathers, which the mean correlation does
 * not show.  DUHL_CD_ASYNC is therefore guarded on the device.  Each pass is judged as one step
 * from the old iterate to the new one: from sums that its own kernels form on the way -- <v, dv>,
 * ||dv||^2 and the change of the objective's terms in alpha -- the guard finds theta*, the point on
 * that line where a bound on the objective (exact in its quadratic part, the chord of its convex
 * terms in alpha) is smallest.  Sequential exact steps give theta* >= 1; k-fold overshoot of
 * colliding steps gives about 1/k, and below 1/2 the pass has raised the objective.  A pass with
 * theta* < 0.55 is scaled back to theta* -- v and the alpha_j it visited are blended with their old
 * values, so the objective never rises from pass to pass, whatever the data -- and counted, and the
 * bound on concurrent steps (the library's own, or max_inflight) is halved; it is doubled again
 * after 4 passes with theta* >= 0.8 and no damped one between them, then after 8, 16, ... (a level
 * that failed once is tried again ever later).  v is held in fp32: a pass whose ||dv||^2 does not stand clear of the
 * rounding of v (steps below about 1e-3 of ||v||, near convergence) cannot be judged this way;
 * it is undone only if the objective rose by more than 1e-6 of its value and otherwise changes
 * nothing in the books once a pass has been damped, so the bound found while the steps were large
 * stays in force.  The host
 * learns of a halving without waiting; in passes it had already enqueued with the old bound, part
 * of the workers sit each sub-pass out instead, so that such a pass solves a random half
 * (quarter, ...) of its working set.  After duhl_set_data_* the bound starts halved for the Lasso and
 * the elastic net (from alpha = 0 every coordinate moves and the first pass is the one that
 * overshoots), in full for the SVM dual.  duhl_cd_stats reports the counts.
 * DUHL_CD_ATOMIC is not guarded.
 *   DUHL_CD_ATOMIC  each step reads the live v and adds a_j*delta to it with fp32 atomics;
 *                   iterates depend on timing.
 *   DUHL_CD_ASYNC   dense data: the pass is cut into sub-passes of max_inflight coordinates;
 *                   workers solve their share one after the other against a private copy of v and
 *                   the changes are merged after each sub-pass (no atomics, reproducible for a
 *                   given seed).  Columns of more than 53,248 entries are solved by workers that
 *                   span several compute units and wait for each other once per coordinate; that
 *                   wait is bounded, and if it ever expires (the device shared with work that
 *                   starves part of a worker for seconds) the pass ends early, alpha and v are
 *                   undefined and the next call that returns a scalar fails with DUHL_EHIP until
 *                   the data are set again.
 *                   Sparse data: sub-passes of max_inflight coordinates, one kernel launch each;
 *                   the steps of a sub-pass run concurrently, read v as the sub-passes before it
 *                   left it (or fresher) and add to it with fp32 atomics; iterates depend on timing.
 * In all schemes v = A alpha (- b) keeps holding up to fp32 rounding. */
duhl_status duhl_cd_epoch(duhl_ctx *ctx, duhl_cd_mode mode, const int32_t *order,
                          int64_t n_order, uint64_t seed, int max_inflight);

/* The guard of DUHL_CD_ASYNC (see duhl_cd_epoch), since the data were set: passes_damped = passes
 * scaled back (or undone) because their steps overshot; inflight_now = the bound on concurrent steps
 * the library would choose now for a pass over the current working set (max_inflight = 0);
 * steps_kept = coordinate steps taken by the passes that were not undone (a pass enqueued before the
 * host knew of a halving solves only part of its working set, see duhl_cd_epoch; dense data:
 * counted, sparse data: the pass's length less the share that sat out); last_theta = theta* of the
 * last guarded pass (1 if it could not be judged).  All host, each may be NULL.
 * Waits for the compute stream. */
duhl_status duhl_cd_stats(duhl_ctx *ctx, int64_t *passes_damped, int64_t *inflight_now, int64_t *steps_kept,
                          double *last_theta);

/* The outer loop, run natively: Algorithm 1 with the selection of eq. (11) when every gap is
 * refreshed each round, Algorithm 2 (selection by eq. (13) on a gap memory that may be stale,
 * columns copied beside the passes) otherwise.  One round is
 *     refresh gap memory -> select m (rule, seed + round) -> `passes` x duhl_cd_epoch(mode) -> commit
 * with the commit before the passes when the copies cannot overlap them (device residency, first
 * round, or fewer than |current| + m slots).  What a round refreshes:
 *   device residency, no sample list:  all n gaps (the working set is the exact top m);
 *   device residency with sample_dev:  the current working set and this round's window of the list;
 *   host residency:  every column held in a device slot, plus this round's window of the list --
 *                    evaluated by the GPU over the host link (sample_dev), or by host_threads host
 *                    threads from host memory while the passes run (sample_host, Algorithm 2
 *                    unit A's loop; their result enters the gap memory at the end of the round).
 * The window is sample_per_round consecutive entries of the list (sample_len entries, each in
 * [0,n), no duplicates), advancing and wrapping from round to round.
 * Every check_every-th round (0 = 1) the sum of the gap memory as the selection saw it is read
 * back (this waits for the compute stream): with all gaps fresh it is the duality gap of eq. (2),
 * otherwise an estimate from stale entries, which is not trusted before the windows have covered
 * the whole list once.  The loop ends when it is <= gap_tol (pass a negative gap_tol to run
 * max_rounds rounds; see `confirm`) or after max_rounds rounds, and waits for the compute stream.
 * Requires data, no pending selection; 1 <= m <= min(n, budget_cols). */
typedef struct duhl_run_opts {
    int64_t m;                  /* working-set size                                              */
    int passes;                 /* theta of Section 5.2: passes per round, >= 1.  0: chosen by the loop --
                                   the first round runs one pass and times its two phases (refresh +
                                   selection: G, one pass: C); from the second round on
                                   round(sqrt(G/C)) + 1 passes, at most 8 (a selection that costs many
                                   passes is worth several of them, cf. Section 5.2); host residency: 8 */
    duhl_cd_mode mode;
    int max_inflight;           /* as for duhl_cd_epoch                                          */
    duhl_select_rule rule;
    uint64_t seed;
    int64_t max_rounds;
    double gap_tol;
    int check_every;
    const int32_t *sample_dev;  /* device list, or NULL                                          */
    const int32_t *sample_host; /* the same list in host memory (only read when host_threads > 0) */
    int64_t sample_len, sample_per_round;
    int host_threads;           /* 0: the GPU evaluates the window                               */
    int confirm;                /* != 0 with a sample list: when the estimate passes gap_tol, refresh
                                   all n gaps (host residency: one pass over the host link), test
                                   their sum -- the true total gap -- and go on if it fails.  Host
                                   residency without a sample list always confirms: the columns
                                   outside the device slots are never refreshed otherwise        */
    int adapt_inflight;         /* != 0 (concurrent modes): on every checked round read the objective;
                                   exact steps never raise it, so if it rose the concurrent steps
                                   collided -- alpha and v go back to the last checked round that was
                                   fine and max_inflight is halved for the rest of the run        */
    int host_wait_all;          /* host_threads > 0: != 0 lets the threads finish the round's whole
                                   window before the round ends (reproducible rounds: which entries
                                   are refreshed no longer depends on timing); 0 stops them when the
                                   passes and copies are done, as unit A is stopped in Algorithm 2 */
    int max_extra_passes;       /* host residency, copies running beside the passes: after the round's
                                   `passes`, up to this many more, one at a time, for as long as the
                                   round's column copies are still in flight (theta sized to the copy,
                                   Section 5.2: unit B works on until its next working set has arrived).
                                   0: none */
} duhl_run_opts;

typedef struct duhl_run_stats {
    int64_t rounds;             /* rounds whose passes were run                                  */
    int64_t passes;             /* passes run in total                                           */
    int converged;              /* 1 if the loop ended on gap_tol                                */
    int confirmations;          /* full refreshes made to confirm the estimate                   */
    double gap_memory_sum;      /* sum of the gap memory at the last check                       */
    double rho;                 /* eq. (7) at the last check                                     */
    int64_t columns_swapped;    /* columns copied into slots, summed over the checked rounds     */
    int64_t host_sampled;       /* gap-memory entries refreshed by host threads                  */
    double seconds;             /* wall time of the call                                         */
    int inflight_halvings;      /* times adapt_inflight went back and halved the bound           */
    int inflight_last;          /* max_inflight in force at the end (0: the library's own bound) */
    int passes_per_round;       /* passes per round in force at the end (what passes = 0 chose)  */
} duhl_run_stats;

duhl_status duhl_run(duhl_ctx *ctx, const duhl_run_opts *opts, duhl_run_stats *stats);

/* O(alpha) from the stored v and alpha (Appendix C).  objective: host.  Waits. */
duhl_status duhl_objective(duhl_ctx *ctx, double *objective);

/* v := A alpha - b (Lasso) or A alpha (SVM) from scratch; removes the rounding drift of many
 * atomic adds.  Reads every column with alpha_j != 0 (from the host when not in a slot). */
duhl_status duhl_recompute_v(duhl_ctx *ctx);

/* Copy state to / from host memory (fp32; DUHL_P: int32, the current working set).  len must
 * be n (ALPHA, Z, SQNORM), d (V) or the working-set size (P, see duhl_working_set_size).
 * Both wait for the compute stream.  duhl_set accepts ALPHA, V and Z only. */
duhl_status duhl_get(duhl_ctx *ctx, duhl_what what, void *dst_host, int64_t len);
duhl_status duhl_set(duhl_ctx *ctx, duhl_what what, const void *src_host, int64_t len);

/* Device address of a state array, for callers that keep their own views (borrowed). */
duhl_status duhl_device_ptr(duhl_ctx *ctx, duhl_what what, void **ptr);

/* Measurement aid, no part of the method: read `bytes` (a multiple of 16) of device memory at
 * dev (16-byte aligned) `reps` times with a plain streaming kernel on the compute stream and
 * return the shortest launch time in milliseconds.  It is the yardstick the gap pass (Section 3,
 * eq. (4): one read of every column) is compared with: what a read-only pass over the same
 * memory can reach on the device at hand.  Waits. */
duhl_status duhl_probe_stream_read(duhl_ctx *ctx, const void *dev, int64_t bytes, int reps,
                                   double *best_ms);

/* Measurement aid, no part of the method: `ops` (rounded up to a multiple of the grid) fp32 atomic
 * adds of +0 to pseudo-random elements of v -- which leave v as it is -- `reps` times on the
 * compute stream; adds_per_s (host) = the best rate.  It is the yardstick of the concurrent pass on
 * CSR data (Appendix D's update of v, one atomic add per non-zero of a step's row): the device
 * performs such adds at a fixed rate however many threads issue them, and a pass cannot take less
 * than its non-zeros divided by that rate.  Waits.  DUHL_ESTATE before the data are set. */
duhl_status duhl_probe_scatter_add(duhl_ctx *ctx, int64_t ops, int reps, double *adds_per_s);

/* The threshold of the last selection (eq. (13)): the smallest score among the selected
 * coordinates -- for DUHL_SELECT_GAP the m-th largest entry of the gap memory z as the selection
 * saw it (entries equal to it are taken in index order until m are chosen).  threshold: host.
 * Waits.  DUHL_ESTATE before the first selection. */
duhl_status duhl_selection_threshold(duhl_ctx *ctx, float *threshold);

/* Columns that duhl_gap(NULL) refreshes at the speed of device memory: with host residency the
 * number of device slots in use (the working set, and earlier members that have not been evicted
 * yet); n with device residency.  count: host.  Waits; meant for reports, not for the round loop. */
duhl_status duhl_resident_columns(duhl_ctx *ctx, int64_t *count);

/* The column swap of the last committed selection (host residency): how many columns were copied into
 * device slots and how long the copy stream took over them, from the moment it could start (the
 * plan was made, and in-place replacement had waited for the passes) to the last copy -- with
 * DUHL_RESIDENT_HOST_PAGEABLE this includes the host threads' staging.  columns, copy_ms: host.
 * Waits for both streams; meant for reports.  DUHL_ESTATE while a selection is pending or before
 * the first one. */
duhl_status duhl_swap_stats(duhl_ctx *ctx, int64_t *columns, double *copy_ms);

/* Size of the current working set (0 before the first commit). */
int64_t duhl_working_set_size(const duhl_ctx *ctx);

/* Text of the last error of this context ("" if none); valid until the next call on it. */
const char *duhl_last_error(const duhl_ctx *ctx);

/* Release everything the library allocated.  NULL is allowed. */
void duhl_destroy(duhl_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* DUHL_H */
