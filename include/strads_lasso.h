/*
 * strads_lasso.h -- C ABI of the MI355X (gfx950) library for one hot path:
 * scheduling rounds of SAP/STRADS-scheduled parallel coordinate descent for the
 * Lasso (Lee, Kim, Ho, Gibson, Xing, "Structure-Aware Dynamic Scheduler for
 * Parallel Machine Learning", Section 2.1: Algorithm 1, eq. (1), eq. (2)).
 *
 * Problem (eq. (1) with squared loss):  min_beta  1/2 ||y - X beta||^2 + lambda ||beta||_1
 * over a design X (N rows, J columns) whose columns are standardised to unit
 * l2 norm (dense designs: also zero mean), no intercept.
 *
 * One round (Algorithm 1's loop body, Steps 1-4 of Section 2.1):
 *   1. draw P' = l_prime distinct candidate coordinates, probability proportional
 *      to (delta beta_j)^2 + eta           (Step 1 with Theorem 1's squared weight)
 *   2. candidate dependencies |x_a^T x_b|; walk the candidates in draw order and
 *      keep one iff its dependency with everything kept so far is < rho   (Step 2)
 *   3. for every kept j, from the SAME residual r = y - X beta:
 *        beta_j <- S(x_j^T r + beta_j, lambda)                         (eq. (2))
 *   4. r <- r - sum_j x_j * (change of beta_j);  delta beta_j <- |change|  (Step 4)
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE are HIP device addresses on the GPU that is current
 *     when the call is made; pointers marked HOST are ordinary host memory.
 *   - The library never allocates or frees device memory: the caller supplies one
 *     workspace (size from strads_lasso_workspace_bytes) and owns X, y and the
 *     stream.  All of them are borrowed and must outlive the handle.  X and y
 *     are never written.
 *   - Every function returns STRADS_OK (0) or a negative STRADS_E_* code; on
 *     error no output argument is written.  Nothing aborts or throws.
 *   - Work is enqueued on the caller's stream.  Calls on one handle must not
 *     overlap (the handle's workspace is shared state).  A handle with n_shards > 1 also owns
 *     n_shards - 1 streams of its own (default priority, created at create, destroyed at destroy):
 *     every call that enqueues rounds makes them wait for the caller's stream first and makes the
 *     caller's stream wait for them before it returns, so from outside the work is still ordered
 *     as if it ran on the caller's stream; the shards overlap within one strads_lasso_run call.
 */
#ifndef STRADS_LASSO_H
#define STRADS_LASSO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STRADS_OK                     0
#define STRADS_E_INVALID_ARG         -1
#define STRADS_E_WORKSPACE_TOO_SMALL -2
#define STRADS_E_HIP                 -3   /* a HIP runtime call or kernel launch failed */
#define STRADS_E_DIVERGED            -4   /* objective is not finite: updating correlated coordinates together (rho too
                                             large, or no dependency check) can make the iteration blow up */
#define STRADS_E_UNSUPPORTED         -5
#define STRADS_E_TOO_LARGE           -6   /* a size exceeds the fixed maximum of an entry point that allocates nothing */

#define STRADS_LAYOUT_DENSE_COLMAJOR  0   /* x[j*n + i] = X_ij, fp32, leading dimension n */
#define STRADS_LAYOUT_CSC             1   /* values / row_idx / col_ptr */
#define STRADS_LAYOUT_GENO2           2   /* genotype counts in {0,1,2}, 2 bits each, with a mean and a scale per
                                             column: X_ij = fl(fl(g_ij - col_mean[j]) * col_scale[j]), both
                                             operations rounded to fp32.  x points at 32-bit words: column j
                                             starts at word j * geno_words(n); word w of a column holds rows
                                             16w .. 16w+15, row 16w+e in bits 2e, 2e+1; rows past n hold 0.
                                             geno_words(n) = 4 * ceil(n / 64) (columns are 16-byte aligned).
                                             16 times fewer bytes than fp32 for every pass over X. */

#define STRADS_MAX_L_PRIME         8192   /* largest supported candidate count per round */
/* Loss function of eq. (1) (Section 2.1 allows the squared and the logistic loss).
 *   SQUARED   L = 1/2 ||y - X beta||^2; the state vector r kept between rounds is the residual
 *             y - X beta, and eq. (2) is beta_j <- S(x_j^T r + beta_j, lambda).
 *   LOGISTIC  L = sum_i log(1 + exp(-y_i x_i^T beta)) with labels y_i in {-1, +1} (not checked).  The
 *             paper gives no formula; a coordinate step minimises the quadratic upper bound of
 *             curvature 1/4 (unit-norm columns): beta_j <- S(beta_j + 4 x_j^T w, 4 lambda) with
 *             w_i = y_i / (1 + exp(y_i x_i^T beta)).  The state vector r is -X beta (zero at start),
 *             maintained by the same residual update; "z" in strads_lasso_last_round is x_j^T w, and
 *             the optimality test uses g = X^T w. */
#define STRADS_LOSS_SQUARED  0
#define STRADS_LOSS_LOGISTIC 1

#define STRADS_MAX_SHARDS             8   /* largest supported number of scheduler shards */

/* Stages of one round, in stream order, as timed by strads_lasso_stage_times */
#define STRADS_STAGE_SAMPLER     0   /* Step 1: keys, top-P' selection, draw order */
#define STRADS_STAGE_CAND_DOTS   1   /* dynamic dependencies only: x_j^T r and the tentative change of
                                        every candidate, and the list of those that would move */
#define STRADS_STAGE_GRAM_TILES  2   /* Step 2: candidate Gram, MFMA tile kernel (K-slices) */
#define STRADS_STAGE_GRAM_MASK   3   /* Step 2: K-slice sum and |g| < rho conflict bits */
#define STRADS_STAGE_FILTER      4   /* Step 2: greedy choice of B_1 (dynamic dependencies: and its commit) */
#define STRADS_STAGE_UPDATE      5   /* eq. (2): x_j^T r for B_1, soft-threshold, bookkeeping (nothing with
                                        dynamic dependencies or "dots_with_gram": done in earlier stages) */
#define STRADS_STAGE_RESIDUAL    6   /* r <- r - X_B * change */
#define STRADS_N_STAGES          7

/* Dependency rule of Step 2 */
#define STRADS_DEPS_STATIC        0  /* Algorithm 1: d(a,b) = |x_a^T x_b| for every candidate pair */
#define STRADS_DEPS_DYNAMIC       1  /* Section 1 "Dynamic Block Structures" / Step 4: a candidate whose
                                        coefficient would not change this round (its update from the
                                        current residual is zero) has no dependency with anyone;
                                        d(a,b) = |x_a^T x_b| only between two candidates that both move.
                                        The Gram and the greedy walk then run over the movers only. */
#define STRADS_DEPS_NONE          2  /* no dependency check: the first p_max candidates of the draw (all of
                                        them if p_max = 0) are updated together.  With the uniform priority
                                        this is the Shotgun scheduler Section 5.1 compares against. */

/* Priority of Step 1: the draw takes coordinate j with probability proportional to */
#define STRADS_PRIORITY_SQUARED   0  /* (delta beta_j)^2 + eta   (Theorem 1) */
#define STRADS_PRIORITY_LINEAR    1  /* |delta beta_j| + eta     (Algorithm 1 and Step 1 as printed) */
#define STRADS_PRIORITY_UNIFORM   2  /* 1: no priority.  With STRADS_DEPS_STATIC this is the "static
                                        correlation" scheduler of Section 5.1. */

typedef struct strads_lasso strads_lasso_t;   /* opaque, host side */

typedef struct {
    int64_t        n;             /* rows N (> 0) */
    int64_t        j;             /* columns J (> 0, < 2^31) */
    int32_t        layout;        /* STRADS_LAYOUT_* */
    const float   *x;             /* DEVICE. dense: n*j values, column-major; CSC: nnz values;
                                     GENO2: the packed words (cast), 16-byte aligned */
    const int32_t *row_idx;       /* DEVICE, CSC only: nnz row indices, increasing within a column.  CSC sums are kept in
                                     2^-40 fixed point: |x_a^T x_b| must stay below 2^22 and every |value * change of
                                     beta_j| of a round below 2^22 / |B_1| (at least 512; unit-norm columns and a
                                     converging iteration are far inside); a residual update that leaves the range
                                     writes NaN into r, which strads_lasso_run reports as STRADS_E_DIVERGED */
    const int64_t *col_ptr;       /* DEVICE, CSC only: j+1 offsets, col_ptr[0] = 0 */
    const float   *col_mean;      /* DEVICE, GENO2 only: j column means */
    const float   *col_scale;     /* DEVICE, GENO2 only: j column scales (1 / l2 norm of the centred column) */
    const float   *y;             /* DEVICE, n values */
    float          lambda;        /* regularisation weight of eq. (1), >= 0, finite */
    float          rho;           /* dependency threshold of Step 2, > 0 */
    float          eta;           /* priority floor of Algorithm 1, >= 1e-30 */
    float          c_init;        /* Algorithm 1's large initial constant C: initial delta beta (> 0) */
    int32_t        l_prime;       /* P': candidates per round, 1..STRADS_MAX_L_PRIME; clamped to j */
    int32_t        p_max;         /* P: cap on the kept set; 0 = keep every admissible candidate */
    uint64_t       seed;          /* keys the counter-based random stream with (round, j) */
    int32_t        keep_gram;     /* nonzero: also store the full fp32 candidate Gram of the last
                                     round so strads_lasso_last_round can return it (costs
                                     4*L^2 bytes of workspace and one extra write per round) */
    int32_t        max_col_nnz;   /* CSC only: an upper bound (>= 1) on the nonzeros of any column;
                                     sizes the per-round inverted index; checked at create */
    int32_t        deps;          /* STRADS_DEPS_*: dependency rule of Step 2 */
    int32_t        priority;      /* STRADS_PRIORITY_*: weight of Step 1's draw */
    int32_t        n_shards;      /* S scheduler shards taking turns (Section 3): coordinate j belongs to
                                     shard j mod S for good, round t is shard (t mod S)'s turn and draws its
                                     candidates (l_prime clamped to floor(j / S)) from that shard only.
                                     0 or 1: one scheduler.  With S > 1 the shards' scheduling work
                                     (draw, Gram, greedy walk) runs on library-owned streams concurrently;
                                     the updates are applied in round order.  At most STRADS_MAX_SHARDS. */
    int32_t        loss;          /* STRADS_LOSS_*: the loss L of eq. (1) */
    void          *workspace;     /* DEVICE, 256-byte aligned, caller-allocated */
    size_t         workspace_bytes;
    void          *stream;        /* hipStream_t owned by the caller (NULL = the default stream) */
} strads_lasso_config_t;

typedef struct {
    int64_t round;                /* index t of the round this describes (0-based) */
    int32_t n_cand;               /* |U|  = min(l_prime, j) */
    int32_t n_kept;               /* |B_1| */
    int32_t n_moved;              /* kept coordinates whose beta changed */
    int32_t near_rho_pairs;       /* candidate pairs with | |x_a^T x_b| - rho | <= 1e-6 */
    float   max_abs_delta;        /* max |change of beta_j| over the kept set */
} strads_round_info_t;

typedef struct {
    int64_t rounds_done;          /* rounds executed by this call */
    int64_t updates_done;         /* sum of |B_1| over those rounds */
    double  objective;            /* eq. (1) at exit */
    float   kkt_violation;        /* max_j violation at the last check (absolute) */
    int32_t converged;            /* 1 iff kkt_violation <= kkt_tol * lambda at exit */
    int32_t graph_replays;        /* HIP-graph launches this call made (each = "graph_rounds" rounds) */
} strads_run_info_t;

/* Bytes of workspace a configuration needs (depends on n, j, layout, l_prime, keep_gram, deps, n_shards
 * and, for CSC, max_col_nnz only; pointers in cfg are ignored).  Makes no device call.
 * Returns 0 if cfg is NULL or a size field is invalid. */
size_t strads_lasso_workspace_bytes(const strads_lasso_config_t *cfg);

/* Validate cfg, carve the workspace and enqueue Algorithm 1's initialisation:
 * beta = 0, delta beta = c_init for every j, r = y, round counter = 0.  For a CSC design it also
 * checks col_ptr (starts at 0, non-decreasing, no column above max_col_nnz) on the device and
 * waits for that check; row indices must lie in [0, n) and are not checked.
 * *out receives a host-side handle (free it with strads_lasso_destroy). */
int strads_lasso_create(const strads_lasso_config_t *cfg, strads_lasso_t **out);

/* Enqueue one round (Algorithm 1's loop body) on the stream.  info == NULL: returns
 * without synchronising.  info != NULL (HOST): waits for the round and fills it. */
int strads_lasso_round(strads_lasso_t *h, strads_round_info_t *info);

/* Run rounds until max_rounds have been done or, every check_every rounds
 * (check_every <= 0: never), the optimality violation of eq. (1)
 *   v_j = max(|x_j^T r| - lambda, 0)            if beta_j == 0
 *       = |x_j^T r - lambda * sign(beta_j)|     otherwise
 * satisfies max_j v_j <= kkt_tol * lambda.  Synchronises at each check and at
 * exit.  out (HOST, may be NULL) receives the summary.  Returns STRADS_E_DIVERGED
 * if the objective at exit is not finite. */
int strads_lasso_run(strads_lasso_t *h, int64_t max_rounds, float kkt_tol, int32_t check_every,
                     strads_run_info_t *out);

/* Objective of eq. (1) at the current state, 1/2 sum r_i^2 + lambda sum |beta_j|,
 * accumulated in fp64 from the fp32 state.  Synchronises.  out is HOST. */
int strads_lasso_objective(strads_lasso_t *h, double *out);

/* max_j v_j (see strads_lasso_run) at the current state.  Streams all of X once.
 * Synchronises.  max_violation is HOST.  g_or_null (DEVICE, j floats, may be
 * NULL) receives x_j^T r for every column. */
int strads_lasso_kkt(strads_lasso_t *h, float *max_violation, float *g_or_null);

/* Copy the solver state out of / into the handle.  All pointers DEVICE
 * (beta, dbeta: j floats; r: n floats); any may be NULL to skip it.  round is
 * HOST.  The random stream is a pure function of (seed, round, j), so a state
 * restored with its round index continues exactly. */
int strads_lasso_get_state(strads_lasso_t *h, float *beta, float *dbeta, float *r, int64_t *round);
int strads_lasso_set_state(strads_lasso_t *h, const float *beta, const float *dbeta, const float *r,
                           int64_t round);

/* Stage outputs of the most recent round, for parity checks.  Output arrays are
 * DEVICE and sized for l_prime entries (gram_or_null: n_cand*n_cand floats,
 * row-major, only when the handle was created with keep_gram); any may be NULL.
 * cand: candidates in draw order; kept_pos: positions into cand of the kept set
 * (increasing); z: x_j^T r per kept coordinate; delta: change of beta_j per kept
 * coordinate.  n_cand / n_kept are HOST.  Synchronises.
 * With dynamic dependencies the Gram holds x_a^T x_b for pairs of movers and 0 elsewhere. */
int strads_lasso_last_round(strads_lasso_t *h, int32_t *cand, int32_t *kept_pos, float *z, float *delta,
                            float *gram_or_null, int32_t *n_cand, int32_t *n_kept);

/* Dynamic dependencies only: per candidate of the most recent round (DEVICE arrays of l_prime
 * floats, any may be NULL) z_cand = x_j^T r and delta_cand = the change its update would make
 * (S(z + beta_j, lambda) - beta_j; nonzero = "moves"); n_movers is HOST.  Synchronises.
 * Returns STRADS_E_UNSUPPORTED on a handle with static dependencies. */
int strads_lasso_last_candidates(strads_lasso_t *h, float *z_cand, float *delta_cand, int32_t *n_movers);

/* Stage entry: the sampling keys log2(w_j) - log2(-log2 u_j) of Step 1 that round
 * `round` would use with the current delta beta (j floats, DEVICE). */
int strads_lasso_stage_keys(strads_lasso_t *h, int64_t round, float *keys_out);

/* Stage entry: run only the dependency filter of Step 2 on a caller-supplied
 * Gram.  gram: DEVICE, l*l floats row-major (symmetric), 1 <= l <= l_prime.
 * kept_pos: DEVICE, l ints.  n_kept: HOST.  Uses the handle's rho and p_max and
 * overwrites the handle's last-round filter outputs.  Synchronises. */
int strads_lasso_stage_filter(strads_lasso_t *h, const float *gram, int32_t l, int32_t *kept_pos,
                              int32_t *n_kept);

/* For callers that cannot allocate device memory or let a library do it (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it): the dependency filter of strads_lasso_stage_filter without a
 * handle and without a workspace.  The conflict bitmask and the other scratch of its kernels live in a
 * file-scope device array inside the library, STRADS_FILTER_STATIC_MAX_L^2 / 8 bytes + 64 KiB + 256 bytes
 * (8.06 MiB), which every GPU the library runs on holds until the process ends.  The call makes no
 * allocation of any kind and does not synchronise: it enqueues three kernels on `stream` and returns.
 *   gram      DEVICE, l*l floats row-major, symmetric (only |gram[a][b]| < rho is looked at, a != b)
 *   l         1 .. STRADS_FILTER_STATIC_MAX_L; larger: STRADS_E_TOO_LARGE, nothing enqueued
 *   rho       > 0; p_max >= 0 (0 = no cap)
 *   kept_pos  DEVICE, room for l ints: receives the kept positions in increasing order
 *   n_kept    DEVICE, one int: how many
 *   stream    hipStream_t of the caller (NULL = the default stream); outputs are valid once the work
 *             enqueued on it has finished
 * All calls on one GPU share that GPU's array: calls that overlap in time on the same GPU (different
 * streams or threads) race and must be serialised by the caller.  The first call on a device looks up the
 * array's address there (make it outside a graph capture).  On error no output is written. */
#define STRADS_FILTER_STATIC_MAX_L 8192
int strads_lasso_filter_static(const float *gram, int32_t l, float rho, int32_t p_max, int32_t *kept_pos,
                               int32_t *n_kept, void *stream);

/* Launch-shape knobs for measurement sweeps (never change results except the
 * fp32 summation order of the Gram when split_k changes, and of the residual update):
 *   "gram_split_k"  0 = automatic, else the number of K-slices per Gram tile
 *   "select_cap"    boundary-list length above which the sampler's final
 *                   selection falls back to its multi-pass path (default 4096)
 *   "graph_rounds"  > 0: strads_lasso_run records this many consecutive rounds once as a HIP graph and
 *                   replays it (rounds left over are enqueued one by one); 0 (default) = never.
 *                   Replays and directly enqueued rounds give identical results.  Needs a caller
 *                   stream that can be captured (not the legacy default stream); otherwise the
 *                   library falls back to enqueueing.  On ROCm 7.2 a replay runs the shards'
 *                   branches one after the other, so it only pays for n_shards = 1.
 *   "gram_xcd_map"  1 (default): the Gram tile kernel's workgroups are numbered so that those sharing an
 *                   L2 (one of the eight XCDs) work on the same K-slices; 0: tile by tile.  Results are
 *                   identical.  Dense and packed designs with static or no dependencies only.
 *   "gram_tile256"  how Step 2's Gram is tiled.  1 (default): lists of more than 4096 candidates over 16-byte
 *                   aligned fp32 columns of at least 4096 rows, under Algorithm 1's dependency rule (and shorter
 *                   lists over columns long enough that every compute unit gets at least 180 stages of 32
 *                   rows of a tile to multiply), are
 *                   multiplied in 256 x 256 tiles handed out from a queue (strads_lasso_gram256_plan); every
 *                   other shape in 128 x 128 tiles with K-slices.  0: always 128 x 128.  2: 256 x 256 wherever
 *                   the design is fp32, aligned and the rule static (STRADS_E_UNSUPPORTED if the workspace
 *                   lacks room for the tile slots).  The routes differ in fp32 summation order only.
 *   "gram_direct"   1 (default): under Algorithm 1's dependency rule, the Gram of a long list over short columns
 *                   (at most 1024 rows and at least 1024 candidates, or at most 2048 rows and at least 3072
 *                   candidates; dense fp32 or packed designs) is multiplied in 64 x 64 tiles that run over all
 *                   rows and write the conflict bits themselves: no K-slices and no second kernel that sums
 *                   them.  0: never.  2: for every list of such a design (STRADS_E_UNSUPPORTED where the rule is
 *                   not Algorithm 1's, the design is sparse, the 256 x 256 tiles are in use or "gram_split_k"
 *                   is set).  The routes differ in fp32 summation order only.
 *   "dots_with_gram" 1 (default): fp32 dense designs with l_prime <= 4096, Algorithm 1's dependency rule and
 *                   one scheduler take x_j^T r for every candidate in extra workgroups of the Gram
 *                   launch, and the filter's workgroup applies eq. (2) to the kept ones; 0: a kernel
 *                   after the filter takes the products for the kept set only.  Identical results.
 *   "early_keys"     1 (default): when rounds are enqueued back to back (strads_lasso_run) with one scheduler,
 *                   the launch of the round's last kernel (of the residual update) also carries the next
 *                   round's key pass; 0: every round starts with its own
 *                   key pass.  Identical results.
 *   "residual_fused" 1 (default): dense designs apply r -= X_B delta_B in one kernel where one exists for the
 *                   shape (l_prime <= 4096; more than 1024 candidates over 16-byte aligned columns of at least
 *                   32768 rows);
 *                   0: always the two-stage update (partial sums per column group, then their sum).  The
 *                   routes differ in fp32 summation order only.
 *   "profile_level", "profile_rounds"   see strads_lasso_stage_times
 * Returns STRADS_E_INVALID_ARG for an unknown name or a value out of range. */
int strads_lasso_set_tuning(strads_lasso_t *h, const char *name, int64_t value);

/* Host only, no GPU call: the work queue of the tile kernel for long candidate lists (Section 2.1, Step 2: the
 * pairwise dependencies of the P' candidates; see "gram_tile256") for l candidates over n rows.  The Gram's upper
 * triangle is cut into tiles of 256 x 256 entries and every tile's n rows into stages of 32; an item of the
 * queue is a stage range of one tile.  Items shrink as the queue empties (whole tiles first, 32 stages at the
 * end) and workgroups take them in order as they become free; each item is written to a tile slot of its own
 * and a tile's slots are consecutive, in row order.
 *   n_items     HOST int32: number of items (= tile slots)
 *   items       HOST int32 [items_cap][5]: (tile row, tile column, first stage, end stage, slot) of the first
 *               items_cap items in queue order; may be NULL if items_cap is 0
 *   first_slot, n_slots   HOST int32 [T][T], T = ceil(l / 256): slot range of each tile (0, 0 below the diagonal) */
int strads_lasso_gram256_plan(int64_t n, int32_t l, int32_t items_cap, int32_t *n_items, int32_t *items,
                              int32_t *first_slot, int32_t *n_slots);

/* Host only, no GPU call: the tile kernel that Step 2's Gram (Section 2.1, Step 2: the pairwise dependencies of
 * the P' candidates) of l candidates over n rows takes by default, for a design of the given layout
 * (STRADS_LAYOUT_*) under the given dependency rule (STRADS_DEPS_*): edge (HOST int32) as
 * strads_lasso_gram_tile_edge reports it.  A handle may differ: fp32 columns that are not 16-byte aligned never
 * take the 256 x 256 tiles, and tunings ("gram_tile256", "gram_direct", "gram_split_k") override the default.
 * STRADS_E_INVALID_ARG for n < 1, l outside 1 .. STRADS_MAX_L_PRIME, an unknown layout or rule, or a NULL edge. */
int strads_lasso_gram_default_tile_edge(int64_t n, int32_t l, int32_t layout, int32_t deps, int32_t *edge);

/* Which tile kernel forms Step 2's Gram for this handle as it is tuned now: edge (HOST int32) = 256 (tiles of
 * 256 x 256 from a queue, see "gram_tile256"), 128 (tiles of 128 x 128 with K-slices), 64 (tiles of 64 x 64 over
 * all rows, see "gram_direct"), or 0 (a sparse design or no dependency check: no tile kernel). */
int strads_lasso_gram_tile_edge(strads_lasso_t *h, int32_t *edge);

/* Average duration in milliseconds of each stage (HOST array of STRADS_N_STAGES floats) over the
 * rounds enqueued since profiling was switched on or since the last call, measured with HIP events
 * recorded on the handle's stream.  Switch on with strads_lasso_set_tuning(h, "profile_level", v):
 * v = 1 records only around the Gram tile kernel (other entries read 0), v = 2 records every stage
 * boundary, v = 0 switches off.  "profile_rounds" (default 256, set it while profiling is off) is the
 * number of rounds the event pool holds; later rounds are not recorded.  Synchronises and resets
 * the pool.  rounds_timed is HOST. */
int strads_lasso_stage_times(strads_lasso_t *h, float *avg_ms, int32_t *rounds_timed);

/* Duration in milliseconds (HOST float) of the most recent pass over all columns (strads_lasso_kkt,
 * or a check inside strads_lasso_run), from HIP events recorded around its kernels on the handle's
 * stream: the kernels alone, without the read-back of the result.  0 if profiling ("profile_level")
 * was off during that pass or no pass has been made. */
int strads_lasso_last_kkt_ms(strads_lasso_t *h, float *ms);

void strads_lasso_destroy(strads_lasso_t *h);

/* 1 if the library was built as a debug build (-DSTRADS_DEBUG_SYNC), else 0.  A debug build waits for the
 * stream and checks the error state after every kernel launch, so that a failing kernel is reported by the
 * call that launched it (every call then synchronises; "graph_rounds" is refused), and
 * strads_lasso_create checks the unit-norm precondition: a design with a column whose l2 norm differs from
 * 1 by more than 1e-3 is rejected with STRADS_E_INVALID_ARG (one pass over the design). */
int strads_lasso_debug_build(void);

const char *strads_lasso_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* STRADS_LASSO_H */
