// Internal declarations shared by the HIP translation units of libstrads_lasso.
// Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "strads_lasso.h"

namespace strads {

constexpr int kHistBins = 2048;        // 11-bit digits of the orderable 32-bit key
constexpr int kGramTile = 128;         // candidate-Gram output tile edge (per workgroup)
#ifndef STRADS_GRAM_KT
#define STRADS_GRAM_KT 32
#endif
#ifndef STRADS_GRAM_OCC
#define STRADS_GRAM_OCC 2
#endif
constexpr int kGramKT = STRADS_GRAM_KT;   // K (row) extent of one LDS stage, floats (16 or 32)
constexpr int kGramOcc = STRADS_GRAM_OCC; // Gram workgroups resident per compute unit (LDS and registers allow it)
constexpr int kMaxResidualGroups = 64; // column groups of the residual update
constexpr int kObjBlocks = 256;        // workgroups of the objective reduction
constexpr int kSelectCapDefault = 4096;
constexpr int kStageEvents = STRADS_N_STAGES + 1;

// Device-side scalars of one round, kept in one small block of the workspace.
struct RoundScalars {
    unsigned long long updates_total;   // sum of |B_1| over all rounds since create
    unsigned long long next_round;      // index t of the round this shard runs next (keys the random
                                        // stream); advanced on the device so that a recorded HIP graph
                                        // of rounds can be replayed without new kernel arguments
    uint32_t n_sel;        // keys strictly above the 22-bit boundary prefix
    uint32_t n_bnd;        // keys on the boundary prefix
    uint32_t bin0, rem1;   // first digit of the L'-th key, rank still to find below it
    uint32_t prefix22, rem2;
    int32_t n_kept;
    int32_t n_moved;
    int32_t near_rho_pairs;
    float max_abs_delta;
    uint32_t kkt_max_bits; // float bits of the running max violation (>= 0, so uint order = float order)
    uint32_t bad_input;    // set by the create-time check of a CSC design
    int32_t n_movers;      // dynamic dependencies: candidates whose update is not zero
    int32_t n_mkept;       // dynamic dependencies: movers that passed the filter
    uint32_t gram_next;    // 256-wide Gram tiles: next item of the kernel's queue (zero between rounds)
    uint32_t overflow;     // CSC designs: a product left the range of the fixed-point accumulators (sticky until
                           // the state is set again); the residual is then written as NaN
    uint32_t chunk_nz[STRADS_MAX_L_PRIME / 64];    // 256-wide Gram tiles: [c] != 0: a row of candidates 64c .. 64c+63
                           // has a conflict bit in mask word c + 2 or beyond (set by the mask kernel, cleared by the
                           // greedy walk; a mark too many costs time only)
};

// Decomposition of a candidate Gram into workgroup jobs (see gram.hip).  With dynamic
// dependencies it is chosen on the device from the number of movers.
struct GramShape {
    int32_t L, Lpad, T;                 // columns, padded to the tile, tiles per side
    int32_t split_off, split_diag;      // K-slices of an off-diagonal / a diagonal tile
    int32_t pad_;
    int64_t kchunk_off, kchunk_diag;    // rows per slice (multiples of kGramKT)
};

struct Workspace {
    // offsets in bytes from the workspace base.  beta, dbeta, r, objpart, objout are shared by all
    // scheduler shards; everything else exists once per shard, lane_stride bytes apart.
    size_t beta, dbeta, r;
    size_t w;               // float [Npad]: logistic loss, the weights eq. (2)'s dot products are taken with
    size_t jobtab;          // int32 [jobs]: static dependencies, dense/packed: job of each Gram workgroup
    size_t big_tables;      // dense fp32 designs: queue and per-tile slot ranges of the 256-wide Gram tiles
    size_t keys;            // uint32 [J]
    size_t hist;            // uint32 [2][kHistBins]
    size_t scalars;         // RoundScalars
    size_t sel;             // uint64 [2 * STRADS_MAX_L_PRIME]
    size_t bnd;             // uint64 [J]
    size_t cand;            // int32 [Lpad]
    size_t partial;         // float [split_max][Lpad][Lpad]   (dense Gram K-slices)
    size_t gram;            // float [Lpad][Lpad] (keep_gram only)
    size_t mask;            // uint64 [Lpad][Lpad/64]
    size_t kept_pos, kept;  // int32 [Lpad]
    size_t z, delta;        // float [Lpad]
    size_t mv_col;          // int32 [Lpad]
    size_t mv_delta;        // float [Lpad]
    size_t rpart;           // float [kMaxResidualGroups][Npad]
    size_t objpart;         // double [kObjBlocks]
    size_t objout;          // double [1]
    // dynamic dependencies (per candidate position, then per mover)
    size_t zc, dc, nbc;     // float [Lpad]: x_j^T r, tentative change, tentative new beta
    size_t mpos, mcand;     // int32 [Lpad]: candidate position / column id of each mover, draw order
    size_t mkept_pos;       // int32 [Lpad]: positions into the mover list that passed the filter
    size_t dshape;          // GramShape of the current round's movers
    size_t dtable;          // GramShape [STRADS_MAX_L_PRIME / kGramTile + 1], by number of tiles per side
    size_t csc_scratch;     // CSC only: see csc.hip
    size_t csc_scratch_bytes;
    size_t lane_begin, lane_stride;   // the per-shard block of shard s starts at lane_begin + s * lane_stride
    size_t total;
};

} // namespace strads

struct strads_lasso {
    strads_lasso_config_t cfg;
    strads::Workspace ws;
    char *base;
    hipStream_t stream;
    int32_t L;          // min(l_prime, J)
    int32_t Lpad;       // L rounded up to the Gram tile
    int64_t Npad;       // N rounded up to 64; r[N .. Npad) is kept at zero
    float step_scale;   // 1 / curvature of the coordinate step: 1 (squared loss), 4 (logistic loss)
    int32_t split_max;  // K-slices the workspace was sized for
    int32_t split_user; // tuning override (0 = automatic)
    size_t partial_floats;   // floats of ws.partial
    int32_t dots_with_gram;  // short lists: every candidate's x_j^T r rides along with the Gram launch and the filter's
                             // workgroup commits B_1 (tuning "dots_with_gram", default 1; see dots_ride_with_gram)
    int32_t early_keys;      // rounds enqueued back to back: the next round's key pass rides with the last kernel of the
                             // residual update (tuning "early_keys", default 1; one scheduler)
    int32_t next_keys_done;  // the round about to be enqueued already has its keys and first histogram
    int32_t residual_fused;  // lists of at most 1024 candidates update the residual in one kernel (tuning "residual_fused", default 1)
    int32_t jobtab_on;  // the Gram workgroups take their jobs from ws.jobtab (tuning "gram_xcd_map", default 1)
    int32_t *jobtab_host;   // shard 0 only: host staging copy of the table
    int32_t tile256;    // Gram of long lists in 256 x 256 tiles: 0 never, 1 where it is the default, 2 wherever the
                        // workspace has the partial planes for it (tuning "gram_tile256", default 1)
    int32_t big_items;  // items in that route's queue; 0: the 128 x 128 kernel is used
    int32_t direct;     // Gram of a long list over short columns in 64 x 64 tiles that write the conflict bits themselves:
                        // 0 never, 1 where it is the default, 2 wherever it applies (tuning "gram_direct", default 1)
    int32_t select_cap;
    int64_t round;
    bool vec4;          // dense columns are 16-byte aligned (N % 4 == 0 and x aligned)
    // optional stage timing with HIP events on the caller's stream
    int32_t profile_level;   // 0 off, 1 Gram tile kernel only, 2 every stage boundary
    int32_t profile_rounds;  // rounds the event pool can hold
    int32_t profiled;        // rounds recorded so far
    hipEvent_t *events;      // [profile_rounds][kStageEvents]
    // scheduler shards (Section 3).  The handle the caller holds is shard 0 and owns the others.
    int32_t n_lanes;         // S
    int32_t lane_id;         // this handle's shard
    int64_t Js;              // coordinates of this shard: #{j < J : j mod S == lane_id}
    strads_lasso *lanes[STRADS_MAX_SHARDS];   // shard 0 only: [0] is the handle itself
    hipEvent_t ev_resid;     // recorded after this shard's residual update
    hipEvent_t ev_fork;      // shard 0 only: the caller's stream at the start of an enqueueing call
    hipEvent_t ev_kkt[2];    // shard 0 only: around the kernels of the pass over all columns (profiling)
    float last_kkt_ms;
    hipEvent_t ev_join;      // this shard's stream at the end of an enqueueing call
    int64_t rounds_since_fork;   // shard 0 only: rounds enqueued since the shards' streams were last forked
    // HIP graph of graph_rounds consecutive rounds, recorded once per starting shard and replayed by
    // strads_lasso_run (shard 0 only)
    int32_t graph_rounds;                       // 0: never use graphs
    hipGraph_t graph[STRADS_MAX_SHARDS];
    hipGraphExec_t graph_exec[STRADS_MAX_SHARDS];
    strads::GramShape shape_table[STRADS_MAX_L_PRIME / strads::kGramTile + 1];   // host copy of ws.dtable

    template <class T> T *at(size_t off) const { return reinterpret_cast<T *>(base + off); }
};

namespace strads {

// Status of the launches a launcher has just made.  A debug build (-DSTRADS_DEBUG_SYNC) also waits for
// them and reports what the kernels themselves ran into, so that a failure is pinned to the launcher that
// caused it instead of surfacing at some later call.  (Not while the stream is being captured into a
// graph: nothing runs then.)
inline hipError_t launch_status(hipStream_t stream)
{
    hipError_t e = hipGetLastError();
#ifdef STRADS_DEBUG_SYNC
    if (e == hipSuccess) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &cs) != hipSuccess) { (void)hipGetLastError(); cs = hipStreamCaptureStatusNone; }
        if (cs == hipStreamCaptureStatusNone) {
            e = hipStreamSynchronize(stream);
            if (e == hipSuccess) e = hipGetLastError();
        }
    }
#else
    (void)stream;
#endif
    return e;
}

int gram_split_auto(int64_t n, int32_t lpad);
size_t gram_partial_floats(int64_t n, int32_t lpad, bool dynamic);   // floats of K-slice partial tiles to reserve
void gram_shape_table(int64_t n, int32_t lpad, GramShape *out);      // out[t], t = 0 .. lpad/kGramTile
bool gram256_default(int64_t n, int32_t lpad, int32_t layout, int32_t deps);
int32_t gram256_items(int64_t n, int32_t lpad);                      // items (= tile slots) of the 256-wide route's queue
bool gram_direct_default(int64_t n, int32_t lpad);                   // see k_gram_direct
size_t gram256_table_bytes(int64_t n, int32_t lpad);
int32_t gram256_tables(int64_t n, int32_t lpad, void *out);          // host image of ws.big_tables
int32_t gram256_plan_host(int64_t n, int32_t lpad, int32_t cap, int32_t *items5, int32_t *first, int32_t *count);
size_t gram_job_table_entries(int64_t n, int32_t lpad);              // capacity needed for gram_job_table
int32_t gram_job_table(const strads_lasso *h, int32_t *out);         // out[blockIdx.x] = job; returns the job count
Workspace carve(int64_t n, int64_t j, int32_t layout, int32_t l, int32_t keep_gram, int32_t max_col_nnz, int32_t deps,
                int32_t n_shards);
Workspace workspace_of_lane(const Workspace &w0, int32_t lane);

// Each launcher enqueues on h->stream and returns the hipError_t of the launch.
hipError_t launch_sampler(strads_lasso *h, bool keys_done);                             // Step 1 -> cand[L]; round index from the device
hipError_t launch_set_next_round(strads_lasso *h, hipStream_t stream, int64_t next_round);
hipError_t launch_keys_only(strads_lasso *h, int64_t round, float *keys);  // stage entry
hipError_t launch_gram_dense(strads_lasso *h, int part);  // Step 2a; part 0: K-slice tiles, part 1: sum + conflict mask
hipError_t launch_mask_from_gram(strads_lasso *h, const float *gram, int32_t l);
// the same two steps on buffers named one by one (no handle): conflict bits of an l x l Gram into lpad rows of
// lpad / 64 words, then the greedy walk over them
hipError_t launch_mask_from_gram_plain(hipStream_t stream, const float *gram, int32_t l, int32_t lpad, float rho,
                                       uint64_t *mask);
hipError_t launch_filter_plain(hipStream_t stream, const uint64_t *mask, int32_t l, int32_t lpad, int32_t p_max,
                               const int32_t *cand, int32_t *kept_pos, int32_t *kept, RoundScalars *sc, int32_t *n_out);
hipError_t launch_filter(strads_lasso *h, int32_t l, bool count_updates, bool commit, bool marked);       // Step 2b -> kept_pos, kept, n_kept;
                                                          // commit: and eq. (2) for B_1 from the candidates' tentative updates
hipError_t launch_keep_all(strads_lasso *h);              // no dependency check: B_1 = first p_max candidates
// dynamic dependencies
hipError_t launch_dots_cand(strads_lasso *h);             // x_j^T r and tentative change of every candidate
hipError_t launch_movers(strads_lasso *h);                // mover list + Gram decomposition for it
hipError_t launch_filter_movers(strads_lasso *h);         // greedy walk over the movers -> mkept_pos, n_mkept; then
                                                          // B_1 = non-movers + kept movers; beta, delta beta
hipError_t launch_scatter_mover_gram(strads_lasso *h, float *out);   // L x L image of the mover Gram
hipError_t launch_dots_dense(strads_lasso *h);                             // x_j^T r for the kept set + eq. (2) update
struct KeysArgs;
KeysArgs keys_args(strads_lasso *h);                      // arguments of pass 1 of the selection
// want_next_keys: another round follows at once; *next_keys_done: its key pass rode along (one scheduler, short lists)
hipError_t launch_residual_dense(strads_lasso *h, bool want_next_keys, bool *next_keys_done);                         // r -= X_B delta_B
hipError_t launch_residual_apply(strads_lasso *h, int groups, bool want_next_keys, bool *next_keys_done);   // r -= sum of the groups' partial sums
int residual_groups(int64_t n, int32_t l);
hipError_t launch_objective(strads_lasso *h);                              // -> objout
hipError_t launch_logistic_weights(strads_lasso *h);                       // r (= -X beta) -> w
// the vector eq. (2) and the optimality test take dot products with
inline const float *dots_vector(const strads_lasso *h)
{
    return reinterpret_cast<const float *>(h->base + (h->cfg.loss == STRADS_LOSS_LOGISTIC ? h->ws.w : h->ws.r));
}
// Short candidate lists of an fp32 design under Algorithm 1's dependency rule, one scheduler: a round
// is a chain of short kernels and what it costs is their number.  Then the pass that takes x_j^T r is
// made for all candidates by extra workgroups of the Gram launch (CandDots), and the filter's
// workgroup applies eq. (2) to the ones it kept.  (With several schedulers the Gram of a round is
// formed before the previous round's residual exists, so its products cannot be taken there.)
constexpr int kShortList = 4096;
inline bool dots_ride_with_gram(const strads_lasso *h)
{
    return h->dots_with_gram && h->cfg.deps == STRADS_DEPS_STATIC && h->cfg.layout == STRADS_LAYOUT_DENSE_COLMAJOR &&
           h->n_lanes == 1 && h->L <= kShortList && h->big_items == 0;
}
// Whether Step 2's Gram goes straight to conflict bits in 64 x 64 tiles (k_gram_direct): Algorithm 1's rule, a dense
// or packed design, the automatic K decomposition, and the 256-wide tiles not in use.
inline bool gram_direct_on(const strads_lasso *h)
{
    if (h->cfg.deps != STRADS_DEPS_STATIC || h->cfg.layout == STRADS_LAYOUT_CSC || h->big_items > 0 || h->split_user > 0)
        return false;
    return h->direct == 2 || (h->direct == 1 && gram_direct_default(h->cfg.n, h->Lpad));
}
struct CandDots;
CandDots cand_dots_args(strads_lasso *h);                 // arguments of the candidates' tentative updates
hipError_t launch_kkt_dense(strads_lasso *h, float *g_or_null);            // -> scalars.kkt_max_bits
hipError_t launch_init_state(strads_lasso *h);
hipError_t launch_check_unit_norm(strads_lasso *h);       // sets bit 1 of scalars.bad_input if a column's l2 norm is not 1
hipError_t launch_init_lane(strads_lasso *h);             // zero a shard's histograms and round scalars
hipError_t launch_clear_kkt(strads_lasso *h);
hipError_t sampler_prepare();
hipError_t gram_prepare();
hipError_t filter_prepare();
hipError_t update_prepare();
// packed genotype design (STRADS_LAYOUT_GENO2); the Gram uses launch_gram_dense with a decoding loader
inline int64_t geno_words(int64_t n) { return (n + 63) / 64 * 4; }   // 32-bit words per column
hipError_t launch_dots_geno(strads_lasso *h);
hipError_t launch_dots_cand_geno(strads_lasso *h);
hipError_t launch_residual_geno(strads_lasso *h, bool want_next_keys, bool *next_keys_done);
hipError_t launch_kkt_geno(strads_lasso *h, float *g_or_null);
// CSC design
hipError_t launch_gram_csc(strads_lasso *h);
hipError_t launch_dots_csc(strads_lasso *h);
hipError_t launch_dots_cand_csc(strads_lasso *h);         // dynamic dependencies: all candidates, nothing committed
hipError_t launch_residual_csc(strads_lasso *h, bool want_next_keys, bool *next_keys_done);
hipError_t launch_kkt_csc(strads_lasso *h, float *g_or_null);
size_t csc_scratch_bytes(int64_t n, int32_t l, int32_t max_col_nnz);
hipError_t csc_prepare();
hipError_t launch_csc_init(strads_lasso *h, uint32_t *bad_dev);

} // namespace strads
