// C ABI of libstrads_lasso: argument checking, workspace carving and the order in which the
// kernels of one round (Algorithm 1's loop body) are enqueued on the caller's stream.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "strads_internal.h"

namespace strads {

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

Workspace carve(int64_t n, int64_t j, int32_t layout, int32_t l, int32_t keep_gram, int32_t max_col_nnz, int32_t deps,
                int32_t n_shards)
{
    Workspace w;
    memset(&w, 0, sizeof(w));
    const int64_t S = n_shards > 1 ? n_shards : 1;
    const int64_t js = (j + S - 1) / S;                  // coordinates of the largest shard
    const int64_t lpad = (l + kGramTile - 1) / kGramTile * kGramTile;
    const int64_t npad = (n + 63) / 64 * 64;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    // shared by all shards: the solver state and the objective scratch
    w.beta = take((size_t)j * 4);
    w.dbeta = take((size_t)j * 4);
    w.r = take((size_t)npad * 4);
    w.w = take((size_t)npad * 4);
    w.jobtab = take(layout != STRADS_LAYOUT_CSC && deps != STRADS_DEPS_DYNAMIC
                        ? gram_job_table_entries(n, (int32_t)lpad) * 4 : 256);
    w.big_tables = take(layout == STRADS_LAYOUT_DENSE_COLMAJOR ? gram256_table_bytes(n, (int32_t)lpad) : 256);
    w.objpart = take((size_t)kObjBlocks * 8);
    w.objout = take(8);
    // once per shard
    w.lane_begin = off;
    w.keys = take((size_t)js * 4);
    w.hist = take((size_t)2 * kHistBins * 4);
    w.scalars = take(sizeof(RoundScalars));
    w.sel = take((size_t)2 * STRADS_MAX_L_PRIME * 8);
    w.bnd = take((size_t)js * 8);
    w.cand = take((size_t)lpad * 4);
    if (layout != STRADS_LAYOUT_CSC)
        w.partial = take(gram_partial_floats(n, (int32_t)lpad, deps == STRADS_DEPS_DYNAMIC) * 4);
    else
        w.partial = take(256);
    w.gram = take(keep_gram ? (size_t)lpad * lpad * 4 : 256);
    w.mask = take((size_t)lpad * (lpad / 64) * 8);
    w.kept_pos = take((size_t)lpad * 4);
    w.kept = take((size_t)lpad * 4);
    w.z = take((size_t)lpad * 4);
    w.delta = take((size_t)lpad * 4);
    w.mv_col = take((size_t)lpad * 4);
    w.mv_delta = take((size_t)lpad * 4);
    w.rpart = take((size_t)kMaxResidualGroups * npad * 4);
    const size_t dyn = deps == STRADS_DEPS_DYNAMIC ? (size_t)lpad * 4 : 256;
    w.zc = take((size_t)lpad * 4);            // every candidate's tentative update
    w.dc = take((size_t)lpad * 4);
    w.nbc = take((size_t)lpad * 4);
    w.mpos = take(dyn);
    w.mcand = take(dyn);
    w.mkept_pos = take(dyn);
    w.dshape = take(sizeof(GramShape));
    w.dtable = take(sizeof(GramShape) * (STRADS_MAX_L_PRIME / kGramTile + 1));
    w.csc_scratch_bytes = layout == STRADS_LAYOUT_CSC ? csc_scratch_bytes(n, l, max_col_nnz) : 0;
    w.csc_scratch = take(w.csc_scratch_bytes ? w.csc_scratch_bytes : 256);
    w.lane_stride = off - w.lane_begin;
    w.total = w.lane_begin + (size_t)S * w.lane_stride;
    return w;
}

Workspace workspace_of_lane(const Workspace &w0, int32_t lane)
{
    Workspace w = w0;
    const size_t d = (size_t)lane * w0.lane_stride;
    size_t *per_lane[] = {&w.keys, &w.hist, &w.scalars, &w.sel, &w.bnd, &w.cand, &w.partial, &w.gram, &w.mask,
                          &w.kept_pos, &w.kept, &w.z, &w.delta, &w.mv_col, &w.mv_delta, &w.rpart, &w.zc, &w.dc,
                          &w.nbc, &w.mpos, &w.mcand, &w.mkept_pos, &w.dshape, &w.dtable, &w.csc_scratch};
    for (size_t *f : per_lane) *f += d;
    return w;
}

static bool sizes_ok(const strads_lasso_config_t *c)
{
    if (!c) return false;
    if (c->n <= 0 || c->j <= 0 || c->j >= (int64_t)1 << 31) return false;
    if (c->layout != STRADS_LAYOUT_DENSE_COLMAJOR && c->layout != STRADS_LAYOUT_CSC &&
        c->layout != STRADS_LAYOUT_GENO2) return false;
    if (c->l_prime < 1 || c->l_prime > STRADS_MAX_L_PRIME) return false;
    if (c->layout == STRADS_LAYOUT_CSC && (c->n >= (int64_t)1 << 31 || c->max_col_nnz < 1)) return false;
    if (c->deps != STRADS_DEPS_STATIC && c->deps != STRADS_DEPS_DYNAMIC && c->deps != STRADS_DEPS_NONE) return false;
    if (c->priority != STRADS_PRIORITY_SQUARED && c->priority != STRADS_PRIORITY_LINEAR &&
        c->priority != STRADS_PRIORITY_UNIFORM) return false;
    if (c->n_shards < 0 || c->n_shards > STRADS_MAX_SHARDS || (int64_t)c->n_shards > c->j) return false;
    if (c->loss != STRADS_LOSS_SQUARED && c->loss != STRADS_LOSS_LOGISTIC) return false;
    return true;
}

static int32_t shard_count(const strads_lasso_config_t *c) { return c->n_shards > 1 ? c->n_shards : 1; }

// candidates per round: P' clamped to the size of the smallest shard
static int32_t clamp_l(const strads_lasso_config_t *c)
{
    const int64_t smallest = c->j / shard_count(c);
    return (int64_t)c->l_prime < smallest ? c->l_prime : (int32_t)smallest;
}

} // namespace strads

using namespace strads;

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) return STRADS_E_HIP; } while (0)

// (Re)build the Gram job table of the current decomposition on the host and copy it to the workspace
// (shared by all shards: they have the same candidate count).  The staging buffer belongs to the handle,
// so the copy may still be in flight when this returns; callers synchronise before it is rebuilt.
static int upload_job_table(strads_lasso *h)
{
    const size_t cap = gram_job_table_entries(h->cfg.n, h->Lpad);
    if (!h->jobtab_host) h->jobtab_host = (int32_t *)malloc(cap * sizeof(int32_t));
    if (!h->jobtab_host) return STRADS_E_INVALID_ARG;
    const int32_t total = gram_job_table(h, h->jobtab_host);
    if ((size_t)total > cap) return STRADS_E_INVALID_ARG;
    HIP_TRY(hipMemcpyAsync(h->base + h->ws.jobtab, h->jobtab_host, (size_t)total * sizeof(int32_t),
                           hipMemcpyHostToDevice, h->stream));
    return STRADS_OK;
}

// Choose between the two Gram tile kernels (h->tile256, the shape, the partial storage the workspace holds)
// and, for the 256-wide one, build its tables and copy them to the workspace.  Waits for the copy.
static int choose_gram_route(strads_lasso *h)
{
    int32_t items = 0;
    const bool can = h->vec4 && h->cfg.deps == STRADS_DEPS_STATIC && h->cfg.layout == STRADS_LAYOUT_DENSE_COLMAJOR;
    if (can && (h->tile256 == 2 ||
                (h->tile256 == 1 && gram256_default(h->cfg.n, h->Lpad, h->cfg.layout, h->cfg.deps)))) {
        items = gram256_items(h->cfg.n, h->Lpad);
        // one 256 x 256 slot per item must fit the partial storage
        if ((size_t)items * 256 * 256 > h->partial_floats) items = 0;
    }
    if (items > 0) {
        void *img = malloc(gram256_table_bytes(h->cfg.n, h->Lpad));
        if (!img) return STRADS_E_INVALID_ARG;
        gram256_tables(h->cfg.n, h->Lpad, img);
        const hipError_t e1 = hipMemcpyAsync(h->base + h->ws.big_tables, img, gram256_table_bytes(h->cfg.n, h->Lpad),
                                             hipMemcpyHostToDevice, h->stream);
        const hipError_t e2 = hipStreamSynchronize(h->stream);
        free(img);
        if (e1 != hipSuccess || e2 != hipSuccess) return STRADS_E_HIP;
    }
    for (int32_t s = 0; s < h->n_lanes; ++s) h->lanes[s]->big_items = items;
    return STRADS_OK;
}

extern "C" {

size_t strads_lasso_workspace_bytes(const strads_lasso_config_t *cfg)
{
    if (!sizes_ok(cfg)) return 0;
    return carve(cfg->n, cfg->j, cfg->layout, clamp_l(cfg), cfg->keep_gram, cfg->max_col_nnz, cfg->deps,
                 shard_count(cfg)).total;
}

int strads_lasso_create(const strads_lasso_config_t *cfg, strads_lasso_t **out)
{
    if (!out || !sizes_ok(cfg)) return STRADS_E_INVALID_ARG;
    if (!cfg->x || !cfg->y || !cfg->workspace) return STRADS_E_INVALID_ARG;
    if (cfg->layout == STRADS_LAYOUT_CSC && (!cfg->row_idx || !cfg->col_ptr)) return STRADS_E_INVALID_ARG;
    if (cfg->layout == STRADS_LAYOUT_GENO2 && (!cfg->col_mean || !cfg->col_scale || ((uintptr_t)cfg->x & 15u) != 0))
        return STRADS_E_INVALID_ARG;
    if (!(cfg->lambda >= 0.f) || !isfinite(cfg->lambda)) return STRADS_E_INVALID_ARG;
    if (!(cfg->rho > 0.f) || isnan(cfg->rho)) return STRADS_E_INVALID_ARG;
    if (!(cfg->eta >= 1e-30f) || !isfinite(cfg->eta)) return STRADS_E_INVALID_ARG;
    if (!(cfg->c_init > 0.f) || !(cfg->c_init <= 1e18f)) return STRADS_E_INVALID_ARG;
    if (cfg->p_max < 0) return STRADS_E_INVALID_ARG;
    if (((uintptr_t)cfg->workspace & 255u) != 0) return STRADS_E_INVALID_ARG;
    if (((uintptr_t)cfg->x & 3u) != 0 || ((uintptr_t)cfg->y & 3u) != 0) return STRADS_E_INVALID_ARG;

    const int32_t L = clamp_l(cfg);
    const int32_t S = shard_count(cfg);
    const Workspace ws = carve(cfg->n, cfg->j, cfg->layout, L, cfg->keep_gram, cfg->max_col_nnz, cfg->deps, S);
    if (cfg->workspace_bytes < ws.total) return STRADS_E_WORKSPACE_TOO_SMALL;

    strads_lasso *h = (strads_lasso *)calloc(1, sizeof(strads_lasso));
    if (!h) return STRADS_E_INVALID_ARG;
    h->cfg = *cfg;
    h->ws = ws;
    h->base = (char *)cfg->workspace;
    h->stream = (hipStream_t)cfg->stream;
    h->L = L;
    h->Lpad = (L + kGramTile - 1) / kGramTile * kGramTile;
    h->Npad = (cfg->n + 63) / 64 * 64;
    h->split_max = cfg->layout != STRADS_LAYOUT_CSC ? gram_split_auto(cfg->n, h->Lpad) : 1;
    h->partial_floats = cfg->layout != STRADS_LAYOUT_CSC
                            ? gram_partial_floats(cfg->n, h->Lpad, cfg->deps == STRADS_DEPS_DYNAMIC) : 0;
    h->split_user = 0;
    h->step_scale = cfg->loss == STRADS_LOSS_LOGISTIC ? 4.f : 1.f;
    h->dots_with_gram = 1;
    h->early_keys = 1;
    h->next_keys_done = 0;
    h->residual_fused = 1;
    h->jobtab_on = cfg->layout != STRADS_LAYOUT_CSC && cfg->deps != STRADS_DEPS_DYNAMIC ? 1 : 0;
    h->tile256 = 1;
    h->big_items = 0;
    h->direct = 1;
    h->select_cap = kSelectCapDefault;
    h->round = 0;
    h->profile_level = 0;
    h->profile_rounds = 256;
    h->profiled = 0;
    h->events = nullptr;
    h->vec4 = cfg->layout == STRADS_LAYOUT_DENSE_COLMAJOR && (cfg->n % 4 == 0) && (((uintptr_t)cfg->x & 15u) == 0);

    h->n_lanes = S;
    h->graph_rounds = 0;                        // off unless asked for (set_tuning "graph_rounds")
    h->lane_id = 0;
    h->lanes[0] = h;
    int rc = STRADS_OK;
    if (sampler_prepare() != hipSuccess || gram_prepare() != hipSuccess || filter_prepare() != hipSuccess ||
        update_prepare() != hipSuccess ||
        (cfg->layout == STRADS_LAYOUT_CSC && csc_prepare() != hipSuccess))
        rc = STRADS_E_HIP;
    // the other scheduler shards: same problem, own per-shard block of the workspace, own stream
    for (int32_t s = 1; s < S && rc == STRADS_OK; ++s) {
        strads_lasso *ln = (strads_lasso *)malloc(sizeof(strads_lasso));
        if (!ln) { rc = STRADS_E_INVALID_ARG; break; }
        *ln = *h;
        ln->ws = workspace_of_lane(ws, s);
        ln->lane_id = s;
        ln->stream = nullptr;
        ln->ev_resid = ln->ev_join = ln->ev_fork = nullptr;
        ln->ev_kkt[0] = ln->ev_kkt[1] = nullptr;
        ln->last_kkt_ms = 0.f;
        h->lanes[s] = ln;
        if (hipStreamCreateWithFlags(&ln->stream, hipStreamNonBlocking) != hipSuccess) rc = STRADS_E_HIP;
    }
    for (int32_t s = 0; s < S && rc == STRADS_OK; ++s) {
        strads_lasso *ln = h->lanes[s];
        ln->Js = (cfg->j - s + S - 1) / S;
        if (S > 1 && (hipEventCreateWithFlags(&ln->ev_resid, hipEventDisableTiming) != hipSuccess ||
                      hipEventCreateWithFlags(&ln->ev_join, hipEventDisableTiming) != hipSuccess))
            rc = STRADS_E_HIP;
    }
    if (rc == STRADS_OK && S > 1 && hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming) != hipSuccess)
        rc = STRADS_E_HIP;

    // everything below is enqueued on the caller's stream and waited for before create returns
    if (rc == STRADS_OK && launch_init_state(h) != hipSuccess) rc = STRADS_E_HIP;
    if (rc == STRADS_OK && h->jobtab_on) rc = upload_job_table(h);
    if (rc == STRADS_OK) rc = choose_gram_route(h);
    for (int32_t s = 0; s < S && rc == STRADS_OK; ++s) {
        strads_lasso *ln = h->lanes[s];
        if (s > 0 && (hipMemsetAsync(h->base + ln->ws.hist, 0, (size_t)2 * kHistBins * 4, h->stream) != hipSuccess ||
                      hipMemsetAsync(h->base + ln->ws.scalars, 0, sizeof(RoundScalars), h->stream) != hipSuccess))
            rc = STRADS_E_HIP;
        if (rc == STRADS_OK && launch_set_next_round(ln, h->stream, s) != hipSuccess) rc = STRADS_E_HIP;
        if (rc == STRADS_OK && cfg->deps == STRADS_DEPS_DYNAMIC) {
            // Gram decomposition per mover-tile count, looked up by the mover kernel every round
            gram_shape_table(cfg->n, h->Lpad, h->shape_table);
            if (hipMemcpyAsync(h->base + ln->ws.dtable, h->shape_table,
                               sizeof(GramShape) * (size_t)(h->Lpad / kGramTile + 1), hipMemcpyHostToDevice,
                               h->stream) != hipSuccess)
                rc = STRADS_E_HIP;
        }
        if (rc == STRADS_OK && cfg->layout == STRADS_LAYOUT_CSC) {
            // the sparse kernels size their buckets from max_col_nnz: col_ptr is checked against it
            // (bad_input of shard 0 is read back below); every shard's counters start at zero
            strads_lasso tmp = *ln;
            tmp.stream = h->stream;
            if (launch_csc_init(&tmp, &h->at<RoundScalars>(ln->ws.scalars)->bad_input) != hipSuccess) rc = STRADS_E_HIP;
        }
    }
#ifdef STRADS_DEBUG_SYNC
    // debug build: the unit-norm precondition of eq. (2)'s update is checked, one pass over the design
    if (rc == STRADS_OK && launch_check_unit_norm(h) != hipSuccess) rc = STRADS_E_HIP;
#endif
    if (rc == STRADS_OK) {
        RoundScalars sc;
        if (hipMemcpyAsync(&sc, h->base + ws.scalars, sizeof(sc), hipMemcpyDeviceToHost, h->stream) != hipSuccess ||
            hipStreamSynchronize(h->stream) != hipSuccess)
            rc = STRADS_E_HIP;
        else if (sc.bad_input != 0)
            rc = STRADS_E_INVALID_ARG;
    }
    if (rc != STRADS_OK) {
        strads_lasso_destroy(h);
        return rc;
    }
    *out = h;
    return STRADS_OK;
}

static void drop_events(strads_lasso *h);
static void drop_graphs(strads_lasso *h);

void strads_lasso_destroy(strads_lasso_t *h)
{
    if (!h) return;
    drop_events(h);
    drop_graphs(h);
    for (int32_t s = 0; s < h->n_lanes; ++s) {
        strads_lasso *ln = h->lanes[s];
        if (!ln) continue;
        if (s > 0 && ln->stream) { (void)hipStreamSynchronize(ln->stream); (void)hipStreamDestroy(ln->stream); }
        if (ln->ev_resid) (void)hipEventDestroy(ln->ev_resid);
        if (ln->ev_join) (void)hipEventDestroy(ln->ev_join);
        if (s > 0) free(ln);
    }
    if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
    if (h->jobtab_host) (void)hipStreamSynchronize(h->stream);    // its copy to the workspace may be in flight
    free(h->jobtab_host);
    for (int i = 0; i < 2; ++i) if (h->ev_kkt[i]) (void)hipEventDestroy(h->ev_kkt[i]);
    free(h);
}

// Stage boundaries of a round, in stream order: boundary b precedes stage b (STRADS_STAGE_*)
// and boundary STRADS_N_STAGES closes the round.
static inline int mark(strads_lasso *h, int boundary)
{
    if (h->profile_level == 0 || h->profiled >= h->profile_rounds) return STRADS_OK;
    if (h->profile_level == 1 && boundary != STRADS_STAGE_GRAM_TILES && boundary != STRADS_STAGE_GRAM_TILES + 1)
        return STRADS_OK;
    HIP_TRY(hipEventRecord(h->events[(size_t)h->profiled * kStageEvents + boundary], h->stream));
    return STRADS_OK;
}

// Enqueue round h->round.  With S scheduler shards it is shard (round mod S)'s turn: its draw, Gram
// and greedy walk go to its own stream and depend on nothing another shard does, so they overlap
// with the other shards' work; whatever reads or writes the residual waits for the previous
// round's residual update, so the updates are applied in round order (Section 3: the schedulers
// prepare concurrently and take turns to dispatch).
static int enqueue_round(strads_lasso *top, bool more_follows)
{
    const int32_t S = top->n_lanes;
    strads_lasso *h = top->lanes[top->round % S];
    strads_lasso *prev = top->lanes[(top->round + S - 1) % S];
    const bool csc = h->cfg.layout == STRADS_LAYOUT_CSC, geno = h->cfg.layout == STRADS_LAYOUT_GENO2;
    const bool dynamic = h->cfg.deps == STRADS_DEPS_DYNAMIC;
    const bool unchecked = h->cfg.deps == STRADS_DEPS_NONE;
#define MARK(b) do { const int rc_ = mark(top, (b)); if (rc_ != STRADS_OK) return rc_; } while (0)
    // (the first round after a fork needs no event: the fork itself orders it after everything before)
#define AFTER_PREVIOUS_ROUND() do { if (S > 1 && top->rounds_since_fork > 0) HIP_TRY(hipStreamWaitEvent(h->stream, prev->ev_resid, 0)); } while (0)
    MARK(STRADS_STAGE_SAMPLER);
    HIP_TRY(launch_sampler(h, top->next_keys_done != 0));   // the round index is the shard's device-side counter
    top->next_keys_done = 0;
    MARK(STRADS_STAGE_CAND_DOTS);
    if (dynamic) {
        // every candidate's update from the current residual; the movers; how to tile their Gram
        AFTER_PREVIOUS_ROUND();
        if (h->cfg.loss == STRADS_LOSS_LOGISTIC) HIP_TRY(launch_logistic_weights(h));
        if (csc) HIP_TRY(launch_dots_cand_csc(h));
        else if (geno) HIP_TRY(launch_dots_cand_geno(h));
        else HIP_TRY(launch_dots_cand(h));
        HIP_TRY(launch_movers(h));
    }
    const bool ride = dots_ride_with_gram(h);   // the candidates' x_j^T r is taken by the Gram launch
    MARK(STRADS_STAGE_GRAM_TILES);
    if (ride && h->cfg.loss == STRADS_LOSS_LOGISTIC) HIP_TRY(launch_logistic_weights(h));
    if (!unchecked) { if (csc) HIP_TRY(launch_gram_csc(h)); else HIP_TRY(launch_gram_dense(h, 0)); }
    MARK(STRADS_STAGE_GRAM_MASK);
    if (!unchecked && !csc) HIP_TRY(launch_gram_dense(h, 1));
    MARK(STRADS_STAGE_FILTER);
    if (unchecked) HIP_TRY(launch_keep_all(h));
    else if (dynamic) HIP_TRY(launch_filter_movers(h));
    else HIP_TRY(launch_filter(h, h->L, true, ride, !csc && h->big_items > 0));   // (the 256-wide tiles' mask kernel marks chunks)
    MARK(STRADS_STAGE_UPDATE);
    if (!dynamic) AFTER_PREVIOUS_ROUND();
    if (!dynamic && !ride && h->cfg.loss == STRADS_LOSS_LOGISTIC) HIP_TRY(launch_logistic_weights(h));
    if (dynamic || ride) { /* B_1 was committed by the filter's workgroup */ }
    else if (csc) HIP_TRY(launch_dots_csc(h));
    else if (geno) HIP_TRY(launch_dots_geno(h));
    else HIP_TRY(launch_dots_dense(h));
    MARK(STRADS_STAGE_RESIDUAL);
    {
        // the round that follows at once gets its key pass from extra workgroups of this round's last kernel
        bool done = false;
        const bool want = more_follows && top->early_keys != 0;
        if (csc) HIP_TRY(launch_residual_csc(h, want, &done));
        else if (geno) HIP_TRY(launch_residual_geno(h, want, &done));
        else HIP_TRY(launch_residual_dense(h, want, &done));
        top->next_keys_done = done ? 1 : 0;
    }
    MARK(STRADS_N_STAGES);
    if (S > 1) HIP_TRY(hipEventRecord(h->ev_resid, h->stream));
#undef MARK
#undef AFTER_PREVIOUS_ROUND
    if (top->profile_level != 0 && top->profiled < top->profile_rounds) top->profiled += 1;
    top->round += 1;
    top->rounds_since_fork += 1;
    return STRADS_OK;
}

// The shards' streams start after everything already on the caller's stream ...
static int fork_lanes(strads_lasso *h)
{
    h->rounds_since_fork = 0;
    if (h->n_lanes == 1) return STRADS_OK;
    HIP_TRY(hipEventRecord(h->ev_fork, h->stream));
    for (int32_t s = 1; s < h->n_lanes; ++s) HIP_TRY(hipStreamWaitEvent(h->lanes[s]->stream, h->ev_fork, 0));
    return STRADS_OK;
}

// ... and the caller's stream continues after everything the shards were given.
static int join_lanes(strads_lasso *h)
{
    for (int32_t s = 1; s < h->n_lanes; ++s) {
        HIP_TRY(hipEventRecord(h->lanes[s]->ev_join, h->lanes[s]->stream));
        HIP_TRY(hipStreamWaitEvent(h->stream, h->lanes[s]->ev_join, 0));
    }
    return STRADS_OK;
}

static void drop_events(strads_lasso *h)
{
    if (h->events) {
        for (size_t i = 0; i < (size_t)h->profile_rounds * kStageEvents; ++i)
            if (h->events[i]) (void)hipEventDestroy(h->events[i]);
        free(h->events);
        h->events = nullptr;
    }
    h->profile_level = 0;
    h->profiled = 0;
}

// Round scalars of shard `lane`, read on the caller's stream (which every enqueueing call leaves
// ordered after the shards' streams).
static int read_lane_scalars(strads_lasso *h, int32_t lane, RoundScalars *host)
{
    HIP_TRY(hipMemcpyAsync(host, h->base + h->lanes[lane]->ws.scalars, sizeof(RoundScalars), hipMemcpyDeviceToHost,
                           h->stream));
    HIP_TRY(hipStreamSynchronize(h->stream));
    return STRADS_OK;
}

static int read_scalars(strads_lasso *h, RoundScalars *host) { return read_lane_scalars(h, 0, host); }

// the shard that ran the most recent round
static int32_t last_lane(const strads_lasso *h) { return h->round > 0 ? (int32_t)((h->round - 1) % h->n_lanes) : 0; }

static int total_updates(strads_lasso *h, unsigned long long *out)
{
    unsigned long long sum = 0;
    for (int32_t s = 0; s < h->n_lanes; ++s) {
        RoundScalars sc;
        const int rs = read_lane_scalars(h, s, &sc);
        if (rs != STRADS_OK) return rs;
        sum += sc.updates_total;
    }
    *out = sum;
    return STRADS_OK;
}

static void drop_graphs(strads_lasso *h)
{
    for (int32_t s = 0; s < STRADS_MAX_SHARDS; ++s) {
        if (h->graph_exec[s]) (void)hipGraphExecDestroy(h->graph_exec[s]);
        if (h->graph[s]) (void)hipGraphDestroy(h->graph[s]);
        h->graph_exec[s] = nullptr;
        h->graph[s] = nullptr;
    }
}

// Record h->graph_rounds rounds, starting with the shard whose turn it is, into a HIP graph:
// the caller's stream is put in capture mode, the fork makes the shards' streams part of the
// capture, the join brings them back.  Nothing runs; the host-side round counter is restored.
// Kernel arguments are fixed per handle (the round index lives on the device), so the graph
// stays valid until a tuning knob that changes a launch is touched.
static int record_graph(strads_lasso *h, int32_t first_lane)
{
    const int64_t round0 = h->round;
    if (hipStreamBeginCapture(h->stream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
        // e.g. the caller handed over the legacy default stream, which cannot be captured:
        // from now on rounds are enqueued one by one
        (void)hipGetLastError();
        h->graph_rounds = 0;
        return STRADS_E_UNSUPPORTED;
    }
    int rc = fork_lanes(h);
    for (int32_t i = 0; i < h->graph_rounds && rc == STRADS_OK; ++i) rc = enqueue_round(h, i + 1 < h->graph_rounds);
    if (rc == STRADS_OK) rc = join_lanes(h);
    hipGraph_t g = nullptr;
    const hipError_t e = hipStreamEndCapture(h->stream, &g);
    h->round = round0;
    if (rc != STRADS_OK || e != hipSuccess || !g) {
        if (g) (void)hipGraphDestroy(g);
        return rc != STRADS_OK ? rc : STRADS_E_HIP;
    }
    hipGraphExec_t ex = nullptr;
    if (hipGraphInstantiate(&ex, g, nullptr, nullptr, 0) != hipSuccess) {
        (void)hipGraphDestroy(g);
        return STRADS_E_HIP;
    }
    h->graph[first_lane] = g;
    h->graph_exec[first_lane] = ex;
    return STRADS_OK;
}

// Enqueue `count` rounds: whole groups of graph_rounds as graph replays, the rest one by one.
static int enqueue_rounds(strads_lasso *h, int64_t count, int32_t *replays)
{
    while (h->graph_rounds > 0 && h->profile_level == 0 && count >= h->graph_rounds) {
        const int32_t lane = (int32_t)(h->round % h->n_lanes);
        if (!h->graph_exec[lane]) {
            const int rc = record_graph(h, lane);
            if (rc == STRADS_E_UNSUPPORTED) break;      // this stream cannot be captured
            if (rc != STRADS_OK) return rc;
        }
        HIP_TRY(hipGraphLaunch(h->graph_exec[lane], h->stream));
        *replays += 1;
        h->round += h->graph_rounds;
        count -= h->graph_rounds;
    }
    if (count > 0) {
        int rc = fork_lanes(h);
        for (int64_t i = 0; i < count && rc == STRADS_OK; ++i) rc = enqueue_round(h, i + 1 < count);
        if (rc == STRADS_OK) rc = join_lanes(h);
        if (rc != STRADS_OK) return rc;
    }
    return STRADS_OK;
}

int strads_lasso_round(strads_lasso_t *h, strads_round_info_t *info)
{
    if (!h) return STRADS_E_INVALID_ARG;
    int rc = fork_lanes(h);
    if (rc == STRADS_OK) rc = enqueue_round(h, false);
    if (rc == STRADS_OK) rc = join_lanes(h);
    if (rc != STRADS_OK) return rc;
    if (info) {
        RoundScalars sc;
        const int rs = read_lane_scalars(h, last_lane(h), &sc);
        if (rs != STRADS_OK) return rs;
        info->round = h->round - 1;
        info->n_cand = h->L;
        info->n_kept = sc.n_kept;
        info->n_moved = sc.n_moved;
        info->near_rho_pairs = sc.near_rho_pairs;
        info->max_abs_delta = sc.max_abs_delta;
    }
    return STRADS_OK;
}

int strads_lasso_objective(strads_lasso_t *h, double *out)
{
    if (!h || !out) return STRADS_E_INVALID_ARG;
    HIP_TRY(launch_objective(h));
    double v = 0.0;
    HIP_TRY(hipMemcpyAsync(&v, h->base + h->ws.objout, sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(hipStreamSynchronize(h->stream));
    *out = v;
    return STRADS_OK;
}

int strads_lasso_kkt(strads_lasso_t *h, float *max_violation, float *g_or_null)
{
    if (!h || !max_violation) return STRADS_E_INVALID_ARG;
    const bool timed = h->profile_level != 0;
    if (timed) {
        for (int i = 0; i < 2; ++i)
            if (!h->ev_kkt[i]) HIP_TRY(hipEventCreate(&h->ev_kkt[i]));
        HIP_TRY(hipEventRecord(h->ev_kkt[0], h->stream));
    }
    if (h->cfg.loss == STRADS_LOSS_LOGISTIC) HIP_TRY(launch_logistic_weights(h));
    if (h->cfg.layout == STRADS_LAYOUT_DENSE_COLMAJOR) HIP_TRY(launch_kkt_dense(h, g_or_null));
    else if (h->cfg.layout == STRADS_LAYOUT_GENO2) HIP_TRY(launch_kkt_geno(h, g_or_null));
    else HIP_TRY(launch_kkt_csc(h, g_or_null));
    if (timed) HIP_TRY(hipEventRecord(h->ev_kkt[1], h->stream));
    RoundScalars sc;
    const int rs = read_scalars(h, &sc);
    if (rs != STRADS_OK) return rs;
    h->last_kkt_ms = 0.f;
    if (timed) HIP_TRY(hipEventElapsedTime(&h->last_kkt_ms, h->ev_kkt[0], h->ev_kkt[1]));
    float v;
    memcpy(&v, &sc.kkt_max_bits, 4);
    *max_violation = v;
    return STRADS_OK;
}

int strads_lasso_run(strads_lasso_t *h, int64_t max_rounds, float kkt_tol, int32_t check_every,
                     strads_run_info_t *out)
{
    if (!h || max_rounds < 0 || !(kkt_tol >= 0.f)) return STRADS_E_INVALID_ARG;
    int64_t done = 0;
    float viol = INFINITY;
    int converged = 0;
    int32_t replays = 0;
    // |B_1| is summed on the device; rounds between checks are only enqueued, never waited for
    unsigned long long upd0 = 0, upd1 = 0;
    { const int rs = total_updates(h, &upd0); if (rs != STRADS_OK) return rs; }
    while (done < max_rounds) {
        int64_t burst = max_rounds - done;
        if (check_every > 0 && burst > check_every) burst = check_every;
        int rc = enqueue_rounds(h, burst, &replays);
        if (rc != STRADS_OK) return rc;
        done += burst;
        if (check_every > 0) {
            rc = strads_lasso_kkt(h, &viol, nullptr);
            if (rc != STRADS_OK) return rc;
            if (viol <= kkt_tol * h->cfg.lambda) { converged = 1; break; }
        }
    }
    double obj = 0.0;
    const int rc = strads_lasso_objective(h, &obj);
    if (rc != STRADS_OK) return rc;
    { const int rs = total_updates(h, &upd1); if (rs != STRADS_OK) return rs; }
    if (out) {
        out->rounds_done = done;
        out->updates_done = (int64_t)(upd1 - upd0);
        out->objective = obj;
        out->kkt_violation = viol;
        out->converged = converged;
        out->graph_replays = replays;
    }
    return isfinite(obj) ? STRADS_OK : STRADS_E_DIVERGED;
}

int strads_lasso_get_state(strads_lasso_t *h, float *beta, float *dbeta, float *r, int64_t *round)
{
    if (!h) return STRADS_E_INVALID_ARG;
    if (beta) HIP_TRY(hipMemcpyAsync(beta, h->base + h->ws.beta, (size_t)h->cfg.j * 4, hipMemcpyDeviceToDevice, h->stream));
    if (dbeta) HIP_TRY(hipMemcpyAsync(dbeta, h->base + h->ws.dbeta, (size_t)h->cfg.j * 4, hipMemcpyDeviceToDevice, h->stream));
    if (r) HIP_TRY(hipMemcpyAsync(r, h->base + h->ws.r, (size_t)h->cfg.n * 4, hipMemcpyDeviceToDevice, h->stream));
    HIP_TRY(hipStreamSynchronize(h->stream));
    if (round) *round = h->round;
    return STRADS_OK;
}

int strads_lasso_set_state(strads_lasso_t *h, const float *beta, const float *dbeta, const float *r, int64_t round)
{
    if (!h || round < 0) return STRADS_E_INVALID_ARG;
    if (h->next_keys_done) {
        // (only after a failed enqueue) a key pass made ahead for the round that did not follow: forget it
        HIP_TRY(hipMemsetAsync(h->base + h->ws.hist, 0, (size_t)kHistBins * 4, h->stream));
        h->next_keys_done = 0;
    }
    if (beta) HIP_TRY(hipMemcpyAsync(h->base + h->ws.beta, beta, (size_t)h->cfg.j * 4, hipMemcpyDeviceToDevice, h->stream));
    if (dbeta) HIP_TRY(hipMemcpyAsync(h->base + h->ws.dbeta, dbeta, (size_t)h->cfg.j * 4, hipMemcpyDeviceToDevice, h->stream));
    if (r) HIP_TRY(hipMemcpyAsync(h->base + h->ws.r, r, (size_t)h->cfg.n * 4, hipMemcpyDeviceToDevice, h->stream));
    // shard s runs next the first round >= `round` whose turn is s's
    for (int32_t s = 0; s < h->n_lanes; ++s) {
        const int64_t S = h->n_lanes;
        HIP_TRY(launch_set_next_round(h->lanes[s], h->stream, round + ((s - round % S) + S) % S));
    }
    HIP_TRY(hipStreamSynchronize(h->stream));
    h->round = round;
    return STRADS_OK;
}

int strads_lasso_last_round(strads_lasso_t *h, int32_t *cand, int32_t *kept_pos, float *z, float *delta,
                            float *gram_or_null, int32_t *n_cand, int32_t *n_kept)
{
    if (!h) return STRADS_E_INVALID_ARG;
    if (gram_or_null && (!h->cfg.keep_gram || h->cfg.deps == STRADS_DEPS_NONE)) return STRADS_E_INVALID_ARG;
    const int32_t lane = last_lane(h);
    const Workspace &ws = h->lanes[lane]->ws;           // outputs of the shard that ran the round
    const size_t lb = (size_t)h->L * 4;
    if (cand) HIP_TRY(hipMemcpyAsync(cand, h->base + ws.cand, lb, hipMemcpyDeviceToDevice, h->stream));
    if (kept_pos) HIP_TRY(hipMemcpyAsync(kept_pos, h->base + ws.kept_pos, lb, hipMemcpyDeviceToDevice, h->stream));
    if (z) HIP_TRY(hipMemcpyAsync(z, h->base + ws.z, lb, hipMemcpyDeviceToDevice, h->stream));
    if (delta) HIP_TRY(hipMemcpyAsync(delta, h->base + ws.delta, lb, hipMemcpyDeviceToDevice, h->stream));
    if (gram_or_null && h->cfg.deps == STRADS_DEPS_DYNAMIC) {
        strads_lasso view = *h->lanes[lane];            // the shard's buffers, on the caller's stream
        view.stream = h->stream;
        HIP_TRY(launch_scatter_mover_gram(&view, gram_or_null));
    } else if (gram_or_null) {
        HIP_TRY(hipMemcpy2DAsync(gram_or_null, lb, h->base + ws.gram, (size_t)h->Lpad * 4, lb, (size_t)h->L,
                                 hipMemcpyDeviceToDevice, h->stream));
    }
    RoundScalars sc;
    const int rs = read_lane_scalars(h, lane, &sc);
    if (rs != STRADS_OK) return rs;
    if (n_cand) *n_cand = h->L;
    if (n_kept) *n_kept = sc.n_kept;
    return STRADS_OK;
}

int strads_lasso_last_candidates(strads_lasso_t *h, float *z_cand, float *delta_cand, int32_t *n_movers)
{
    if (!h) return STRADS_E_INVALID_ARG;
    if (h->cfg.deps != STRADS_DEPS_DYNAMIC) return STRADS_E_UNSUPPORTED;
    const size_t lb = (size_t)h->L * 4;
    const int32_t lane = last_lane(h);
    const Workspace &ws = h->lanes[lane]->ws;
    if (z_cand) HIP_TRY(hipMemcpyAsync(z_cand, h->base + ws.zc, lb, hipMemcpyDeviceToDevice, h->stream));
    if (delta_cand) HIP_TRY(hipMemcpyAsync(delta_cand, h->base + ws.dc, lb, hipMemcpyDeviceToDevice, h->stream));
    RoundScalars sc;
    const int rs = read_lane_scalars(h, lane, &sc);
    if (rs != STRADS_OK) return rs;
    if (n_movers) *n_movers = sc.n_movers;
    return STRADS_OK;
}

int strads_lasso_stage_keys(strads_lasso_t *h, int64_t round, float *keys_out)
{
    if (!h || !keys_out || round < 0) return STRADS_E_INVALID_ARG;
    HIP_TRY(launch_keys_only(h, round, keys_out));
    HIP_TRY(hipStreamSynchronize(h->stream));
    return STRADS_OK;
}

int strads_lasso_stage_filter(strads_lasso_t *h, const float *gram, int32_t l, int32_t *kept_pos, int32_t *n_kept)
{
    if (!h || !gram || !kept_pos || !n_kept || l < 1 || l > h->L) return STRADS_E_INVALID_ARG;
    HIP_TRY(launch_mask_from_gram(h, gram, l));
    HIP_TRY(launch_filter(h, l, false, false, false));
    RoundScalars sc;
    const int rs = read_scalars(h, &sc);
    if (rs != STRADS_OK) return rs;
    if (sc.n_kept > 0) {
        HIP_TRY(hipMemcpyAsync(kept_pos, h->base + h->ws.kept_pos, (size_t)sc.n_kept * 4, hipMemcpyDeviceToDevice,
                               h->stream));
        HIP_TRY(hipStreamSynchronize(h->stream));
    }
    *n_kept = sc.n_kept;
    return STRADS_OK;
}

int strads_lasso_gram256_plan(int64_t n, int32_t l, int32_t items_cap, int32_t *n_items, int32_t *items,
                              int32_t *first_slot, int32_t *n_slots)
{
    if (n < 1 || l < 1 || l > STRADS_MAX_L_PRIME || items_cap < 0 || !n_items || (items_cap > 0 && !items) ||
        !first_slot || !n_slots)
        return STRADS_E_INVALID_ARG;
    const int32_t lpad = (l + kGramTile - 1) / kGramTile * kGramTile;
    *n_items = gram256_plan_host(n, lpad, items_cap, items, first_slot, n_slots);
    return STRADS_OK;
}

int strads_lasso_gram_default_tile_edge(int64_t n, int32_t l, int32_t layout, int32_t deps, int32_t *edge)
{
    if (n < 1 || l < 1 || l > STRADS_MAX_L_PRIME || !edge || layout < STRADS_LAYOUT_DENSE_COLMAJOR ||
        layout > STRADS_LAYOUT_GENO2 || deps < STRADS_DEPS_STATIC || deps > STRADS_DEPS_NONE)
        return STRADS_E_INVALID_ARG;
    const int32_t lpad = (l + kGramTile - 1) / kGramTile * kGramTile;
    if (layout == STRADS_LAYOUT_CSC || deps == STRADS_DEPS_NONE) *edge = 0;
    else if (gram256_default(n, lpad, layout, deps)) *edge = 256;
    else if (deps == STRADS_DEPS_STATIC && gram_direct_default(n, lpad)) *edge = 64;
    else *edge = kGramTile;
    return STRADS_OK;
}

int strads_lasso_gram_tile_edge(strads_lasso_t *h, int32_t *edge)
{
    if (!h || !edge) return STRADS_E_INVALID_ARG;
    if (h->cfg.layout == STRADS_LAYOUT_CSC || h->cfg.deps == STRADS_DEPS_NONE) { *edge = 0; return STRADS_OK; }
    *edge = h->cfg.deps == STRADS_DEPS_STATIC && h->big_items > 0 ? 256 : (gram_direct_on(h) ? 64 : kGramTile);
    return STRADS_OK;
}

int strads_lasso_set_tuning(strads_lasso_t *h, const char *name, int64_t value)
{
    if (!h || !name) return STRADS_E_INVALID_ARG;
    if (strcmp(name, "graph_rounds") == 0) {
        if (value < 0 || value > 4096) return STRADS_E_INVALID_ARG;
#ifdef STRADS_DEBUG_SYNC
        if (value > 0) return STRADS_E_UNSUPPORTED;     // a debug build waits after every launch; a capture cannot
#endif
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);
        h->graph_rounds = (int32_t)value;
        return STRADS_OK;
    }
    if (strcmp(name, "gram_split_k") == 0) {
        if (value < 0 || value > h->split_max) return STRADS_E_INVALID_ARG;
        if (value != 0 && h->cfg.deps == STRADS_DEPS_DYNAMIC) return STRADS_E_UNSUPPORTED;   // chosen on the device
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);                                 // recorded launches carry the old decomposition
        for (int32_t s = 0; s < h->n_lanes; ++s) h->lanes[s]->split_user = (int32_t)value;
        if (h->jobtab_on) {                             // the job numbering follows the decomposition
            const int rc = upload_job_table(h);
            if (rc != STRADS_OK) return rc;
            HIP_TRY(hipStreamSynchronize(h->stream));
        }
        return STRADS_OK;
    }
    if (strcmp(name, "gram_xcd_map") == 0) {
        if (value < 0 || value > 1) return STRADS_E_INVALID_ARG;
        if (h->cfg.layout == STRADS_LAYOUT_CSC || h->cfg.deps == STRADS_DEPS_DYNAMIC) return STRADS_E_UNSUPPORTED;
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);
        for (int32_t s = 0; s < h->n_lanes; ++s) h->lanes[s]->jobtab_on = (int32_t)value;
        return STRADS_OK;
    }
    if (strcmp(name, "gram_tile256") == 0) {
        if (value < 0 || value > 2) return STRADS_E_INVALID_ARG;
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);
        for (int32_t s = 0; s < h->n_lanes; ++s) h->lanes[s]->tile256 = (int32_t)value;
        const int rc = choose_gram_route(h);
        if (rc != STRADS_OK) return rc;
        return value == 2 && h->big_items == 0 ? STRADS_E_UNSUPPORTED : STRADS_OK;
    }
    if (strcmp(name, "gram_direct") == 0) {
        if (value < 0 || value > 2) return STRADS_E_INVALID_ARG;
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);
        for (int32_t s = 0; s < h->n_lanes; ++s) h->lanes[s]->direct = (int32_t)value;
        return value == 2 && !gram_direct_on(h) ? STRADS_E_UNSUPPORTED : STRADS_OK;
    }
    if (strcmp(name, "dots_with_gram") == 0) {
        if (value < 0 || value > 1) return STRADS_E_INVALID_ARG;
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);
        for (int32_t s = 0; s < h->n_lanes; ++s) h->lanes[s]->dots_with_gram = (int32_t)value;
        return STRADS_OK;
    }
    if (strcmp(name, "early_keys") == 0) {
        if (value < 0 || value > 1) return STRADS_E_INVALID_ARG;
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);
        h->early_keys = (int32_t)value;
        return STRADS_OK;
    }
    if (strcmp(name, "residual_fused") == 0) {
        if (value < 0 || value > 1) return STRADS_E_INVALID_ARG;
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);
        for (int32_t s = 0; s < h->n_lanes; ++s) h->lanes[s]->residual_fused = (int32_t)value;
        return STRADS_OK;
    }
    if (strcmp(name, "profile_rounds") == 0) {
        if (value < 1 || value > 1 << 20 || h->profile_level != 0) return STRADS_E_INVALID_ARG;
        h->profile_rounds = (int32_t)value;
        return STRADS_OK;
    }
    if (strcmp(name, "profile_level") == 0) {
        if (value < 0 || value > 2) return STRADS_E_INVALID_ARG;
        if (value != 0 && h->n_lanes > 1) return STRADS_E_UNSUPPORTED;   // stages of different shards overlap
        HIP_TRY(hipStreamSynchronize(h->stream));
        const int32_t keep_rounds = h->profile_rounds;
        drop_events(h);
        h->profile_rounds = keep_rounds;
        if (value == 0) return STRADS_OK;
        const size_t n = (size_t)h->profile_rounds * kStageEvents;
        h->events = (hipEvent_t *)calloc(n, sizeof(hipEvent_t));
        if (!h->events) return STRADS_E_INVALID_ARG;
        for (size_t i = 0; i < n; ++i)
            if (hipEventCreate(&h->events[i]) != hipSuccess) { drop_events(h); return STRADS_E_HIP; }
        h->profile_level = (int32_t)value;
        return STRADS_OK;
    }
    if (strcmp(name, "select_cap") == 0) {
        if (value < 1 || value > 2 * STRADS_MAX_L_PRIME) return STRADS_E_INVALID_ARG;
        HIP_TRY(hipStreamSynchronize(h->stream));
        drop_graphs(h);
        for (int32_t s = 0; s < h->n_lanes; ++s) h->lanes[s]->select_cap = (int32_t)value;
        return STRADS_OK;
    }
    return STRADS_E_INVALID_ARG;
}

int strads_lasso_stage_times(strads_lasso_t *h, float *avg_ms, int32_t *rounds_timed)
{
    if (!h || !avg_ms || !rounds_timed) return STRADS_E_INVALID_ARG;
    HIP_TRY(hipStreamSynchronize(h->stream));
    double sum[STRADS_N_STAGES];
    for (int s = 0; s < STRADS_N_STAGES; ++s) sum[s] = 0.0;
    for (int32_t r = 0; r < h->profiled; ++r) {
        hipEvent_t *e = h->events + (size_t)r * kStageEvents;
        for (int s = 0; s < STRADS_N_STAGES; ++s) {
            if (h->profile_level == 1 && s != STRADS_STAGE_GRAM_TILES) continue;
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, e[s], e[s + 1]));
            sum[s] += ms;
        }
    }
    for (int s = 0; s < STRADS_N_STAGES; ++s) avg_ms[s] = h->profiled > 0 ? (float)(sum[s] / h->profiled) : 0.f;
    *rounds_timed = h->profiled;
    h->profiled = 0;
    return STRADS_OK;
}

int strads_lasso_last_kkt_ms(strads_lasso_t *h, float *ms)
{
    if (!h || !ms) return STRADS_E_INVALID_ARG;
    *ms = h->last_kkt_ms;
    return STRADS_OK;
}

int strads_lasso_debug_build(void)
{
#ifdef STRADS_DEBUG_SYNC
    return 1;
#else
    return 0;
#endif
}

const char *strads_lasso_strerror(int code)
{
    switch (code) {
    case STRADS_OK: return "ok";
    case STRADS_E_INVALID_ARG: return "invalid argument";
    case STRADS_E_WORKSPACE_TOO_SMALL: return "workspace too small";
    case STRADS_E_HIP: return "HIP runtime error";
    case STRADS_E_DIVERGED: return "objective is not finite";
    case STRADS_E_UNSUPPORTED: return "not supported";
    case STRADS_E_TOO_LARGE: return "size exceeds the fixed maximum of this entry point";
    default: return "unknown error";
    }
}

} // extern "C"
