// Step 2 of SAP for the Lasso, second half (Algorithm 1's choice of B_1: at most P of the drawn
// candidates, every pair of them correlated below rho): walk the candidates in draw order and keep
// one iff it conflicts with nothing kept so far.
//
// The walk is sequential in the kept set, so the work is arranged to keep the serial chain short.
// One small workgroup takes the candidates 64 at a time (a "chunk").  `dead` (one bit per candidate,
// in LDS) marks candidates that conflict with something already kept.
//   * Wavefront 0 decides the chunk: candidates that are alive and have no conflict with another
//     alive candidate of the chunk are kept at once; only the few with an in-chunk conflict are
//     walked one by one (scalar bit operations on the chunk's 64x64 diagonal block, which its lanes
//     load themselves).
//   * The other wavefronts hold the chunks' conflict rows (words right of the chunk's own word) in
//     registers and OR the rows of the newly kept candidates into `dead` for later chunks.  The mask
//     was written by workgroups all over the chip, so its first read by this workgroup comes from
//     memory, a microsecond or more away, while a chunk is decided in a fraction of that: the rows
//     are fetched several chunks ahead of their use.
// The details, and what they are there to avoid, are at k_filter.
// Only bits (a, b) with b in a's 128-tile or right of it are read, matching what the Gram
// kernel writes.  Bit-exact: the result depends on the conflict bits only.
#include <string.h>

#include "strads_internal.h"

namespace strads {

__device__ __forceinline__ uint64_t readlane64(uint64_t v, int l)
{
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}

constexpr int kMaxWords = STRADS_MAX_L_PRIME / 64;   // mask words per row (128)

// Dynamic dependencies: what the walk over the movers is followed by, in the same workgroup (a
// kernel of its own would cost a launch boundary, a good part of a short round).
struct CommitArgs {
    int32_t on;                 // 0: plain filter (the fields below are unused); kCommitDynamic; kCommitKept
    int32_t L;                  // all candidates of the round
    const float *zc, *dc, *nbc; // every candidate's x_j^T r, tentative change and tentative value
    const int32_t *cand;        // all candidates in draw order
    const int32_t *mpos;        // mover -> candidate position
    float *beta, *dbeta;
    int32_t *kept_pos, *kept;
    float *z, *delta;
};

constexpr int32_t kCommitDynamic = 1;  // dynamic dependencies: the walk ran over the movers, see commit_dynamic
constexpr int32_t kCommitKept = 2;     // Algorithm 1's rule: eq. (2) for the kept candidates from their tentative updates

// Assemble B_1 = (candidates that do not move) + (movers that passed the filter), in draw order,
// cut at the cap, and commit it: beta_j <- its tentative value, delta beta_j <- |change| (0 for a
// kept candidate that does not move).  mkept[a] (LDS, one byte per candidate position) says whether a
// mover at position a passed the filter.  Three phases with a barrier between them, whatever the
// length of the list: one keep bit per candidate, gathered into 64-bit words by wavefront ballots;
// the number of kept candidates before every word (one wavefront); the writes.
//
// e_*: what the caller requested early of candidates tid + k * blockDim.x, k < K (see k_filter).
template <int K>
__device__ __forceinline__ void commit_dynamic(const CommitArgs &cm, int32_t p_max, const uint8_t *mkept,
                                               RoundScalars *__restrict__ sc, const int32_t *e_cand,
                                               const float *e_dc, const float *e_zc, const float *e_nbc)
{
    __shared__ uint64_t keepw[kMaxWords];
    __shared__ int32_t before[kMaxWords + 1];
    const int tid = threadIdx.x, lane = tid & 63;
    const int nthreads = blockDim.x;
    const int32_t L = cm.L;
    const int32_t cap = p_max > 0 ? p_max : L;
    const int32_t nwords = (L + 63) / 64;
#pragma unroll
    for (int k = 0; k < K; ++k) {                                   // whole wavefronts: nthreads is a multiple of 64
        const int32_t a = tid + k * nthreads;
        if (k * nthreads < nwords * 64) {
            const bool keep = a < L && (e_dc[k] == 0.f || mkept[a]);
            const uint64_t m = __ballot(keep);
            if (lane == 0 && a < nwords * 64) keepw[a >> 6] = m;
        }
    }
    // (the rest of a long list four positions per thread at a time, their loads requested together: one
    // trip to memory per four positions instead of one per position)
    constexpr int kBatch = 4;
    for (int32_t a0 = K * nthreads; a0 < nwords * 64; a0 += kBatch * nthreads) {
        float d4[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int32_t a = a0 + u * nthreads + tid;
            d4[u] = a < L ? cm.dc[a] : 1.f;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int32_t a = a0 + u * nthreads + tid;
            if (a0 + u * nthreads < nwords * 64) {                  // whole wavefronts
                const bool keep = a < L && (d4[u] == 0.f || mkept[a]);
                const uint64_t m = __ballot(keep);
                if (lane == 0 && a < nwords * 64) keepw[a >> 6] = m;
            }
        }
    }
    __syncthreads();
    if (tid < 64) {                                                 // at most 128 words: two per lane
        const int32_t w0 = 2 * lane, w1 = 2 * lane + 1;
        const int32_t c0 = w0 < nwords ? __popcll(keepw[w0]) : 0, c1 = w1 < nwords ? __popcll(keepw[w1]) : 0;
        int32_t incl = c0 + c1;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int32_t v = __shfl_up(incl, d);
            if (lane >= d) incl += v;
        }
        if (w0 < nwords) before[w0] = incl - c0 - c1;
        if (w1 < nwords) before[w1] = incl - c1;
        if (lane == 63) before[kMaxWords] = incl;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int32_t a = tid + k * nthreads;
        if (a >= L) continue;
        const uint64_t w = keepw[a >> 6];
        if (!((w >> (a & 63)) & 1ull)) continue;
        const int32_t idx = before[a >> 6] + __popcll(w & ((1ull << (a & 63)) - 1ull));
        if (idx >= cap) continue;
        const int32_t j = e_cand[k];
        cm.kept_pos[idx] = a;
        cm.kept[idx] = j;
        cm.z[idx] = e_zc[k];
        cm.delta[idx] = e_dc[k];
        cm.beta[j] = e_nbc[k];
        cm.dbeta[j] = fabsf(e_dc[k]);
    }
    for (int32_t a0 = tid + K * nthreads; a0 < L; a0 += kBatch * nthreads) {
        int32_t j4[kBatch];
        float d4[kBatch], z4[kBatch], nb4[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int32_t a = a0 + u * nthreads, at = a < L ? a : 0;
            j4[u] = cm.cand[at]; d4[u] = cm.dc[at]; z4[u] = cm.zc[at]; nb4[u] = cm.nbc[at];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int32_t a = a0 + u * nthreads;
            if (a >= L) continue;
            const uint64_t w = keepw[a >> 6];
            if (!((w >> (a & 63)) & 1ull)) continue;
            const int32_t idx = before[a >> 6] + __popcll(w & ((1ull << (a & 63)) - 1ull));
            if (idx >= cap) continue;
            cm.kept_pos[idx] = a;
            cm.kept[idx] = j4[u];
            cm.z[idx] = z4[u];
            cm.delta[idx] = d4[u];
            cm.beta[j4[u]] = nb4[u];
            cm.dbeta[j4[u]] = fabsf(d4[u]);
        }
    }
    if (tid == 0) {
        const int32_t total = before[kMaxWords];
        const int32_t nk = total < cap ? total : cap;
        sc->n_kept = nk;
        sc->updates_total += (unsigned long long)nk;
    }
}

// TPR = holder threads per row of a chunk (4; 8 for rows of more than 64 words), IPT = words of a row per
// holder thread = ceil(W / TPR): 4, 8 or 16.  A = chunks whose words a thread has in registers or on
// their way there (chunk c waits in set c mod A).
//
// The workgroup is five (nine) wavefronts, one to three per SIMD: with sixteen the chunk loop was bound
// by instruction issue, four wavefronts taking turns on every SIMD for a few dozen instructions each.
// Roles, one barrier per chunk c:
//   wavefront 0 decides chunk c.  The dead bits of the chunk are dead[c]: what the rows kept in chunks
//     <= c-2 do to word c was ORed in by the holders, what the rows kept in chunk c-1 do to it by
//     wavefront 0 itself when it decided c-1 (its lanes hold word c of those rows; LDS operations of
//     one wavefront complete in order).  Lane l loads words c and c+1 of row 64c + l itself, A chunks
//     early, so a chunk costs it one LDS round trip and a few dozen instructions.  That chain is what
//     the walk is bound by (measured: some 500 cycles from the barrier to the chunk's dead word in a
//     scalar register, 250 for the quick decision, 250 to get the results into LDS; a lone wavefront
//     spends about ten cycles per instruction of a dependent chain with its branches).
//   holders (the other wavefronts; TPR threads per row of a chunk, thread j of a row owning words j, j+TPR, ...):
//     OR the words they hold of the rows kept in chunk c-1 into dead[w], w > c, and refill those
//     registers with chunk c-1+A.
// Each role runs its own loop (same trip count, same barriers), every load in it is unconditional,
// from an address clamped into the mask, and sits at a fixed place of the unrolled body: only then
// does the compiler wait for the load it needs rather than for all outstanding ones, which would put
// a memory round trip into every chunk.  Nothing is stored to global memory inside the loop for the
// same reason.  Rows at or past L and words at or right of a row's diagonal word are written by the
// mask kernel for every row below Lpad; words left of the diagonal are never used.
//
// FLAGS: the mask kernel has marked the chunks (sc->chunk_nz) any of whose rows has a nonzero word two or more
// words right of its diagonal word, which are the words the holders use.  The holders neither fetch nor look at
// the rows of an unmarked chunk: with few conflicts (a long list drawn from nearly orthogonal columns) the walk
// is otherwise bound by one compute unit reading the whole mask, 8 MB for 8000 candidates.  The marks are read
// once at the start, and cleared for the next round at the end.
template <int IPT, int A, int TPR, bool FLAGS>
__global__ __launch_bounds__(64 + 64 * TPR) void k_filter(const uint64_t *__restrict__ mask, int32_t L, int32_t W,
                                                           const GramShape *__restrict__ gdev,
                                                           int32_t p_max, const int32_t *__restrict__ cand,
                                                           int32_t *kept_pos, int32_t *__restrict__ kept,
                                                           RoundScalars *__restrict__ sc, int32_t *__restrict__ n_out,
                                                           int count_updates, CommitArgs cm)
{
    constexpr int kThreads = 64 + 64 * TPR;
    __shared__ uint8_t mkept[STRADS_MAX_L_PRIME];       // dynamic dependencies: 1 = a mover at this candidate position was kept
    if (gdev) { L = gdev->L; W = gdev->Lpad / 64; }   // dynamic dependencies: the movers, counted on the device
    if (cm.on == kCommitDynamic)
        for (int32_t a = threadIdx.x; a < cm.L; a += kThreads) mkept[a] = 0;      // (the barriers below order it)
    // Short and medium lists that end with eq. (2) for kept candidates: what that needs of the
    // thread's first candidates (positions in the round's candidate list) is requested now, and has
    // arrived long before the walk is over.
    constexpr int kEarly = IPT <= 8 ? 4 : 0;
    int32_t e_cand[kEarly > 0 ? kEarly : 1];
    float e_dc[kEarly > 0 ? kEarly : 1], e_zc[kEarly > 0 ? kEarly : 1], e_nbc[kEarly > 0 ? kEarly : 1];
    if (cm.on != 0) {
#pragma unroll
        for (int k = 0; k < kEarly; ++k) {
            const int32_t a = (int32_t)threadIdx.x + k * kThreads;
            const int32_t at = a < cm.L ? a : 0;
            e_cand[k] = cm.cand[at]; e_dc[k] = cm.dc[at]; e_zc[k] = cm.zc[at]; e_nbc[k] = cm.nbc[at];
        }
    }
    if (L <= 0) {                                      // nothing moves this round
        if (threadIdx.x == 0) *n_out = 0;
        if (cm.on == kCommitDynamic) {
            __syncthreads();
            commit_dynamic<kEarly>(cm, p_max, mkept, sc, e_cand, e_dc, e_zc, e_nbc);
        }
        return;
    }
    __shared__ uint64_t dead[kMaxWords];
    __shared__ uint64_t keptw_all[kMaxWords];     // [c]: the candidates kept in chunk c
    __shared__ int32_t nkb[kMaxWords + 1];        // [c]: kept before chunk c.  (Positions go to global memory
                                                  // after the walk.)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int32_t cap = (p_max > 0 && cm.on != kCommitDynamic) ? p_max : L;   // the movers' walk has no cap: commit_dynamic applies it
    const int32_t chunks = (L + 63) / 64;
    const int64_t chunk_stride = (int64_t)64 * W; // words from a chunk's rows to the next chunk's
    const int32_t c_max = W - 1;                  // chunk index up to which a chunk's rows lie inside the mask (chunks <= W)

    __shared__ uint8_t nzc[FLAGS ? kMaxWords : 1];  // [c]: the holders have something to do for chunk c
    for (int i = tid; i < W; i += kThreads) {
        dead[i] = 0;
        // (the first A chunks are fetched before the marks have arrived)
        if constexpr (FLAGS) nzc[i] = (i < A || sc->chunk_nz[i] != 0u) ? 1 : 0;
    }
    if (tid == 0) nkb[0] = 0;
    __syncthreads();

    int32_t n_done = 0;                           // chunks decided
    if (wave == 0) {
        // ---- the decider ----
        // words c and c+1 of row 64c + lane
        uint64_t dgq[A], nxq[A];
        // chunks are fetched in order, so the address is carried along: from chunk to chunk the
        // diagonal word moves 64 rows down and one word right; past the last chunk inside the mask
        // the pointer stays (the values are not used)
        const uint64_t *dptr = mask + (int64_t)lane * W;
        int32_t c_next = 0;                       // the chunk dptr points at
        auto fetch_diag = [&](uint64_t &d0, uint64_t &d1) {
            d0 = dptr[0];
            d1 = dptr[c_next < c_max ? 1 : 0];
            if (c_next < c_max) { dptr += chunk_stride + 1; ++c_next; }
        };
#pragma unroll
        for (int d = 0; d < A; ++d) fetch_diag(dgq[d], nxq[d]);
        int32_t nk = 0;                           // kept so far
        const uint32_t lane_lo = lane < 32 ? 1u << lane : 0u, lane_hi = lane >= 32 ? 1u << (lane - 32) : 0u;
        const uint64_t last_valid = (L & 63) ? (1ull << (L & 63)) - 1ull : ~0ull;     // live lanes of the last chunk
        for (int32_t c0 = 0; c0 < chunks; c0 += A) {
            bool stop = false;
#pragma unroll
            for (int d = 0; d < A; ++d) {
                const int32_t c = c0 + d;
                if (stop || c >= chunks) break;
                const uint64_t cur = dead[c];
                const uint64_t dgv = dgq[d], nxv = nxq[d];
                fetch_diag(dgq[d], nxq[d]);
                const uint64_t alive = ~cur & (c + 1 < chunks ? ~0ull : last_valid);
                uint64_t keptw = 0;
                if (nk < cap) {
                    // lanes whose row meets another alive candidate of this chunk need the serial walk
                    const uint64_t tangled = __ballot((dgv & alive) != 0) & alive;
                    const uint64_t freeb = alive & ~tangled;
                    if (tangled == 0 && nk + __popcll(freeb) <= cap) {
                        keptw = freeb;
                        nk += __popcll(freeb);
                    } else {
                        uint64_t todo = alive;
                        while (todo != 0 && nk < cap) {       // uniform across the wavefront
                            // free candidates before the next tangled one are kept in one step
                            const uint64_t tn = todo & tangled;
                            const int l = tn ? __ffsll((long long)tn) - 1 : 64;
                            uint64_t run = todo & (l >= 64 ? ~0ull : ((1ull << l) - 1ull));
                            int32_t nrun = __popcll(run);
                            if (nk + nrun > cap) {            // the cap cuts the run: keep its first cap-nk bits
                                while (nrun > cap - nk) { run &= ~(1ull << (63 - __builtin_clzll(run))); --nrun; }
                                keptw |= run; nk += nrun; todo = 0; break;
                            }
                            keptw |= run; nk += nrun; todo &= ~run;
                            if (l >= 64 || nk >= cap) break;
                            keptw |= 1ull << l;
                            ++nk;
                            todo &= ~(1ull << l);
                            todo &= ~readlane64(dgv, l);
                        }
                    }
                }
                if (lane == 0) { keptw_all[c] = keptw; nkb[c + 1] = nk; }
                // what this chunk's kept rows do to the next chunk's word
                const bool mine = (((uint32_t)keptw & lane_lo) | ((uint32_t)(keptw >> 32) & lane_hi)) != 0u;
                if (mine && nxv != 0 && c + 1 < chunks)
                    atomicOr((unsigned long long *)&dead[c + 1], (unsigned long long)nxv);
                __syncthreads();
                n_done = c + 1;
                stop = nk >= cap;
            }
            if (stop) break;
        }
    } else {
        // ---- the holders ----
        const int hid = tid - 64;
        const int row = hid / TPR, j = hid % TPR; // the thread's row of every chunk; it owns words j + TPR q
        const uint32_t row_lo = row < 32 ? 1u << row : 0u, row_hi = row >= 32 ? 1u << (row - 32) : 0u;
        uint64_t pre[A][IPT];
        // chunk c's words of this thread are at mask + (64 c + row) W + j + 4 q; chunks are fetched in
        // order, so the row pointer is carried along (it stays on the last chunk inside the mask)
        const uint64_t *rowp = mask + (int64_t)row * W;
        int32_t c_next = 0;
        int32_t wq[IPT];                          // j + TPR q, clamped into the row
#pragma unroll
        for (int q = 0; q < IPT; ++q) wq[q] = j + TPR * q < W ? j + TPR * q : W - 1;
        auto fetch = [&](uint64_t (&dst)[IPT], bool on) {
            if (on) {                           // (uniform; always true without FLAGS)
#pragma unroll
                for (int q = 0; q < IPT; ++q) {
                    if constexpr (FLAGS) {      // (the clamped word index computed here: registers are short)
                        const int32_t w = j + TPR * q;
                        dst[q] = rowp[w < W ? w : W - 1];
                    } else {
                        dst[q] = rowp[wq[q]];
                    }
                }
            }
            if (c_next < c_max) { rowp += chunk_stride; ++c_next; }
        };
        auto marked = [&](int32_t c) -> bool {    // uniform
            if constexpr (FLAGS) return c < chunks && __builtin_amdgcn_readfirstlane((int)nzc[c]) != 0;
            return true;
        };
#pragma unroll
        for (int d = 0; d < A; ++d) fetch(pre[d], true);
        for (int32_t c0 = 0; c0 < chunks; c0 += A) {
            bool stop = false;
#pragma unroll
            for (int d = 0; d < A; ++d) {
                const int32_t c = c0 + d;
                if (stop || c >= chunks) break;
                if (c > 0) {
                    // the rows kept in chunk c-1 -> dead[w], w > c
                    uint64_t (&prev)[IPT] = pre[(d + A - 1) % A];
                    const uint64_t keptw = keptw_all[c - 1];
                    if ((((uint32_t)keptw & row_lo) | ((uint32_t)(keptw >> 32) & row_hi)) != 0u && marked(c - 1)) {
#pragma unroll
                        for (int q = 0; q < IPT; ++q) {
                            const int32_t w = j + TPR * q;
                            const uint64_t v = prev[q];
                            if (w > c && w < W && v != 0)
                                atomicOr((unsigned long long *)&dead[w], (unsigned long long)v);
                        }
                    }
                    fetch(prev, marked(c - 1 + A));   // chunk c-1 is done with its registers: they take chunk c-1+A
                }
                __syncthreads();
                n_done = c + 1;
                stop = nkb[c + 1] >= cap;
            }
            if (stop) break;
        }
    }
    __syncthreads();
    n_done = __builtin_amdgcn_readfirstlane(n_done);
    if constexpr (FLAGS)
        for (int i = tid; i < W; i += kThreads) sc->chunk_nz[i] = 0u;

    // The kept positions, in order, from the per-chunk words: candidate a is number
    // nkb[a / 64] + (kept candidates of its chunk before it); with them the column ids and, where the
    // candidates' updates are already known, eq. (2) and Step 4 for B_1.
    const int32_t nkf = nkb[n_done];
    const int32_t a_end = n_done * 64 < L ? n_done * 64 : L;
    int32_t a_first = tid;
    if (cm.on == kCommitKept) {
#pragma unroll
        for (int k = 0; k < kEarly; ++k) {      // the candidates whose values were requested at the start
            const int32_t a = tid + k * kThreads;
            if (a < a_end) {
                const uint64_t w = keptw_all[a >> 6];
                if ((w >> (a & 63)) & 1ull) {
                    const int32_t i = nkb[a >> 6] + __popcll(w & ((1ull << (a & 63)) - 1ull));
                    const int32_t j = e_cand[k];
                    kept_pos[i] = a;
                    kept[i] = j;
                    cm.z[i] = e_zc[k];
                    cm.delta[i] = e_dc[k];
                    cm.beta[j] = e_nbc[k];
                    cm.dbeta[j] = fabsf(e_dc[k]);
                }
            }
        }
        a_first = tid + kEarly * kThreads;
    }
    // (four positions per thread at a time, their loads requested together)
    constexpr int kBatch = 4;
    for (int32_t a0 = a_first; a0 < a_end; a0 += kBatch * kThreads) {
        int32_t j4[kBatch];                       // the candidate's column; dynamic dependencies: its place in the candidate list
        float d4[kBatch], z4[kBatch], nb4[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int32_t a = a0 + u * kThreads, at = a < a_end ? a : 0;
            j4[u] = cm.on == kCommitDynamic ? cm.mpos[at] : cand[at];
            if (cm.on == kCommitKept) { d4[u] = cm.dc[at]; z4[u] = cm.zc[at]; nb4[u] = cm.nbc[at]; }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int32_t a = a0 + u * kThreads;
            if (a >= a_end) continue;
            const uint64_t w = keptw_all[a >> 6];
            if (!((w >> (a & 63)) & 1ull)) continue;
            const int32_t i = nkb[a >> 6] + __popcll(w & ((1ull << (a & 63)) - 1ull));
            kept_pos[i] = a;
            if (cm.on == kCommitKept) {
                kept[i] = j4[u];
                cm.z[i] = z4[u];
                cm.delta[i] = d4[u];
                cm.beta[j4[u]] = nb4[u];
                cm.dbeta[j4[u]] = fabsf(d4[u]);
            } else if (cm.on == kCommitDynamic) {
                mkept[j4[u]] = 1;                 // a is a position in the mover list here
            } else {
                kept[i] = j4[u];
            }
        }
    }
    if (cm.on == kCommitDynamic) {
        if (tid == 0) *n_out = nkf;
        __syncthreads();
        commit_dynamic<kEarly>(cm, p_max, mkept, sc, e_cand, e_dc, e_zc, e_nbc);
        return;
    }
    if (tid == 0) {
        *n_out = nkf;
        if (count_updates) sc->updates_total += (unsigned long long)nkf;
    }
}

// Launch for row width W (words); with gdev the kernel takes the actual length and width from
// device memory (they can only be smaller).
// marked: the mask was written this round by the kernel that marks chunks in sc->chunk_nz (see k_filter).
static hipError_t launch_filter_kernel(hipStream_t stream, const uint64_t *mask, RoundScalars *sc, int32_t l, int32_t W,
                                       const GramShape *gdev, int32_t p_max,
                                       const int32_t *cand, int32_t *kept_pos, int32_t *kept, int32_t *n_out,
                                       bool count_updates, const CommitArgs &cm, bool marked)
{
#define STRADS_FILTER(IPT, A, TPR, FLAGS) hipLaunchKernelGGL((k_filter<IPT, A, TPR, FLAGS>), dim3(1), dim3(64 + 64 * TPR), 0, stream, mask, l, W, gdev, p_max, cand, kept_pos, kept, sc, n_out, count_updates ? 1 : 0, cm)
    // words of a row per holder thread = ceil(W / threads per row); short rows can afford more chunks in flight
    if (W <= 16) STRADS_FILTER(4, 8, 4, false);
    else if (W <= 32) STRADS_FILTER(4, 6, 8, false);
    else if (W <= 64) { if (marked) STRADS_FILTER(8, 4, 8, true); else STRADS_FILTER(8, 4, 8, false); }
    else { if (marked) STRADS_FILTER(16, 3, 8, true); else STRADS_FILTER(16, 3, 8, false); }
#undef STRADS_FILTER
    return launch_status(stream);
}

static CommitArgs commit_args(strads_lasso *h, int32_t mode)
{
    CommitArgs cm;
    cm.on = mode;
    cm.L = h->L;
    cm.zc = h->at<float>(h->ws.zc);
    cm.dc = h->at<float>(h->ws.dc);
    cm.nbc = h->at<float>(h->ws.nbc);
    cm.cand = h->at<int32_t>(h->ws.cand);
    cm.mpos = h->at<int32_t>(h->ws.mpos);
    cm.beta = h->at<float>(h->ws.beta);
    cm.dbeta = h->at<float>(h->ws.dbeta);
    cm.kept_pos = h->at<int32_t>(h->ws.kept_pos);
    cm.kept = h->at<int32_t>(h->ws.kept);
    cm.z = h->at<float>(h->ws.z);
    cm.delta = h->at<float>(h->ws.delta);
    return cm;
}

hipError_t launch_filter(strads_lasso *h, int32_t l, bool count_updates, bool commit, bool marked)
{
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    return launch_filter_kernel(h->stream, h->at<uint64_t>(h->ws.mask), sc, l, h->Lpad / 64, nullptr, h->cfg.p_max,
                                h->at<int32_t>(h->ws.cand),
                                h->at<int32_t>(h->ws.kept_pos), h->at<int32_t>(h->ws.kept), &sc->n_kept, count_updates,
                                commit_args(h, commit ? kCommitKept : 0), marked);
}

// Dynamic dependencies: the walk runs over the movers only (their conflict mask has the row
// width of the padded mover count) and leaves mkept_pos, n_mkept; the same workgroup then
// assembles and commits B_1 (kept_pos, kept, z, delta, n_kept; beta and delta beta), where the cap
// on |B_1| is applied.
hipError_t launch_filter_movers(strads_lasso *h)
{
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    return launch_filter_kernel(h->stream, h->at<uint64_t>(h->ws.mask), sc, h->L, h->Lpad / 64,
                                h->at<GramShape>(h->ws.dshape), h->cfg.p_max,
                                h->at<int32_t>(h->ws.mcand), h->at<int32_t>(h->ws.mkept_pos),
                                h->at<int32_t>(h->ws.kept), &sc->n_mkept, false, commit_args(h, kCommitDynamic), false);
}

// The greedy walk alone, on buffers named one by one (no handle): mask holds lpad rows of lpad / 64 words as
// k_mask_from_gram writes them, cand l column ids, kept_pos and kept room for l entries, n_out one int.
hipError_t launch_filter_plain(hipStream_t stream, const uint64_t *mask, int32_t l, int32_t lpad, int32_t p_max,
                               const int32_t *cand, int32_t *kept_pos, int32_t *kept, RoundScalars *sc, int32_t *n_out)
{
    CommitArgs cm;
    memset(&cm, 0, sizeof(cm));
    return launch_filter_kernel(stream, mask, sc, l, lpad / 64, nullptr, p_max, cand, kept_pos, kept, n_out, false, cm, false);
}

// No dependency check (the Shotgun scheduler of Section 5.1): B_1 is the head of the draw.
__global__ __launch_bounds__(256) void k_keep_all(const int32_t *__restrict__ cand, int32_t L, int32_t p_max,
                                                  int32_t *__restrict__ kept_pos, int32_t *__restrict__ kept,
                                                  RoundScalars *__restrict__ sc)
{
    const int32_t k = (p_max > 0 && p_max < L) ? p_max : L;
    for (int32_t i = blockIdx.x * 256 + threadIdx.x; i < k; i += gridDim.x * 256) {
        kept_pos[i] = i;
        kept[i] = cand[i];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sc->n_kept = k;
        sc->updates_total += (unsigned long long)k;
    }
}

hipError_t launch_keep_all(strads_lasso *h)
{
    hipLaunchKernelGGL(k_keep_all, dim3((h->L + 255) / 256), dim3(256), 0, h->stream, h->at<int32_t>(h->ws.cand),
                       h->L, h->cfg.p_max, h->at<int32_t>(h->ws.kept_pos), h->at<int32_t>(h->ws.kept),
                       h->at<RoundScalars>(h->ws.scalars));
    return launch_status(h->stream);
}

hipError_t filter_prepare() { return hipSuccess; }   // static LDS only

} // namespace strads
