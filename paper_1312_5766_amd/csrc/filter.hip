// Step 2 of SAP for the Lasso, second half (Algorithm 1: "choose a set B_1 of <= P coefficients
// from U such that |x_j^T x_k| < rho for all pairs"): walk the candidates in draw order and keep
// one iff it conflicts with nothing kept so far.
//
// The walk is sequential in the kept set, so the work is arranged to keep the serial chain short.
// One workgroup of 1024 threads takes the candidates 64 at a time (a "chunk").  `dead` (one bit
// per candidate, in LDS) marks candidates that conflict with something already kept.
//   * The chunk's 64 conflict rows (words at or right of the chunk's own word) live in registers,
//     spread over the threads.  The mask was written by workgroups all over the chip, so its first
//     read by this workgroup comes from HBM, about a microsecond away, while a chunk is decided in
//     a fraction of that: the rows are therefore fetched kFilterAhead chunks ahead of their use.
//     Only the chunk's 64x64 diagonal block goes to LDS, for wavefront 0.
//   * Wavefront 0 decides the chunk: candidates that are alive and have no conflict with another
//     alive candidate of the chunk are kept at once; only the few with an in-chunk conflict are
//     walked one by one (scalar bit operations on the diagonal block).
//   * All threads then OR the words they hold of the newly kept candidates' rows into `dead` for
//     later chunks.
// Only bits (a, b) with b in a's 128-tile or right of it are read, matching what the Gram
// kernel writes.  Bit-exact: the result depends on the conflict bits only.
#include "strads_internal.h"

namespace strads {

__device__ __forceinline__ uint64_t readlane64(uint64_t v, int l)
{
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}

constexpr int kMaxWords = STRADS_MAX_L_PRIME / 64;   // mask words per row (128)
constexpr int kFilterThreads = 1024;
constexpr int kFilterAhead = 4;                     // chunks whose rows are in flight from memory

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
// kept candidate that does not move).  The 1024 threads walk the candidate positions 1024 at a
// time.  mkept_pos[0..nmk): the walk's result, written by this workgroup before a barrier.
__device__ __forceinline__ void commit_dynamic(const CommitArgs &cm, int32_t p_max, const int32_t *mkept_pos,
                                               int32_t nmk, RoundScalars *__restrict__ sc)
{
    __shared__ uint8_t mkept[STRADS_MAX_L_PRIME];       // 1: a mover at this position passed the filter
    __shared__ uint32_t wtot[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t L = cm.L;
    const int32_t cap = p_max > 0 ? p_max : L;
    for (int32_t a = tid; a < L; a += kFilterThreads) mkept[a] = 0;
    __syncthreads();
    for (int32_t i = tid; i < nmk; i += kFilterThreads) mkept[cm.mpos[mkept_pos[i]]] = 1;
    __syncthreads();
    uint32_t base = 0;
    for (int32_t a0 = 0; a0 < L; a0 += kFilterThreads) {
        const int32_t a = a0 + tid;
        const float d = a < L ? cm.dc[a] : 0.f;
        const bool keep = a < L && (d == 0.f || mkept[a]);
        const uint64_t m = __ballot(keep);
        if (lane == 0) wtot[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) { const uint32_t v = wtot[w]; if (w < wave) before += v; total += v; }
        const int32_t idx = (int32_t)(base + before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull)));
        if (keep && idx < cap) {
            const int32_t j = cm.cand[a];
            cm.kept_pos[idx] = a;
            cm.kept[idx] = j;
            cm.z[idx] = cm.zc[a];
            cm.delta[idx] = d;
            cm.beta[j] = cm.nbc[a];
            cm.dbeta[j] = fabsf(d);
        }
        base += total;
        __syncthreads();
    }
    if (tid == 0) {
        const int32_t nk = (int32_t)base < cap ? (int32_t)base : cap;
        sc->n_kept = nk;
        sc->updates_total += (unsigned long long)nk;
    }
}

// IPT = words of a chunk's 64 rows handled per thread = ceil(64 * W / 1024): 1, 2, 4 or 8.
template <int kRowWordsPerThread>
__global__ __launch_bounds__(kFilterThreads) void k_filter(const uint64_t *__restrict__ mask, int32_t L, int32_t W,
                                                           const GramShape *__restrict__ gdev,
                                                           int32_t p_max, const int32_t *__restrict__ cand,
                                                           int32_t *kept_pos, int32_t *__restrict__ kept,
                                                           RoundScalars *__restrict__ sc, int32_t *__restrict__ n_out,
                                                           int count_updates, CommitArgs cm)
{
    if (gdev) { L = gdev->L; W = gdev->Lpad / 64; }   // dynamic dependencies: the movers, counted on the device
    if (L <= 0) {                                      // nothing moves this round
        if (threadIdx.x == 0) *n_out = 0;
        if (cm.on == kCommitDynamic) commit_dynamic(cm, p_max, kept_pos, 0, sc);
        return;
    }
    __shared__ uint64_t diag[2][64];              // word c of chunk c's rows, chunks alternating
    __shared__ uint64_t dead[kMaxWords];
    __shared__ uint64_t keptw_s;
    __shared__ int32_t nk_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t cap = (p_max > 0 && cm.on != kCommitDynamic) ? p_max : L;   // the movers' walk has no cap: commit_dynamic applies it
    const int32_t chunks = (L + 63) / 64;
    const int32_t items = 64 * W;                 // words of one chunk's rows

    for (int i = tid; i < W; i += kFilterThreads) dead[i] = 0;
    if (tid == 0) nk_s = 0;

    // this thread's share of a chunk's 64 x W words: the (row, word) of item tid + q*1024 does not
    // depend on the chunk, so the divisions are done once
    int16_t irow[kRowWordsPerThread], iword[kRowWordsPerThread];
#pragma unroll
    for (int q = 0; q < kRowWordsPerThread; ++q) {
        const int32_t it = tid + q * kFilterThreads;
        const int32_t rw = it / W;
        irow[q] = (int16_t)rw;
        iword[q] = it < items ? (int16_t)(it - rw * W) : (int16_t)-1;     // -1: no such item
    }
    // register sets of the chunks in flight: chunk c waits in set c % kFilterAhead
    uint64_t pre[kFilterAhead][kRowWordsPerThread];
    auto fetch = [&](int32_t c, uint64_t (&dst)[kRowWordsPerThread]) {
#pragma unroll
        for (int q = 0; q < kRowWordsPerThread; ++q) {
            const int32_t a = c * 64 + irow[q], w = iword[q];
            dst[q] = (c < chunks && w >= c && a < L) ? mask[(int64_t)a * W + w] : 0ull;
        }
    };
    // the diagonal block of chunk c: every row of the chunk has exactly one holder of its word c
    auto put_diag = [&](int32_t c, const uint64_t (&src)[kRowWordsPerThread]) {
#pragma unroll
        for (int q = 0; q < kRowWordsPerThread; ++q)
            if (iword[q] == c) diag[c & 1][irow[q]] = src[q];
    };
#pragma unroll
    for (int d = 0; d < kFilterAhead; ++d) fetch(d, pre[d]);
    put_diag(0, pre[0]);
    __syncthreads();

    // one chunk; `mine` is the register set that holds chunk c, `next` holds chunk c+1.
    // Returns true when the cap on the kept set has been reached.
    auto step = [&](int32_t c, uint64_t (&mine)[kRowWordsPerThread], const uint64_t (&next)[kRowWordsPerThread]) -> bool {
        if (wave == 0) {
            const int32_t nk0 = nk_s;
            int32_t nk = nk0;
            const uint64_t cur = dead[c];
            const int32_t nvalid = L - c * 64;
            uint64_t alive = ~cur & (nvalid >= 64 ? ~0ull : ((1ull << nvalid) - 1ull));
            const uint64_t dg = diag[c & 1][lane];
            uint64_t keptw = 0;
            if (nk < cap) {
                // lanes whose row meets another alive candidate of this chunk need the serial walk
                const uint64_t tangled = __ballot((dg & alive) != 0) & alive;
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
                        todo &= ~readlane64(dg, l);
                    }
                }
            }
            if ((keptw >> lane) & 1ull) {
                const int32_t idx = nk0 + __popcll(keptw & ((1ull << lane) - 1ull));
                kept_pos[idx] = c * 64 + lane;
            }
            if (lane == 0) { keptw_s = keptw; nk_s = nk; }
        }
        __syncthreads();
        const uint64_t keptw = keptw_s;
        const bool full = nk_s >= cap;
        // OR the kept rows into dead[w], w > c
        if (!full && keptw != 0) {
#pragma unroll
            for (int q = 0; q < kRowWordsPerThread; ++q) {
                const int32_t w = iword[q];
                if (w > c && ((keptw >> irow[q]) & 1ull)) {
                    const uint64_t v = mine[q];
                    if (v) atomicOr((unsigned long long *)&dead[w], (unsigned long long)v);
                }
            }
        }
        if (c + 1 < chunks) put_diag(c + 1, next);
        fetch(c + kFilterAhead, mine);            // chunk c is done with its registers; in flight for the next chunks
        __syncthreads();
        return full;
    };

    for (int32_t c0 = 0; c0 < chunks; c0 += kFilterAhead) {
        bool stop = false;
#pragma unroll
        for (int d = 0; d < kFilterAhead; ++d) {
            if (!stop && c0 + d < chunks) stop = step(c0 + d, pre[d], pre[(d + 1) % kFilterAhead]);
        }
        if (stop) break;
    }
    // kept column ids, gathered once at the end (a global load inside the loop above would put
    // a memory round trip on the serial chain of every chunk)
    const int32_t nk = nk_s;
    if (cm.on == kCommitDynamic) {
        if (tid == 0) *n_out = nk;
        commit_dynamic(cm, p_max, kept_pos, nk, sc);
        return;
    }
    if (cm.on == kCommitKept) {
        // eq. (2) and Step 4 for B_1, from the update every candidate was found to make when the Gram was formed
        for (int32_t i = tid; i < nk; i += kFilterThreads) {
            const int32_t a = kept_pos[i], j = cand[a];
            const float d = cm.dc[a];
            kept[i] = j;
            cm.z[i] = cm.zc[a];
            cm.delta[i] = d;
            cm.beta[j] = cm.nbc[a];
            cm.dbeta[j] = fabsf(d);
        }
    } else {
        for (int32_t i = tid; i < nk; i += kFilterThreads) kept[i] = cand[kept_pos[i]];
    }
    if (tid == 0) {
        *n_out = nk;
        if (count_updates) sc->updates_total += (unsigned long long)nk;
    }
}

// Launch for row width W (words); with gdev the kernel takes the actual length and width from
// device memory (they can only be smaller).
static hipError_t launch_filter_kernel(strads_lasso *h, int32_t l, int32_t W, const GramShape *gdev, int32_t p_max,
                                       const int32_t *cand, int32_t *kept_pos, int32_t *kept, int32_t *n_out,
                                       bool count_updates, const CommitArgs &cm)
{
#define STRADS_FILTER(IPT) hipLaunchKernelGGL(k_filter<IPT>, dim3(1), dim3(kFilterThreads), 0, h->stream, h->at<uint64_t>(h->ws.mask), l, W, gdev, p_max, cand, kept_pos, kept, h->at<RoundScalars>(h->ws.scalars), n_out, count_updates ? 1 : 0, cm)
    if (W <= 16) STRADS_FILTER(1);
    else if (W <= 32) STRADS_FILTER(2);
    else if (W <= 64) STRADS_FILTER(4);
    else STRADS_FILTER(8);
#undef STRADS_FILTER
    return hipGetLastError();
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

hipError_t launch_filter(strads_lasso *h, int32_t l, bool count_updates, bool commit)
{
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    return launch_filter_kernel(h, l, h->Lpad / 64, nullptr, h->cfg.p_max, h->at<int32_t>(h->ws.cand),
                                h->at<int32_t>(h->ws.kept_pos), h->at<int32_t>(h->ws.kept), &sc->n_kept, count_updates,
                                commit_args(h, commit ? kCommitKept : 0));
}

// Dynamic dependencies: the walk runs over the movers only (their conflict mask has the row
// width of the padded mover count) and leaves mkept_pos, n_mkept; the same workgroup then
// assembles and commits B_1 (kept_pos, kept, z, delta, n_kept; beta and delta beta), where the cap
// on |B_1| is applied.
hipError_t launch_filter_movers(strads_lasso *h)
{
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    return launch_filter_kernel(h, h->L, h->Lpad / 64, h->at<GramShape>(h->ws.dshape), h->cfg.p_max,
                                h->at<int32_t>(h->ws.mcand), h->at<int32_t>(h->ws.mkept_pos),
                                h->at<int32_t>(h->ws.kept), &sc->n_mkept, false, commit_args(h, kCommitDynamic));
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
    return hipGetLastError();
}

hipError_t filter_prepare() { return hipSuccess; }   // static LDS only

} // namespace strads
