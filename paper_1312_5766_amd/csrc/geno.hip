// The worker side of Algorithm 1 (eq. (2), Step 4, residual update, optimality check) for a packed
// genotype design (STRADS_LAYOUT_GENO2): entries g in {0, 1, 2} stored 2 bits each, 16 rows per
// 32-bit word, with X_ij = fl(fl(g_ij - mean_j) * scale_j).  Every pass over X moves 16 times fewer
// bytes than fp32; the residual r (4 bytes per row) would then dominate, so a wavefront works on four
// columns at a time against one read of r.
//
// r[N .. Npad) is kept at zero and so is every code past row N, so rows up to the padded column
// length can be processed without bounds checks.
#include "strads_internal.h"

namespace strads {

// sum over the wavefront, returned in every lane (butterfly: the same tree in every lane)
static __device__ __forceinline__ float gwave_sum_all(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

struct GenoLut { float v[3]; };

static __device__ __forceinline__ GenoLut geno_lut(float mean, float scale)
{
    GenoLut l;
    l.v[0] = __fmul_rn(__fsub_rn(0.f, mean), scale);
    l.v[1] = __fmul_rn(__fsub_rn(1.f, mean), scale);
    l.v[2] = __fmul_rn(__fsub_rn(2.f, mean), scale);
    return l;
}

static __device__ __forceinline__ float geno_value(uint32_t word, int e, const GenoLut &l)
{
    const uint32_t g = (word >> (2 * e)) & 3u;
    return g == 0u ? l.v[0] : (g == 1u ? l.v[1] : l.v[2]);
}

static __device__ __forceinline__ float soft_threshold_g(float a, float lambda)
{
    const float m = fabsf(a) - lambda;
    return m > 0.f ? copysignf(m, a) : 0.f;
}

// ---------------------------------------------------------------------------------------------
// x_j^T r on packed words.  With g the genotype count,
//     x_j^T r = scale_j * (sum_i g_ij r_i  -  mean_j * sum_i r_i),
// so a column needs one multiply-add per entry on the raw count and no per-entry decode; rows past
// N hold count 0 and add nothing.  (This differs from summing the decoded fl(fl(g - mean) * scale)
// entries by rounding only.)
//
// A lane owns a column.  Work proceeds in slabs of SW words (16 SW rows): a wavefront brings its 64
// columns' slab in with 16-byte loads (SW/4 lanes cover one column's piece), turns it through its
// own piece of LDS, and then every lane walks its column's words while the slab of r is read at
// wave-uniform addresses.  Within a word the four byte lanes of (word >> 2q) & 0x03030303
// are entries q, q+4, q+8, q+12; masking in place instead of shifting leaves the count scaled by
// 4^q, which one exact multiply per column removes at the end.
//   short lists (the kept set, the candidates; all columns of a small design): k_geno_dots.  The four
//     wavefronts of a workgroup share 64 columns and take every fourth slab of 128 rows, combined in
//     wavefront order: a round waits on this kernel, and the row range has to be spread to shorten it.
//   all columns of a large design: k_geno_all, persistent wavefronts, slabs of 512 rows, next slab in flight.
constexpr int kSlabShort = 8, kSlabLong = 32;  // words per slab; LDS rows are padded by one word (odd
                                               // stride: lanes reading one word each hit distinct banks)

// A lane's walk over nw words of its column (in LDS) against the rows at rbase (wave-uniform address):
// a_q accumulates entries q, q+4, q+8, q+12 of every word, scaled by 4^q.
static __device__ __forceinline__ void geno_consume(const uint32_t *__restrict__ src, int nw,
                                                    const float *__restrict__ rbase, float &a0, float &a1,
                                                    float &a2, float &a3)
{
#pragma unroll 4
    for (int w = 0; w < nw; ++w) {
        const uint32_t code = src[w];
        const float *rw = rbase + 16 * w;
        uint32_t t0 = code & 0x03030303u, t1 = code & 0x0C0C0C0Cu;
        uint32_t t2 = code & 0x30303030u, t3 = code & 0xC0C0C0C0u;
        // keep the four masked words as they are, so that each entry is one byte-to-float conversion
        asm volatile("" : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3));
#define STRADS_GENO_ACC(A, T, Q)                                                                    \
        A = __builtin_fmaf((float)((T) & 0xFFu), rw[Q], A);                                         \
        A = __builtin_fmaf((float)(((T) >> 8) & 0xFFu), rw[(Q) + 4], A);                            \
        A = __builtin_fmaf((float)(((T) >> 16) & 0xFFu), rw[(Q) + 8], A);                           \
        A = __builtin_fmaf((float)((T) >> 24), rw[(Q) + 12], A)
        STRADS_GENO_ACC(a0, t0, 0);
        STRADS_GENO_ACC(a1, t1, 1);
        STRADS_GENO_ACC(a2, t2, 2);
        STRADS_GENO_ACC(a3, t3, 3);
#undef STRADS_GENO_ACC
    }
}

struct GenoSums { float gr, rs; };             // sum g r, sum r over the slabs a wavefront walked

static __device__ __forceinline__ GenoSums geno_column_sums(const uint32_t *__restrict__ Xw, int64_t words,
                                                            int64_t col, const float *__restrict__ r,
                                                            uint32_t *__restrict__ lds_wave)
{
    constexpr int PH = 4;                      // wavefronts sharing a column
    constexpr int SW = kSlabShort, STRIDE = SW + 1;
    constexpr int CH = SW / 4;                 // 16-byte pieces of a column's slab = lanes per column = passes
    const int lane = threadIdx.x & 63;
    const int phase = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int nslab = (int)((words + SW - 1) / SW);
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f, rs = 0.f;
    for (int sl = phase; sl < nslab; sl += PH) {
        const int64_t w0 = (int64_t)sl * SW;
        // stage: pass i brings 16 bytes of each of 64/CH columns
        uint4 v[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int slot = (64 / CH) * i + lane / CH;
            const int64_t cj = __shfl(col, slot);
            const int64_t w = w0 + 4 * (lane % CH);
            v[i] = w < words ? *reinterpret_cast<const uint4 *>(Xw + cj * words + w) : make_uint4(0u, 0u, 0u, 0u);
        }
        // sum of r over the slab, in a fixed order
        float rpart = 0.f;
#pragma unroll
        for (int k = 0; k < SW / 4; ++k) {
            const int64_t i = 16 * w0 + lane + 64 * k;
            rpart += i < 16 * words ? r[i] : 0.f;
        }
        rs += gwave_sum_all(rpart);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            uint32_t *dst = lds_wave + ((64 / CH) * i + lane / CH) * STRIDE + 4 * (lane % CH);
            dst[0] = v[i].x; dst[1] = v[i].y; dst[2] = v[i].z; dst[3] = v[i].w;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int nw = words - w0 < SW ? (int)(words - w0) : SW;
        geno_consume(lds_wave + lane * STRIDE, nw, r + 16 * w0, a0, a1, a2, a3);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();                    // the slab is consumed before the next one lands
    }
    GenoSums out;
    out.gr = (a0 + 0.25f * a1) + (0.0625f * a2 + 0.015625f * a3);
    out.rs = rs;
    return out;
}

enum { kGenoCommit = 0, kGenoTentative = 1, kGenoAll = 2 };

// MODE kGenoCommit:    eq. (2) and Step 4 for the kept set (count on the device)
// MODE kGenoTentative: dot product and tentative update of every candidate
// MODE kGenoAll:       x_j^T r and the optimality violation of all J columns (see k_kkt), small J
template <int MODE>
__global__ __launch_bounds__(256) void k_geno_dots(const uint32_t *__restrict__ Xw, int64_t words,
                                                   const float *__restrict__ mean, const float *__restrict__ scale,
                                                   const int32_t *__restrict__ list, int64_t n_host,
                                                   RoundScalars *__restrict__ sc, const float *__restrict__ r,
                                                   float lambda, float step, float *__restrict__ beta,
                                                   float *__restrict__ dbeta, float *__restrict__ z,
                                                   float *__restrict__ delta, float *__restrict__ newbeta)
{
    __shared__ uint32_t slab[4][64 * (kSlabShort + 1)];
    __shared__ GenoSums comb[4][64];
    const int64_t n = MODE == kGenoCommit ? (int64_t)sc->n_kept : n_host;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t c = (int64_t)blockIdx.x * 64 + lane;
    if ((int64_t)blockIdx.x * 64 >= n) return;              // whole workgroup
    const bool live = c < n;
    // lanes past the end walk the workgroup's first column and drop the result
    const int64_t cc = live ? c : (int64_t)blockIdx.x * 64;
    const int64_t j = MODE == kGenoAll ? cc : (int64_t)list[cc];
    GenoSums s = geno_column_sums(Xw, words, j, r, slab[wave]);
    comb[wave][lane] = s;
    __syncthreads();
    if (wave != 0) return;
    s.gr = (comb[0][lane].gr + comb[1][lane].gr) + (comb[2][lane].gr + comb[3][lane].gr);
    s.rs = (comb[0][lane].rs + comb[1][lane].rs) + (comb[2][lane].rs + comb[3][lane].rs);
    const float dot = scale[j] * (s.gr - mean[j] * s.rs);
    if (MODE == kGenoAll) {
        float v = 0.f;
        if (live) {
            const float b = beta[j];
            if (z) z[j] = dot;
            v = b == 0.f ? fmaxf(fabsf(dot) - lambda, 0.f) : fabsf(dot - copysignf(lambda, b));
            if (!(v == v)) v = __uint_as_float(0x7F800000u);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_down(v, off));
        if (lane == 0) atomicMax(&sc->kkt_max_bits, __float_as_uint(v));
    } else if (live) {
        const float b = beta[j];
        const float nb = soft_threshold_g(dot * step + b, lambda * step);     // step = 1: eq. (2) as printed
        const float d = nb - b;
        z[c] = dot;
        delta[c] = d;
        if (MODE == kGenoCommit) { beta[j] = nb; dbeta[j] = fabsf(d); }
        else newbeta[c] = nb;
    }
}

// The pass over all J columns (x_j^T r and the optimality violation, see k_kkt) for large J:
// persistent wavefronts take 64 consecutive columns at a time and walk their slabs of 512 rows as in
// geno_column_sums, but keep the next slab's 16-byte loads in flight while the current one is
// turned through LDS and consumed, so that the memory latency is hidden behind the arithmetic.  The
// sum of r is taken once per wavefront.
__global__ __launch_bounds__(256) void k_geno_all(const uint32_t *__restrict__ Xw, int64_t words,
                                                  const float *__restrict__ mean, const float *__restrict__ scale,
                                                  int64_t J, RoundScalars *__restrict__ sc,
                                                  const float *__restrict__ r, float lambda,
                                                  const float *__restrict__ beta, float *__restrict__ g_out)
{
    constexpr int SW = kSlabLong, STRIDE = SW + 1, CH = SW / 4;
    __shared__ uint32_t slab[4][64 * STRIDE];
    __shared__ float vm[4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t *lds_wave = slab[wave];
    const int nslab = (int)((words + SW - 1) / SW);
    const int64_t ngroups = (J + 63) / 64;
    const int64_t nwaves = (int64_t)gridDim.x * 4;

    float rpart = 0.f;                          // sum of r, fixed order
    for (int64_t i = lane; i < 16 * words; i += 64) rpart += r[i];
    const float rs = gwave_sum_all(rpart);

    // the 16-byte pieces of a slab this lane brings in: pass i covers columns 8 i .. 8 i + 7 of the group
    auto fetch = [&](int64_t g, int sl, uint4 (&v)[CH]) {
        const int64_t w = (int64_t)sl * SW + 4 * (lane % CH);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int64_t j = g * 64 + (64 / CH) * i + lane / CH;
            j = j < J ? j : J - 1;              // the last group may be short: its extra lanes repeat a column
            v[i] = w < words ? *reinterpret_cast<const uint4 *>(Xw + j * words + w) : make_uint4(0u, 0u, 0u, 0u);
        }
    };

    float vmax = 0.f;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    uint4 cur[CH], nxt[CH];
    int64_t g = (int64_t)blockIdx.x * 4 + wave;
    int sl = 0;
    if (g < ngroups) fetch(g, 0, cur);
    while (g < ngroups) {
        int64_t g2 = g;
        int sl2 = sl + 1;
        if (sl2 == nslab) { sl2 = 0; g2 = g + nwaves; }
        if (g2 < ngroups) fetch(g2, sl2, nxt);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            uint32_t *dst = lds_wave + ((64 / CH) * i + lane / CH) * STRIDE + 4 * (lane % CH);
            dst[0] = cur[i].x; dst[1] = cur[i].y; dst[2] = cur[i].z; dst[3] = cur[i].w;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int64_t w0 = (int64_t)sl * SW;
        const int nw = words - w0 < SW ? (int)(words - w0) : SW;
        geno_consume(lds_wave + lane * STRIDE, nw, r + 16 * w0, a0, a1, a2, a3);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();        // the slab is consumed before the next one lands
        if (sl == nslab - 1) {                  // column finished
            const int64_t j = g * 64 + lane;
            if (j < J) {
                const float gr = (a0 + 0.25f * a1) + (0.0625f * a2 + 0.015625f * a3);
                const float dot = scale[j] * (gr - mean[j] * rs);
                const float b = beta[j];
                if (g_out) g_out[j] = dot;
                float v = b == 0.f ? fmaxf(fabsf(dot) - lambda, 0.f) : fabsf(dot - copysignf(lambda, b));
                if (!(v == v)) v = __uint_as_float(0x7F800000u);
                vmax = fmaxf(vmax, v);
            }
            a0 = a1 = a2 = a3 = 0.f;
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) cur[i] = nxt[i];
        g = g2;
        sl = sl2;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) vmax = fmaxf(vmax, __shfl_down(vmax, off));
    if (lane == 0) vm[wave] = vmax;
    __syncthreads();
    if (threadIdx.x == 0)
        atomicMax(&sc->kkt_max_bits, __float_as_uint(fmaxf(fmaxf(vm[0], vm[1]), fmaxf(vm[2], vm[3]))));
}

// Residual update, stage 1 (stage 2 is k_residual_apply of the dense path): grid = (blocks of 256
// words = 4096 rows, G column groups).  A thread owns one word's 16 rows; group g sums its movers
// (delta != 0) in list order -> part[g][rows].
__global__ __launch_bounds__(256) void k_geno_residual_partial(const uint32_t *__restrict__ Xw, int64_t words,
                                                               const float *__restrict__ mean,
                                                               const float *__restrict__ scale, int64_t Npad,
                                                               const int32_t *__restrict__ kept,
                                                               const float *__restrict__ delta,
                                                               RoundScalars *__restrict__ sc, float *__restrict__ part)
{
    __shared__ int32_t mcol[256];
    __shared__ float mlut[256][3];              // the column's three values times its change
    __shared__ uint32_t wcnt[4];
    const int k = sc->n_kept;
    const int G = gridDim.y, g = blockIdx.y;
    const int c0 = (int)((int64_t)k * g / G), c1 = (int)((int64_t)k * (g + 1) / G);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t w = (int64_t)blockIdx.x * 256 + tid;
    float acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    for (int cb = c0; cb < c1; cb += 256) {
        const int c = cb + tid;
        const float d = c < c1 ? delta[c] : 0.f;
        const bool mv = d != 0.f;
        const uint64_t m = __ballot(mv);
        if (lane == 0) wcnt[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = 0, tot = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) { const uint32_t v = wcnt[q]; if (q < wave) before += v; tot += v; }
        if (mv) {
            const uint32_t p = before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            const int32_t j = kept[c];
            const GenoLut l = geno_lut(mean[j], scale[j]);
            mcol[p] = j;
            mlut[p][0] = l.v[0] * d; mlut[p][1] = l.v[1] * d; mlut[p][2] = l.v[2] * d;
        }
        __syncthreads();
        if (w < words) {
            for (uint32_t q = 0; q < tot; ++q) {
                const uint32_t word = Xw[(int64_t)mcol[q] * words + w];
                GenoLut l;
                l.v[0] = mlut[q][0]; l.v[1] = mlut[q][1]; l.v[2] = mlut[q][2];
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[e] += geno_value(word, e, l);
            }
        }
        __syncthreads();
    }
    if (w < words) {
        float4 *dst = reinterpret_cast<float4 *>(part + (int64_t)g * Npad + 16 * w);
        dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        dst[2] = make_float4(acc[8], acc[9], acc[10], acc[11]);
        dst[3] = make_float4(acc[12], acc[13], acc[14], acc[15]);
    }
    if (blockIdx.x == 0 && g == 0) {            // round summary, as in the dense path
        uint32_t nm = 0;
        float mx = 0.f;
        for (int c = tid; c < k; c += 256) { const float d = delta[c]; nm += d != 0.f; mx = fmaxf(mx, fabsf(d)); }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) { nm += __shfl_down(nm, off); mx = fmaxf(mx, __shfl_down(mx, off)); }
        __shared__ uint32_t snm[4];
        __shared__ float smx[4];
        if (lane == 0) { snm[wave] = nm; smx[wave] = mx; }
        __syncthreads();
        if (tid == 0) {
            sc->n_moved = (int32_t)(snm[0] + snm[1] + snm[2] + snm[3]);
            sc->max_abs_delta = fmaxf(fmaxf(smx[0], smx[1]), fmaxf(smx[2], smx[3]));
        }
    }
}

// ---------------------------------------------------------------------------------------------
static inline const uint32_t *geno_words_ptr(const strads_lasso *h) { return reinterpret_cast<const uint32_t *>(h->cfg.x); }

// the persistent pass needs enough columns to fill the chip (64 per wavefront)
static inline bool geno_wide(int64_t ncols) { return ncols >= 256 * 256; }

#define STRADS_GENO_DOTS(MODE, LIST, NHOST, Z, DELTA, NB)                                                          \
    do {                                                                                                           \
        const int64_t ncols_ = (NHOST);                                                                            \
        hipLaunchKernelGGL((k_geno_dots<MODE>), dim3((unsigned)((ncols_ + 63) / 64)), dim3(256), 0, h->stream,     \
                           geno_words_ptr(h), geno_words(h->cfg.n), h->cfg.col_mean, h->cfg.col_scale, LIST,       \
                           ncols_, h->at<RoundScalars>(h->ws.scalars), dots_vector(h), h->cfg.lambda,              \
                           h->step_scale, h->at<float>(h->ws.beta), h->at<float>(h->ws.dbeta), Z, DELTA, NB);      \
    } while (0)

hipError_t launch_dots_geno(strads_lasso *h)
{
    // the grid covers all L candidates; workgroups past the kept count (known on the device) leave at once
    STRADS_GENO_DOTS(kGenoCommit, h->at<int32_t>(h->ws.kept), (int64_t)h->L, h->at<float>(h->ws.z),
                     h->at<float>(h->ws.delta), (float *)nullptr);
    return launch_status(h->stream);
}

hipError_t launch_dots_cand_geno(strads_lasso *h)
{
    STRADS_GENO_DOTS(kGenoTentative, h->at<int32_t>(h->ws.cand), (int64_t)h->L, h->at<float>(h->ws.zc),
                     h->at<float>(h->ws.dc), h->at<float>(h->ws.nbc));
    return launch_status(h->stream);
}

hipError_t launch_kkt_geno(strads_lasso *h, float *g_or_null)
{
    hipError_t e = launch_clear_kkt(h);
    if (e != hipSuccess) return e;
    if (geno_wide(h->cfg.j)) {
        // persistent: four workgroups per compute unit (LDS allows no more), fewer if the columns run out
        int64_t g = (h->cfg.j + 255) / 256;
        if (g > 256 * 4) g = 256 * 4;
        hipLaunchKernelGGL(k_geno_all, dim3((unsigned)g), dim3(256), 0, h->stream, geno_words_ptr(h),
                           geno_words(h->cfg.n), h->cfg.col_mean, h->cfg.col_scale, h->cfg.j,
                           h->at<RoundScalars>(h->ws.scalars), dots_vector(h), h->cfg.lambda,
                           h->at<float>(h->ws.beta), g_or_null);
        return launch_status(h->stream);
    }
    STRADS_GENO_DOTS(kGenoAll, (const int32_t *)nullptr, h->cfg.j, g_or_null, (float *)nullptr, (float *)nullptr);
    return launch_status(h->stream);
}
#undef STRADS_GENO_DOTS

hipError_t launch_residual_geno(strads_lasso *h, bool want_next_keys, bool *next_keys_done)
{
    const int64_t words = geno_words(h->cfg.n);
    const int G = residual_groups(16 * words / 4, h->L);    // row blocks here hold 4096 rows, the dense ones 1024
    const dim3 grid((unsigned)((words + 255) / 256), (unsigned)G);
    float *part = h->at<float>(h->ws.rpart);
    hipLaunchKernelGGL(k_geno_residual_partial, grid, dim3(256), 0, h->stream, geno_words_ptr(h), words,
                       h->cfg.col_mean, h->cfg.col_scale, h->Npad, h->at<int32_t>(h->ws.kept),
                       h->at<float>(h->ws.delta), h->at<RoundScalars>(h->ws.scalars), part);
    const hipError_t e = hipGetLastError();
    return e != hipSuccess ? e : launch_residual_apply(h, G, want_next_keys, next_keys_done);     // stage 2 is shared with the dense path
}

} // namespace strads
