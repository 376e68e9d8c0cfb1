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

constexpr int kGenoCols = 4;   // columns a wavefront processes together

static __device__ __forceinline__ float gwave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
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

// x_j^T r for up to kGenoCols columns by one wavefront; out[c] valid in lane 0.  cols[c] < 0: skip.
static __device__ __forceinline__ void geno_dots(const uint32_t *__restrict__ Xw, int64_t words,
                                                 const float *__restrict__ mean, const float *__restrict__ scale,
                                                 const int64_t (&cols)[kGenoCols], const float *__restrict__ r,
                                                 int lane, float (&out)[kGenoCols])
{
    GenoLut lut[kGenoCols];
    const uint32_t *cp[kGenoCols];
#pragma unroll
    for (int c = 0; c < kGenoCols; ++c) {
        const int64_t j = cols[c] >= 0 ? cols[c] : cols[0];
        lut[c] = geno_lut(mean[j], scale[j]);
        cp[c] = Xw + j * words;
    }
    float acc[kGenoCols] = {0.f, 0.f, 0.f, 0.f};
    for (int64_t w = lane; w < words; w += 64) {
        const float4 *r4 = reinterpret_cast<const float4 *>(r + 16 * w);
        const float4 ra = r4[0], rb = r4[1], rc = r4[2], rd = r4[3];
        const float rv[16] = {ra.x, ra.y, ra.z, ra.w, rb.x, rb.y, rb.z, rb.w, rc.x, rc.y, rc.z, rc.w, rd.x, rd.y, rd.z, rd.w};
#pragma unroll
        for (int c = 0; c < kGenoCols; ++c) {
            const uint32_t word = cp[c][w];
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) s += geno_value(word, e, lut[c]) * rv[e];
            acc[c] += s;
        }
    }
#pragma unroll
    for (int c = 0; c < kGenoCols; ++c) out[c] = gwave_sum(acc[c]);
}

// eq. (2) and Step 4 for the kept set (COMMIT) or the tentative update of every candidate (!COMMIT)
template <bool COMMIT>
__global__ __launch_bounds__(256) void k_geno_dots(const uint32_t *__restrict__ Xw, int64_t words,
                                                   const float *__restrict__ mean, const float *__restrict__ scale,
                                                   const int32_t *__restrict__ list, int32_t n_host,
                                                   const RoundScalars *__restrict__ sc, const float *__restrict__ r,
                                                   float lambda, float *__restrict__ beta, float *__restrict__ dbeta,
                                                   float *__restrict__ z, float *__restrict__ delta,
                                                   float *__restrict__ newbeta)
{
    const int n = COMMIT ? sc->n_kept : n_host;
    const int c0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kGenoCols;
    if (c0 >= n) return;                        // whole wavefront
    int64_t cols[kGenoCols];
#pragma unroll
    for (int c = 0; c < kGenoCols; ++c) cols[c] = c0 + c < n ? (int64_t)list[c0 + c] : -1;
    float s[kGenoCols];
    geno_dots(Xw, words, mean, scale, cols, r, threadIdx.x & 63, s);
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int c = 0; c < kGenoCols; ++c) {
            if (cols[c] < 0) continue;
            const int64_t j = cols[c];
            const float b = beta[j];
            const float nb = soft_threshold_g(s[c] + b, lambda);
            const float d = nb - b;
            z[c0 + c] = s[c];
            delta[c0 + c] = d;
            if (COMMIT) { beta[j] = nb; dbeta[j] = fabsf(d); }
            else newbeta[c0 + c] = nb;
        }
    }
}

// optimality violation over all columns (see k_kkt): persistent wavefronts, four columns each step
__global__ __launch_bounds__(256) void k_geno_kkt(const uint32_t *__restrict__ Xw, int64_t words,
                                                  const float *__restrict__ mean, const float *__restrict__ scale,
                                                  int64_t J, const float *__restrict__ r,
                                                  const float *__restrict__ beta, float lambda,
                                                  float *__restrict__ g_out, RoundScalars *__restrict__ sc)
{
    __shared__ float vm[4];
    float vmax = 0.f;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int64_t j0 = ((int64_t)blockIdx.x * 4 + wave) * kGenoCols; j0 < J; j0 += (int64_t)gridDim.x * 4 * kGenoCols) {
        int64_t cols[kGenoCols];
#pragma unroll
        for (int c = 0; c < kGenoCols; ++c) cols[c] = j0 + c < J ? j0 + c : -1;
        float s[kGenoCols];
        geno_dots(Xw, words, mean, scale, cols, r, lane, s);
        if (lane == 0) {
#pragma unroll
            for (int c = 0; c < kGenoCols; ++c) {
                if (cols[c] < 0) continue;
                const float g = s[c], b = beta[cols[c]];
                if (g_out) g_out[cols[c]] = g;
                float v = b == 0.f ? fmaxf(fabsf(g) - lambda, 0.f) : fabsf(g - copysignf(lambda, b));
                if (!(v == v)) v = __uint_as_float(0x7F800000u);
                vmax = fmaxf(vmax, v);
            }
        }
    }
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

hipError_t launch_dots_geno(strads_lasso *h)
{
    const unsigned grid = (unsigned)((h->L + 4 * kGenoCols - 1) / (4 * kGenoCols));
    hipLaunchKernelGGL(k_geno_dots<true>, dim3(grid), dim3(256), 0, h->stream, geno_words_ptr(h), geno_words(h->cfg.n),
                       h->cfg.col_mean, h->cfg.col_scale, h->at<int32_t>(h->ws.kept), 0,
                       h->at<RoundScalars>(h->ws.scalars), h->at<float>(h->ws.r), h->cfg.lambda,
                       h->at<float>(h->ws.beta), h->at<float>(h->ws.dbeta), h->at<float>(h->ws.z),
                       h->at<float>(h->ws.delta), (float *)nullptr);
    return hipGetLastError();
}

hipError_t launch_dots_cand_geno(strads_lasso *h)
{
    const unsigned grid = (unsigned)((h->L + 4 * kGenoCols - 1) / (4 * kGenoCols));
    hipLaunchKernelGGL(k_geno_dots<false>, dim3(grid), dim3(256), 0, h->stream, geno_words_ptr(h), geno_words(h->cfg.n),
                       h->cfg.col_mean, h->cfg.col_scale, h->at<int32_t>(h->ws.cand), h->L,
                       h->at<RoundScalars>(h->ws.scalars), h->at<float>(h->ws.r), h->cfg.lambda,
                       h->at<float>(h->ws.beta), h->at<float>(h->ws.dbeta), h->at<float>(h->ws.zc),
                       h->at<float>(h->ws.dc), h->at<float>(h->ws.nbc));
    return hipGetLastError();
}

hipError_t launch_kkt_geno(strads_lasso *h, float *g_or_null)
{
    hipError_t e = launch_clear_kkt(h);
    if (e != hipSuccess) return e;
    int64_t g = (h->cfg.j + 4 * kGenoCols - 1) / (4 * kGenoCols);
    if (g > 256 * 8) g = 256 * 8;               // persistent: a few workgroups per compute unit
    hipLaunchKernelGGL(k_geno_kkt, dim3((unsigned)g), dim3(256), 0, h->stream, geno_words_ptr(h), geno_words(h->cfg.n),
                       h->cfg.col_mean, h->cfg.col_scale, h->cfg.j, h->at<float>(h->ws.r), h->at<float>(h->ws.beta),
                       h->cfg.lambda, g_or_null, h->at<RoundScalars>(h->ws.scalars));
    return hipGetLastError();
}

hipError_t launch_residual_geno(strads_lasso *h)
{
    const int64_t words = geno_words(h->cfg.n);
    const int G = residual_groups(16 * words / 4, h->L);    // row blocks here hold 4096 rows, the dense ones 1024
    const dim3 grid((unsigned)((words + 255) / 256), (unsigned)G);
    float *part = h->at<float>(h->ws.rpart);
    hipLaunchKernelGGL(k_geno_residual_partial, grid, dim3(256), 0, h->stream, geno_words_ptr(h), words,
                       h->cfg.col_mean, h->cfg.col_scale, h->Npad, h->at<int32_t>(h->ws.kept),
                       h->at<float>(h->ws.delta), h->at<RoundScalars>(h->ws.scalars), part);
    const hipError_t e = hipGetLastError();
    return e != hipSuccess ? e : launch_residual_apply(h, G);     // stage 2 is shared with the dense path
}

} // namespace strads
