// The round for a sparse design in CSC form (column j = rows row_idx[col_ptr[j] .. col_ptr[j+1]),
// increasing, with values val[...]).  Same steps as the dense path (Algorithm 1, eq. (2), Step 2's
// d(x_a, x_b) = |x_a^T x_b|), different kernels:
//
//   candidate Gram   A dense MFMA Gram of gathered sparse columns would multiply zeros.  Instead an
//                    inverted index of the candidate set is built per round (row -> list of
//                    (candidate, value)); candidate a then walks its own rows and, for every other
//                    candidate met in a row, adds the product into an LDS row G[a][*].  The index is
//                    one kernel: every row owns a bucket of fixed capacity (a few times the expected
//                    load), an entry takes the next free slot of its row's bucket with one atomic, and
//                    the few entries that find their bucket full go to one overflow list that every
//                    reader scans too; no counting pass, no scan over the rows, no second pass over
//                    the columns.
//   residual update  r -= sum_j x_j * change_j scatters into rows that several columns may share.
//
// Both accumulate through integer atomics on a 2^-40 fixed-point image of each product (the fp64
// product of two floats is exact; it is rounded once to the grid).  Integer addition is associative,
// so the sums do not depend on the order in which atomics land: results are bit-reproducible, and
// the rounding error (<= 2^-41 per term) is far below fp32 accumulation error.
//
//   dots / KKT       one wavefront per column: 8 bytes per nonzero streamed, r gathered from L2.
#include "strads_internal.h"
#include "keys.h"

namespace strads {

constexpr double kFixScale = 1099511627776.0;          // 2^40
constexpr double kFixInv = 1.0 / 1099511627776.0;
constexpr double kFixTermLimit = 4194304.0;            // 2^22; a residual update of k columns accepts |value * change| < 2^22 / k

__device__ __forceinline__ long long fix40(float a, float b)
{
    return __double2ll_rn((double)a * (double)b * kFixScale);
}

struct CscEntry { int32_t cand; float val; };
struct CscOverflow { int32_t row, cand; float val; };

struct CscScratch {
    uint32_t *cnt;          // [N]   entries that asked for a slot of the row's bucket (zeroed again by the round's last kernel)
    uint32_t *ovf_cnt;      // [1]   entries in the overflow list (likewise)
    CscEntry *bucket;       // [N * cap]  row i owns bucket[i * cap .. +cap)
    CscOverflow *ovf;       // [L * max_col_nnz]  entries whose bucket was full
    long long *racc;        // [N]   fixed-point residual accumulator (returns to zero after apply)
    int32_t cap;            // bucket capacity
};

// Bucket capacity: four times the expected number of candidate entries per row plus 8, rounded up to a
// power of two, between 8 and 64 (N = 10^5, 4000 candidates of 100 nonzeros: load 4, capacity 32, a bucket
// is two cache lines; a row that gets more sends the rest to the overflow list).
static int32_t csc_bucket_cap(int64_t n, int32_t l, int32_t max_col_nnz)
{
    const double load = (double)l * (double)(max_col_nnz > 0 ? max_col_nnz : 1) / (double)(n > 0 ? n : 1);
    int32_t cap = 8;
    while (cap < 64 && (double)cap < 4.0 * load + 8.0) cap *= 2;
    return cap;
}

static size_t up256(size_t v) { return (v + 255) / 256 * 256; }

static CscScratch csc_carve(const strads_lasso *h)
{
    char *p = h->base + h->ws.csc_scratch;
    const size_t n = (size_t)h->cfg.n;
    CscScratch s;
    s.cap = csc_bucket_cap(h->cfg.n, h->L, h->cfg.max_col_nnz);
    s.cnt = (uint32_t *)p;               p += up256(n * 4);
    s.ovf_cnt = (uint32_t *)p;           p += 256;
    s.racc = (long long *)p;             p += up256(n * 8);
    s.bucket = (CscEntry *)p;            p += up256(n * (size_t)s.cap * sizeof(CscEntry));
    s.ovf = (CscOverflow *)p;
    return s;
}

size_t csc_scratch_bytes(int64_t n, int32_t l, int32_t max_col_nnz)
{
    const size_t cap = (size_t)csc_bucket_cap(n, l, max_col_nnz);
    return up256((size_t)n * 4) + 256 + up256((size_t)n * 8) + up256((size_t)n * cap * sizeof(CscEntry)) +
           up256((size_t)l * (size_t)(max_col_nnz > 0 ? max_col_nnz : 1) * sizeof(CscOverflow));
}

__global__ __launch_bounds__(256) void k_csc_check(const int64_t *__restrict__ col_ptr, int64_t J, int32_t max_col_nnz,
                                                   uint32_t *__restrict__ bad)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < J; j += stride) {
        const int64_t d = col_ptr[j + 1] - col_ptr[j];
        if (d < 0 || d > max_col_nnz || (j == 0 && col_ptr[0] != 0)) atomicOr(bad, 1u);
    }
}

__global__ __launch_bounds__(256) void k_csc_zero(uint32_t *__restrict__ cnt, long long *__restrict__ racc, int64_t N,
                                                  uint32_t *__restrict__ bad, uint32_t *__restrict__ ovf_cnt)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += stride) { cnt[i] = 0u; racc[i] = 0; }
    if (blockIdx.x == 0 && threadIdx.x == 0) { *bad = 0u; *ovf_cnt = 0u; }
}

// ---------------------------------------------------------------------------------------------
// inverted index of the candidate set
// ---------------------------------------------------------------------------------------------
// n_dev != NULL (dynamic dependencies): the list is the movers, counted on the device; wavefronts
// past the count have nothing to do.
//
// One wavefront per candidate a: every nonzero (row, value) of its column takes the next slot of the
// row's bucket (cnt[row] counts the requests, so it may pass the capacity); past the capacity the entry
// goes to the overflow list.  The order of the entries in a bucket depends on which atomic lands first;
// nothing downstream depends on it (the products are summed in fixed point).
__global__ __launch_bounds__(256) void k_csc_build(const int32_t *__restrict__ cand, const GramShape *__restrict__ n_dev,
                                                   int32_t L, const int64_t *__restrict__ col_ptr,
                                                   const int32_t *__restrict__ row_idx, const float *__restrict__ val,
                                                   uint32_t *__restrict__ cnt, CscEntry *__restrict__ bucket, int32_t cap,
                                                   uint32_t *__restrict__ ovf_cnt, CscOverflow *__restrict__ ovf)
{
    if (n_dev) L = n_dev->L;
    const int32_t a = (int32_t)blockIdx.x * 4 + (int32_t)(threadIdx.x >> 6);
    if (a >= L) return;
    const int32_t j = cand[a];
    const int64_t p0 = col_ptr[j], p1 = col_ptr[j + 1];
    for (int64_t p = p0 + (threadIdx.x & 63); p < p1; p += 64) {
        const int32_t row = row_idx[p];
        const float v = val[p];
        const uint32_t slot = atomicAdd(&cnt[row], 1u);
        if (slot < (uint32_t)cap) {
            CscEntry e;
            e.cand = a;
            e.val = v;
            bucket[(int64_t)row * cap + slot] = e;
        } else {
            const uint32_t o = atomicAdd(ovf_cnt, 1u);
            CscOverflow e;
            e.row = row;
            e.cand = a;
            e.val = v;
            ovf[o] = e;
        }
    }
}

// G[a][*] for candidate a = blockIdx.x, conflict bits for the words at or right of a's 128-tile
__global__ __launch_bounds__(256) void k_csc_gram(const int32_t *__restrict__ cand, const GramShape *__restrict__ n_dev,
                                                  const int64_t *__restrict__ col_ptr,
                                                  const int32_t *__restrict__ row_idx, const float *__restrict__ val,
                                                  const uint32_t *__restrict__ cnt, const CscEntry *__restrict__ bucket,
                                                  int32_t cap, const uint32_t *__restrict__ ovf_cnt,
                                                  const CscOverflow *__restrict__ ovf, int32_t L, int32_t Lpad,
                                                  float rho, uint64_t *__restrict__ mask, float *__restrict__ gram,
                                                  int32_t *__restrict__ near_pairs)
{
    extern __shared__ long long acc[];            // [Lpad]
    if (n_dev) L = n_dev->L;                      // the movers only; rows past the count are never read
    const int32_t a = blockIdx.x;
    if (a >= L && n_dev) return;
    const int tid = threadIdx.x;
    const int32_t first = (a / kGramTile) * kGramTile;
    for (int32_t b = tid; b < Lpad; b += 256) acc[b] = 0;
    __syncthreads();
    if (a < L) {
        const int32_t j = cand[a];
        const int64_t p0 = col_ptr[j], p1 = col_ptr[j + 1];
        const uint32_t n_ovf = *ovf_cnt;
        for (int64_t p = p0 + tid; p < p1; p += 256) {
            const int32_t row = row_idx[p];
            const float v = val[p];
            const uint32_t asked = cnt[row];
            const uint32_t m = asked < (uint32_t)cap ? asked : (uint32_t)cap;
            const CscEntry *b = bucket + (int64_t)row * cap;
            for (uint32_t q = 0; q < m; ++q) {
                const CscEntry en = b[q];
                if (en.cand >= first || gram)
                    atomicAdd((unsigned long long *)&acc[en.cand], (unsigned long long)fix40(v, en.val));
            }
            if (asked > (uint32_t)cap) {          // the rest of this row's entries are somewhere in the overflow list
                for (uint32_t q = 0; q < n_ovf; ++q) {
                    const CscOverflow en = ovf[q];
                    if (en.row == row && (en.cand >= first || gram))
                        atomicAdd((unsigned long long *)&acc[en.cand], (unsigned long long)fix40(v, en.val));
                }
            }
        }
    }
    __syncthreads();
    int32_t near = 0;
    for (int32_t b0 = (gram ? 0 : first); b0 < Lpad; b0 += 256) {
        const int32_t b = b0 + tid;
        if (b >= Lpad) break;                     // whole wavefronts: Lpad is a multiple of 64
        const float g = (float)((double)acc[b] * kFixInv);
        const bool live = a < L && b < L && a != b;
        const float ag = fabsf(g);
        const uint64_t w = __ballot(live && !(ag < rho));
        if (b >= first && (tid & 63) == 0) mask[(int64_t)a * (Lpad / 64) + (b >> 6)] = w;
        near += (live && b > a && fabsf(ag - rho) <= 1e-6f) ? 1 : 0;
        if (gram) gram[(int64_t)a * Lpad + b] = g;
    }
    if (near) atomicAdd(near_pairs, near);
}

// ---------------------------------------------------------------------------------------------
// eq. (2) for the kept set: one wavefront per column
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum_f(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
    return v;
}

__device__ __forceinline__ float sparse_dot(const float *__restrict__ val, const int32_t *__restrict__ row_idx,
                                            int64_t p0, int64_t p1, const float *__restrict__ r, int lane)
{
    float s = 0.f;
    for (int64_t p = p0 + lane; p < p1; p += 64) s += val[p] * r[row_idx[p]];
    return wave_sum_f(s);
}

__global__ __launch_bounds__(256) void k_csc_dots_update(const float *__restrict__ val,
                                                         const int32_t *__restrict__ row_idx,
                                                         const int64_t *__restrict__ col_ptr,
                                                         const int32_t *__restrict__ kept,
                                                         const RoundScalars *__restrict__ sc, const float *__restrict__ r,
                                                         float lambda, float step, float *__restrict__ beta,
                                                         float *__restrict__ dbeta, float *__restrict__ z,
                                                         float *__restrict__ delta)
{
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= sc->n_kept) return;
    const int32_t j = kept[c];
    const float s = sparse_dot(val, row_idx, col_ptr[j], col_ptr[j + 1], r, threadIdx.x & 63);
    if ((threadIdx.x & 63) == 0) {
        const float b = beta[j];
        const float a = s * step + b;               // step = 1: eq. (2) as printed
        const float m = fabsf(a) - lambda * step;
        const float nb = m > 0.f ? copysignf(m, a) : 0.f;
        const float d = nb - b;
        z[c] = s;
        delta[c] = d;
        beta[j] = nb;
        dbeta[j] = fabsf(d);
    }
}

// Dynamic dependencies: x_j^T r and the tentative update of every candidate (nothing is committed).
__global__ __launch_bounds__(256) void k_csc_dots_cand(const float *__restrict__ val,
                                                       const int32_t *__restrict__ row_idx,
                                                       const int64_t *__restrict__ col_ptr,
                                                       const int32_t *__restrict__ cand, int32_t L,
                                                       const float *__restrict__ r, float lambda, float step,
                                                       const float *__restrict__ beta, float *__restrict__ zc,
                                                       float *__restrict__ dc, float *__restrict__ nbc)
{
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= L) return;
    const int32_t j = cand[c];
    const float s = sparse_dot(val, row_idx, col_ptr[j], col_ptr[j + 1], r, threadIdx.x & 63);
    if ((threadIdx.x & 63) == 0) {
        const float b = beta[j];
        const float a = s * step + b;
        const float m = fabsf(a) - lambda * step;
        const float nb = m > 0.f ? copysignf(m, a) : 0.f;
        zc[c] = s;
        nbc[c] = nb;
        dc[c] = nb - b;
    }
}

__global__ __launch_bounds__(256) void k_csc_residual_acc(const float *__restrict__ val,
                                                          const int32_t *__restrict__ row_idx,
                                                          const int64_t *__restrict__ col_ptr,
                                                          const int32_t *__restrict__ kept,
                                                          const float *__restrict__ delta, RoundScalars *__restrict__ sc,
                                                          long long *__restrict__ racc)
{
    const int k = sc->n_kept;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (blockIdx.x == 0) {                        // round summary, as in the dense path
        __shared__ uint32_t snm[4];
        __shared__ float smx[4];
        uint32_t nm = 0;
        float mx = 0.f;
        for (int q = threadIdx.x; q < k; q += 256) { const float d = delta[q]; nm += d != 0.f; mx = fmaxf(mx, fabsf(d)); }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) { nm += __shfl_down(nm, off); mx = fmaxf(mx, __shfl_down(mx, off)); }
        if ((threadIdx.x & 63) == 0) { snm[threadIdx.x >> 6] = nm; smx[threadIdx.x >> 6] = mx; }
        __syncthreads();
        if (threadIdx.x == 0) {
            sc->n_moved = (int32_t)(snm[0] + snm[1] + snm[2] + snm[3]);
            sc->max_abs_delta = fmaxf(fmaxf(smx[0], smx[1]), fmaxf(smx[2], smx[3]));
        }
    }
    if (c >= k) return;
    const float d = delta[c];
    if (d == 0.f) return;
    const int32_t j = kept[c];
    const int64_t p0 = col_ptr[j], p1 = col_ptr[j + 1];
    bool out_of_range = false;
    const double term_limit = kFixTermLimit / (double)k;
    for (int64_t p = p0 + (threadIdx.x & 63); p < p1; p += 64) {
        const float v = val[p];
        // the accumulator holds sums below 2^23 in magnitude and up to k terms can land on one row: a term at or
        // above 2^22 / k (or not finite: the iteration has blown up) is reported instead of being allowed to wrap
        if (!(fabs((double)v * (double)d) < term_limit)) { out_of_range = true; continue; }
        atomicAdd((unsigned long long *)&racc[row_idx[p]], (unsigned long long)fix40(v, d));
    }
    if (out_of_range) atomicOr(&sc->overflow, 1u);
}

// Workgroups past res_blocks (there are some when another round follows at once, one scheduler) make the
// next round's key pass: it needs delta beta as this round leaves it and nothing this kernel writes.
__global__ __launch_bounds__(256) void k_csc_residual_apply(long long *__restrict__ racc, int64_t N,
                                                            float *__restrict__ r, uint32_t res_blocks,
                                                            KeysArgs next_keys, const RoundScalars *__restrict__ sc,
                                                            uint32_t *__restrict__ cnt, uint32_t *__restrict__ ovf_cnt)
{
    if (blockIdx.x >= res_blocks) {
        keys_hist_block(next_keys, blockIdx.x - res_blocks, gridDim.x - res_blocks);
        return;
    }
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i == 0) *ovf_cnt = 0u;                    // the round's inverted index is done with: empty it for the next round
    if (i >= N) return;
    if (cnt[i] != 0u) cnt[i] = 0u;
    const long long v = racc[i];
    if (sc->overflow) {
        // a product left the accumulator's range (set by the kernel before this one): the sums are not
        // trustworthy, and the residual says so: the objective and the optimality test then read as not finite
        r[i] = __int_as_float(0x7fc00000);
        if (v != 0) racc[i] = 0;
        return;
    }
    if (v != 0) {
        r[i] = (float)((double)r[i] - (double)v * kFixInv);
        racc[i] = 0;
    }
}

__global__ __launch_bounds__(256) void k_csc_kkt(const float *__restrict__ val, const int32_t *__restrict__ row_idx,
                                                 const int64_t *__restrict__ col_ptr, int64_t J,
                                                 const float *__restrict__ r, const float *__restrict__ beta, float lambda,
                                                 float *__restrict__ g_out, RoundScalars *__restrict__ sc)
{
    __shared__ float vm[4];
    float vmax = 0.f;
    for (int64_t j = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); j < J; j += (int64_t)gridDim.x * 4) {
        const float g = sparse_dot(val, row_idx, col_ptr[j], col_ptr[j + 1], r, threadIdx.x & 63);
        if ((threadIdx.x & 63) == 0) {
            if (g_out) g_out[j] = g;
            const float b = beta[j];
            float v;
            if (b == 0.f) v = fmaxf(fabsf(g) - lambda, 0.f);
            else v = fabsf(g - copysignf(lambda, b));
            if (!(v == v)) v = __uint_as_float(0x7F800000u);
            vmax = fmaxf(vmax, v);
        }
    }
    if ((threadIdx.x & 63) == 0) vm[threadIdx.x >> 6] = vmax;
    __syncthreads();
    if (threadIdx.x == 0)
        atomicMax(&sc->kkt_max_bits, __float_as_uint(fmaxf(fmaxf(vm[0], vm[1]), fmaxf(vm[2], vm[3]))));
}

// ---------------------------------------------------------------------------------------------
hipError_t csc_prepare()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_csc_gram), hipFuncAttributeMaxDynamicSharedMemorySize,
                               STRADS_MAX_L_PRIME * 8);
}

// zero the scratch counters and check col_ptr; *bad_host is valid after the stream is synchronised
hipError_t launch_csc_init(strads_lasso *h, uint32_t *bad_dev)
{
    const CscScratch s = csc_carve(h);
    hipLaunchKernelGGL(k_csc_zero, dim3(1024), dim3(256), 0, h->stream, s.cnt, s.racc, h->cfg.n, bad_dev, s.ovf_cnt);
    hipLaunchKernelGGL(k_csc_check, dim3(1024), dim3(256), 0, h->stream, h->cfg.col_ptr, h->cfg.j,
                       h->cfg.max_col_nnz, bad_dev);
    return launch_status(h->stream);
}

hipError_t launch_gram_csc(strads_lasso *h)
{
    const CscScratch s = csc_carve(h);
    // dynamic dependencies: the list is the movers and its length lives on the device
    const bool dynamic = h->cfg.deps == STRADS_DEPS_DYNAMIC;
    const int32_t *cand = dynamic ? h->at<int32_t>(h->ws.mcand) : h->at<int32_t>(h->ws.cand);
    const GramShape *n_dev = dynamic ? h->at<GramShape>(h->ws.dshape) : nullptr;
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    hipLaunchKernelGGL(k_csc_build, dim3((h->L + 3) / 4), dim3(256), 0, h->stream, cand, n_dev, h->L, h->cfg.col_ptr,
                       h->cfg.row_idx, h->cfg.x, s.cnt, s.bucket, s.cap, s.ovf_cnt, s.ovf);
    hipLaunchKernelGGL(k_csc_gram, dim3(h->L), dim3(256), (size_t)h->Lpad * 8, h->stream, cand, n_dev, h->cfg.col_ptr,
                       h->cfg.row_idx, h->cfg.x, s.cnt, s.bucket, s.cap, s.ovf_cnt, s.ovf, h->L, h->Lpad, h->cfg.rho,
                       h->at<uint64_t>(h->ws.mask), h->cfg.keep_gram ? h->at<float>(h->ws.gram) : nullptr,
                       &sc->near_rho_pairs);
    return launch_status(h->stream);
}

hipError_t launch_dots_cand_csc(strads_lasso *h)
{
    hipLaunchKernelGGL(k_csc_dots_cand, dim3((h->L + 3) / 4), dim3(256), 0, h->stream, h->cfg.x, h->cfg.row_idx,
                       h->cfg.col_ptr, h->at<int32_t>(h->ws.cand), h->L, dots_vector(h), h->cfg.lambda, h->step_scale,
                       h->at<float>(h->ws.beta), h->at<float>(h->ws.zc), h->at<float>(h->ws.dc),
                       h->at<float>(h->ws.nbc));
    return launch_status(h->stream);
}

hipError_t launch_dots_csc(strads_lasso *h)
{
    hipLaunchKernelGGL(k_csc_dots_update, dim3((h->L + 3) / 4), dim3(256), 0, h->stream, h->cfg.x, h->cfg.row_idx,
                       h->cfg.col_ptr, h->at<int32_t>(h->ws.kept), h->at<RoundScalars>(h->ws.scalars),
                       dots_vector(h), h->cfg.lambda, h->step_scale, h->at<float>(h->ws.beta),
                       h->at<float>(h->ws.dbeta), h->at<float>(h->ws.z), h->at<float>(h->ws.delta));
    return launch_status(h->stream);
}

hipError_t launch_residual_csc(strads_lasso *h, bool want_next_keys, bool *next_keys_done)
{
    const CscScratch s = csc_carve(h);
    hipLaunchKernelGGL(k_csc_residual_acc, dim3((h->L + 3) / 4), dim3(256), 0, h->stream, h->cfg.x, h->cfg.row_idx,
                       h->cfg.col_ptr, h->at<int32_t>(h->ws.kept), h->at<float>(h->ws.delta),
                       h->at<RoundScalars>(h->ws.scalars), s.racc);
    const unsigned res_blocks = (unsigned)((h->cfg.n + 255) / 256);
    unsigned key_blocks = 0;
    *next_keys_done = false;
    if (want_next_keys && h->n_lanes == 1) {
        key_blocks = (unsigned)((h->Js + 1023) / 1024);             // four keys per thread, at most 256 workgroups
        if (key_blocks > 256u) key_blocks = 256u;
        *next_keys_done = true;
    }
    hipLaunchKernelGGL(k_csc_residual_apply, dim3(res_blocks + key_blocks), dim3(256), 0, h->stream, s.racc,
                       h->cfg.n, h->at<float>(h->ws.r), res_blocks, keys_args(h),
                       h->at<RoundScalars>(h->ws.scalars), s.cnt, s.ovf_cnt);
    return launch_status(h->stream);
}

hipError_t launch_kkt_csc(strads_lasso *h, float *g_or_null)
{
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    hipError_t e = launch_clear_kkt(h);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_csc_kkt, dim3((unsigned)((h->cfg.j + 3) / 4 < 256 * 16 ? (h->cfg.j + 3) / 4 : 256 * 16)), dim3(256), 0, h->stream, h->cfg.x,
                       h->cfg.row_idx, h->cfg.col_ptr, h->cfg.j, dots_vector(h), h->at<float>(h->ws.beta),
                       h->cfg.lambda, g_or_null, sc);
    return launch_status(h->stream);
}

} // namespace strads
