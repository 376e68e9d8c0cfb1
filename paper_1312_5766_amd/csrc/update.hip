// The worker side of Algorithm 1 for a dense column-major design: eq. (2) evaluated for every
// kept coordinate from the SAME residual r = y - X beta (with unit-norm columns
//   x_j^T y - sum_{k != j} x_j^T x_k beta_k  =  x_j^T r + beta_j ),
// the soft-threshold S(a, lambda) = sign(a) max(|a| - lambda, 0), Step 4's bookkeeping
// (delta beta_j <- |change|), the residual update r <- r - sum_j x_j * change_j, the objective of
// eq. (1) and the optimality (KKT) check used as stopping rule.
//
// All of these stream columns of X once; they are HBM-bandwidth work: 16-byte coalesced loads
// along a column, fp32 FMA, fixed-order reductions (no floating-point atomics), so results are
// reproducible run to run.
#include "strads_internal.h"
#include "dots.h"
#include "keys.h"

namespace strads {

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
    return v;
}

// For every kept coordinate c < n_kept: z[c] = x_j^T r (r as it was when the round began), then
// eq. (2) and Step 4 at once: beta_j <- S(z + beta_j, lambda), delta[c] = change, dbeta_j = |change|.
// Kept coordinates are distinct, so each beta_j has exactly one writer.  Launched for the worst
// case (L columns); groups past the device-side count exit.
template <int TPC, bool VEC4>
__global__ __launch_bounds__(256) void k_dots_update(const float *__restrict__ X, int64_t N,
                                                     const int32_t *__restrict__ kept,
                                                     const RoundScalars *__restrict__ sc, const float *__restrict__ r,
                                                     float lambda, float step, float *__restrict__ beta,
                                                     float *__restrict__ dbeta, float *__restrict__ z,
                                                     float *__restrict__ delta)
{
    __shared__ float red[4];
    constexpr int CPB = 256 / TPC;              // columns per workgroup
    const int c = blockIdx.x * CPB + threadIdx.x / TPC;
    if (c >= sc->n_kept) return;                // TPC = 256: whole workgroup; TPC = 64: whole wavefront
    const int32_t j = kept[c];
    const float b = beta[j];                    // requested with the column, not after the reduction
    const float s = column_dot<TPC, VEC4>(X + (int64_t)j * N, r, N, threadIdx.x % TPC, red);
    if (threadIdx.x % TPC == 0) {
        const float nb = soft_threshold(s * step + b, lambda * step);     // step = 1: eq. (2) as printed
        const float d = nb - b;
        z[c] = s;
        delta[c] = d;
        beta[j] = nb;
        dbeta[j] = fabsf(d);
    }
}

// Long columns (a workgroup per column pays one pass over r per column): kept positions 2b and 2b + 1 by
// workgroup b, r read once for both.  Same arithmetic per column as k_dots_update<256, VEC4>.
template <bool VEC4>
__global__ __launch_bounds__(256) void k_dots_update_pair(const float *__restrict__ X, int64_t N,
                                                          const int32_t *__restrict__ kept,
                                                          const RoundScalars *__restrict__ sc,
                                                          const float *__restrict__ r, float lambda, float step,
                                                          float *__restrict__ beta, float *__restrict__ dbeta,
                                                          float *__restrict__ z, float *__restrict__ delta)
{
    __shared__ float red[2][4];
    const int c0 = 2 * (int)blockIdx.x, k = sc->n_kept;
    if (c0 >= k) return;
    const bool two = c0 + 1 < k;
    const int32_t ja = kept[c0], jb = kept[two ? c0 + 1 : c0];
    const float ba = beta[ja], bb = beta[jb];   // requested with the columns, not after the reduction
    float sa, sb;
    column_dot2<VEC4>(X + (int64_t)ja * N, X + (int64_t)jb * N, r, N, (int)threadIdx.x, red, sa, sb);
    if (threadIdx.x == 0) {
        const float na = soft_threshold(sa * step + ba, lambda * step);
        z[c0] = sa;
        delta[c0] = na - ba;
        beta[ja] = na;
        dbeta[ja] = fabsf(na - ba);
        if (two) {
            const float nb = soft_threshold(sb * step + bb, lambda * step);
            z[c0 + 1] = sb;
            delta[c0 + 1] = nb - bb;
            beta[jb] = nb;
            dbeta[jb] = fabsf(nb - bb);
        }
    }
}

template <bool VEC4>
__global__ __launch_bounds__(256) void k_dots_cand_pair(const float *__restrict__ X, int64_t N,
                                                        const int32_t *__restrict__ cand, CandDots cd)
{
    __shared__ float red[2][4];
    cand_dots_pair<VEC4>(X, N, cand, cd, (int)blockIdx.x, red);
}

// Dynamic dependencies: the update every candidate would make from the current residual.  For
// candidate position c < L: zc[c] = x_j^T r, nbc[c] = S(zc + beta_j, lambda), dc[c] = nbc - beta_j.
// Nothing of the solver state is written: which candidates are committed is decided later.
template <int TPC, bool VEC4>
__global__ __launch_bounds__(256) void k_dots_cand(const float *__restrict__ X, int64_t N,
                                                   const int32_t *__restrict__ cand, CandDots cd)
{
    __shared__ float red[4];
    cand_dots_block<TPC, VEC4>(X, N, cand, cd, (int)blockIdx.x, red);
}

// Residual update r <- r - sum_c x_{kept[c]} * delta[c], stage 1.  grid = (row tiles of 1024 rows,
// G column groups).  Group g owns kept positions [k*g/G, k*(g+1)/G) and sums its movers
// (delta != 0) in list order for 4 rows per thread -> part[g][i].
template <bool VEC4>
__global__ __launch_bounds__(256) void k_residual_partial(const float *__restrict__ X, int64_t N, int64_t Npad,
                                                          const int32_t *__restrict__ kept,
                                                          const float *__restrict__ delta,
                                                          RoundScalars *__restrict__ sc, float *__restrict__ part)
{
    __shared__ int32_t mcol[256];
    __shared__ float mdel[256];
    __shared__ uint32_t wcnt[4];
    const int k = sc->n_kept;
    const int G = gridDim.y, g = blockIdx.y;
    const int c0 = (int)((int64_t)k * g / G), c1 = (int)((int64_t)k * (g + 1) / G);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t i = ((int64_t)blockIdx.x * 256 + tid) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int cb = c0; cb < c1; cb += 256) {     // movers of this group, 256 kept positions at a time
        const int c = cb + tid;
        const float d = c < c1 ? delta[c] : 0.f;
        const bool mv = d != 0.f;
        const uint64_t m = __ballot(mv);
        if (lane == 0) wcnt[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = 0, tot = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) { const uint32_t v = wcnt[w]; if (w < wave) before += v; tot += v; }
        if (mv) {
            const uint32_t p = before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            mcol[p] = kept[c];
            mdel[p] = d;
        }
        __syncthreads();
        if (i < N) {
            if (VEC4) {
                uint32_t q = 0;
                for (; q + 3 < tot; q += 4) {
                    const float4 v0 = *reinterpret_cast<const float4 *>(X + (int64_t)mcol[q] * N + i);
                    const float4 v1 = *reinterpret_cast<const float4 *>(X + (int64_t)mcol[q + 1] * N + i);
                    const float4 v2 = *reinterpret_cast<const float4 *>(X + (int64_t)mcol[q + 2] * N + i);
                    const float4 v3 = *reinterpret_cast<const float4 *>(X + (int64_t)mcol[q + 3] * N + i);
                    const float d0 = mdel[q], d1 = mdel[q + 1], d2 = mdel[q + 2], d3 = mdel[q + 3];
                    acc.x += v0.x * d0; acc.y += v0.y * d0; acc.z += v0.z * d0; acc.w += v0.w * d0;
                    acc.x += v1.x * d1; acc.y += v1.y * d1; acc.z += v1.z * d1; acc.w += v1.w * d1;
                    acc.x += v2.x * d2; acc.y += v2.y * d2; acc.z += v2.z * d2; acc.w += v2.w * d2;
                    acc.x += v3.x * d3; acc.y += v3.y * d3; acc.z += v3.z * d3; acc.w += v3.w * d3;
                }
                for (; q < tot; ++q) {
                    const float4 v = *reinterpret_cast<const float4 *>(X + (int64_t)mcol[q] * N + i);
                    const float dd = mdel[q];
                    acc.x += v.x * dd; acc.y += v.y * dd; acc.z += v.z * dd; acc.w += v.w * dd;
                }
            } else {
                for (uint32_t q = 0; q < tot; ++q) {
                    const float *x = X + (int64_t)mcol[q] * N + i;
                    const float dd = mdel[q];
                    acc.x += x[0] * dd;
                    if (i + 1 < N) acc.y += x[1] * dd;
                    if (i + 2 < N) acc.z += x[2] * dd;
                    if (i + 3 < N) acc.w += x[3] * dd;
                }
            }
        }
        __syncthreads();
    }
    if (i < N) *reinterpret_cast<float4 *>(part + (int64_t)g * Npad + i) = acc;

    // round summary for strads_lasso_round's info (one workgroup does it; cheap: k <= 8192)
    if (blockIdx.x == 0 && g == 0) {
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

// stage 2: r[i] -= sum_g part[g][i], groups in order (a kernel boundary, not an in-kernel fence,
// makes the partial sums visible: a device-wide fence would write back every L2 of the 8 dies)
//
// Workgroups past res_blocks (there are some when another round follows at once, one scheduler) make
// the next round's key pass, as in k_residual_fused.
__global__ __launch_bounds__(256) void k_residual_apply(const float *__restrict__ part, int G, int64_t N, int64_t Npad,
                                                        float *__restrict__ r, uint32_t res_blocks, KeysArgs next_keys)
{
    if (blockIdx.x >= res_blocks) {
        keys_hist_block(next_keys, blockIdx.x - res_blocks, gridDim.x - res_blocks);
        return;
    }
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    float s = 0.f;
    int g = 0;
    for (; g + 7 < G; g += 8) {                 // eight independent loads in flight, summed in group order
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = part[(int64_t)(g + q) * Npad + i];
#pragma unroll
        for (int q = 0; q < 8; ++q) s += v[q];
    }
    for (; g < G; ++g) s += part[(int64_t)g * Npad + i];
    r[i] -= s;
}

// The same update in one kernel, for candidate lists of at most 4096: a workgroup of 16 wavefronts
// owns 64 rows (one per lane).  Wavefront w sums the movers w, w+16, ... of the kept list in list
// order, the 16 sums meet in LDS in wavefront order, and the first wavefront subtracts the total
// from r.  No partial sums leave the chip and one kernel boundary is saved, which is what a round
// of a small design spends its time on; long lists keep the two-stage path, whose grid grows with
// the list.
//
// Workgroups past res_blocks (there are some when another round follows at once) make the next
// round's key pass (pass 1 of its selection): it needs delta beta as this round left it, which the
// kernels before this one have written, and nothing this kernel writes, so the two share a launch
// and the next round starts one kernel further on.
constexpr int kFusedResidualMaxL = 4096;
__global__ __launch_bounds__(1024) void k_residual_fused(const float *__restrict__ X, int64_t N,
                                                         const int32_t *__restrict__ kept,
                                                         const float *__restrict__ delta,
                                                         RoundScalars *__restrict__ sc, float *__restrict__ r,
                                                         int32_t lpad, uint32_t res_blocks, KeysArgs next_keys)
{
    if (blockIdx.x >= res_blocks) {
        keys_hist_block(next_keys, blockIdx.x - res_blocks, gridDim.x - res_blocks);
        return;
    }
    __shared__ int32_t mcol[kFusedResidualMaxL];
    __shared__ float mdel[kFusedResidualMaxL];
    __shared__ uint32_t wcnt[16];
    __shared__ float red[16][64];
    __shared__ float wmax[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // everything this thread will want from memory whatever the kept count turns out to be is requested
    // at once (entry tid of the kept list, its row of r), so that the trips overlap instead of following
    // one another: the count, then the list, then the columns
    const int64_t i = (int64_t)blockIdx.x * 64 + lane;
    const int slot = tid < lpad ? tid : 0;      // the lists have lpad entries
    const float d_slot = delta[slot];
    const int32_t col_slot = kept[slot];
    const float r_old = (wave == 0 && i < N) ? r[i] : 0.f;
    const int k = sc->n_kept;                   // <= candidates per round <= kFusedResidualMaxL
    // the movers (delta != 0) of the kept list, in list order, 1024 entries at a time
    uint32_t tot = 0;
    float dmax = 0.f;
    for (int c0 = 0; c0 < k; c0 += 1024) {
        const int a = c0 + tid;
        const float d = a < k ? (c0 == 0 ? d_slot : delta[a]) : 0.f;
        const bool mv = d != 0.f;
        const uint64_t m = __ballot(mv);
        if (lane == 0) wcnt[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = 0, here = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) { const uint32_t v = wcnt[w]; if (w < wave) before += v; here += v; }
        if (mv) {
            const uint32_t p = tot + before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            mcol[p] = c0 == 0 ? col_slot : kept[a];
            mdel[p] = d;
        }
        tot += here;
        dmax = fmaxf(dmax, fabsf(d));
        __syncthreads();
    }

    float acc = 0.f;
    if (i < N) {
        uint32_t q = (uint32_t)wave;
        for (; q + 48u < tot; q += 64u) {       // four columns in flight
            const float v0 = X[(int64_t)mcol[q] * N + i], v1 = X[(int64_t)mcol[q + 16u] * N + i];
            const float v2 = X[(int64_t)mcol[q + 32u] * N + i], v3 = X[(int64_t)mcol[q + 48u] * N + i];
            acc += v0 * mdel[q];
            acc += v1 * mdel[q + 16u];
            acc += v2 * mdel[q + 32u];
            acc += v3 * mdel[q + 48u];
        }
        for (; q < tot; q += 16u) acc += X[(int64_t)mcol[q] * N + i] * mdel[q];
    }
    red[wave][lane] = acc;
    if (blockIdx.x == 0) {                      // round summary for strads_lasso_round's info
        float mx = dmax;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_down(mx, off));
        if (lane == 0) wmax[wave] = mx;
    }
    __syncthreads();
    if (wave == 0 && i < N) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += red[w][lane];
        r[i] = r_old - t;
    }
    if (blockIdx.x == 0 && tid == 0) {
        float mx = 0.f;
        for (int w = 0; w < 16; ++w) mx = fmaxf(mx, wmax[w]);
        sc->n_moved = (int32_t)tot;
        sc->max_abs_delta = mx;
    }
}

// Long candidate lists (more than kFusedResidualMaxL) over 16-byte aligned columns: the same one-kernel
// scheme with 256 rows per workgroup, four per lane, so that a wavefront takes 1 KB of a column at a
// time and has eight columns in flight.  Nothing but X is streamed: no partial sums go through HBM and no
// second kernel adds them up.  Wavefront w sums movers w, w+16, ... in list order, the 16 sums are added
// in wavefront order: the result does not depend on how the launch is laid out.
__global__ __launch_bounds__(1024) void k_residual_rows(const float *__restrict__ X, int64_t N,
                                                        const int32_t *__restrict__ kept,
                                                        const float *__restrict__ delta,
                                                        RoundScalars *__restrict__ sc, float *__restrict__ r,
                                                        int32_t lpad, uint32_t res_blocks, KeysArgs next_keys)
{
    if (blockIdx.x >= res_blocks) {
        keys_hist_block(next_keys, blockIdx.x - res_blocks, gridDim.x - res_blocks);
        return;
    }
    extern __shared__ int32_t rows_lds[];       // [lpad] mover columns, then [lpad] their changes (8 * lpad bytes)
    int32_t *mcol = rows_lds;
    float *mdel = reinterpret_cast<float *>(rows_lds + lpad);
    __shared__ uint32_t wcnt[128];
    __shared__ float4 red[16][64];
    __shared__ float wmax[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroup b runs on XCD b mod 8 and each XCD has its own L2.  A column's 1024-byte piece of one row
    // block does not start on a 128-byte line whenever 4 N is not a multiple of 128, so neighbouring row
    // blocks share a line of every such column: each XCD takes consecutive row blocks, and the shared line
    // comes from memory once per XCD instead of once per block.
    const uint32_t xcd = blockIdx.x & 7u, per = res_blocks >> 3, rem = res_blocks & 7u;
    const uint32_t blk = xcd * per + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    const int64_t i = ((int64_t)blk * 64 + lane) * 4;               // N is a multiple of 4 here
    // everything this thread will want of the kept list whatever its length turns out to be (entries
    // tid, tid + 1024, ... of the lpad-entry lists) and its rows of r are requested at once, before the
    // count is known: one trip to memory instead of one per 1024 entries
    constexpr int kMaxPass = STRADS_MAX_L_PRIME / 1024;
    float dq[kMaxPass];
    int32_t cq[kMaxPass];
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
        const int a = p * 1024 + tid;
        const int at = a < lpad ? a : 0;
        dq[p] = delta[at];
        cq[p] = kept[at];
    }
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 r_old = (wave == 0 && i < N) ? *reinterpret_cast<const float4 *>(r + i) : zero4;
    const int k = sc->n_kept;
    // The movers (delta != 0) of the kept list, in list order.  Entry p * 1024 + tid belongs to group p * 16 + wave
    // (64 consecutive entries); the groups' mover counts meet in LDS once, every wavefront takes their running sum
    // itself (two groups per lane), and each mover's place is its group's offset plus its rank in the group:
    // two barriers whatever the length of the list.
    static_assert(kMaxPass * 16 == 128, "two groups per lane");
    float dmax = 0.f;
    uint64_t ms[kMaxPass];
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
        const int a = p * 1024 + tid;
        if (a >= k) dq[p] = 0.f;
        ms[p] = __ballot(dq[p] != 0.f);
        if (lane == 0) wcnt[p * 16 + wave] = (uint32_t)__popcll(ms[p]);
        dmax = fmaxf(dmax, fabsf(dq[p]));
    }
    __syncthreads();
    const uint32_t c0 = wcnt[2 * lane], c1 = wcnt[2 * lane + 1];
    uint32_t incl = c0 + c1;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    const uint32_t before0 = incl - c0 - c1, before1 = incl - c1;     // movers before groups 2 * lane and 2 * lane + 1
    const uint32_t tot = __shfl(incl, 63);
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
        const int grp = p * 16 + wave;
        const uint32_t e0 = __shfl(before0, grp >> 1), e1 = __shfl(before1, grp >> 1);
        if (dq[p] != 0.f) {
            const uint32_t pos = ((grp & 1) ? e1 : e0) + (uint32_t)__popcll(ms[p] & ((1ull << lane) - 1ull));
            mcol[pos] = cq[p];
            mdel[pos] = dq[p];
        }
    }
    __syncthreads();

    float4 acc = zero4;
    if (i < N) {
        const float *xi = X + i;
        uint32_t q = (uint32_t)wave;
        for (; q + 112u < tot; q += 128u) {     // eight columns in flight
            float4 v[8];
            float dd[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                v[u] = *reinterpret_cast<const float4 *>(xi + (int64_t)mcol[q + 16u * u] * N);
                dd[u] = mdel[q + 16u * u];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                acc.x += v[u].x * dd[u]; acc.y += v[u].y * dd[u]; acc.z += v[u].z * dd[u]; acc.w += v[u].w * dd[u];
            }
        }
        for (; q < tot; q += 16u) {
            const float4 v = *reinterpret_cast<const float4 *>(xi + (int64_t)mcol[q] * N);
            const float dd = mdel[q];
            acc.x += v.x * dd; acc.y += v.y * dd; acc.z += v.z * dd; acc.w += v.w * dd;
        }
    }
    red[wave][lane] = acc;
    if (blockIdx.x == 0) {                      // round summary for strads_lasso_round's info
        float mx = dmax;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_down(mx, off));
        if (lane == 0) wmax[wave] = mx;
    }
    __syncthreads();
    if (wave == 0 && i < N) {
        float4 t = zero4;
#pragma unroll
        for (int w = 0; w < 16; ++w) { const float4 p = red[w][lane]; t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w; }
        *reinterpret_cast<float4 *>(r + i) = make_float4(r_old.x - t.x, r_old.y - t.y, r_old.z - t.z, r_old.w - t.w);
    }
    if (blockIdx.x == 0 && tid == 0) {
        float mx = 0.f;
        for (int w = 0; w < 16; ++w) mx = fmaxf(mx, wmax[w]);
        sc->n_moved = (int32_t)tot;
        sc->max_abs_delta = mx;
    }
}

// eq. (1): 1/2 sum r_i^2 + lambda sum |beta_j|, fp64 accumulation, two fixed-order stages
__global__ __launch_bounds__(256) void k_objective_partial(const float *__restrict__ r, int64_t N,
                                                           const float *__restrict__ beta, int64_t J, double lambda,
                                                           double *__restrict__ part)
{
    __shared__ double red[4];
    double s = 0.0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += stride) { const double v = r[i]; s += 0.5 * v * v; }
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < J; j += stride) s += lambda * fabs((double)beta[j]);
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// eq. (1) with the logistic loss: sum_i log(1 + exp(y_i v_i)) + lambda sum |beta_j|, v = -X beta
__global__ __launch_bounds__(256) void k_objective_logistic_partial(const float *__restrict__ y,
                                                                    const float *__restrict__ v, int64_t N,
                                                                    const float *__restrict__ beta, int64_t J,
                                                                    double lambda, double *__restrict__ part)
{
    __shared__ double red[4];
    double s = 0.0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += stride) {
        const double t = (double)y[i] * (double)v[i];
        s += t > 0.0 ? t + log1p(exp(-t)) : log1p(exp(t));
    }
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < J; j += stride) s += lambda * fabs((double)beta[j]);
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// Logistic loss: the weights w_i = y_i / (1 + exp(-y_i v_i)), v = -X beta, that take the residual's place
// in eq. (2) and in the optimality test; the padding up to Npad stays zero.
__global__ __launch_bounds__(256) void k_logistic_weights(const float *__restrict__ y, const float *__restrict__ v,
                                                          int64_t N, int64_t Npad, float *__restrict__ w)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= Npad) return;
    float out = 0.f;
    if (i < N) {
        const float yi = y[i];
        out = yi / (1.f + expf(-yi * v[i]));
    }
    w[i] = out;
}

__global__ __launch_bounds__(256) void k_objective_final(const double *__restrict__ part, int n, double *__restrict__ out)
{
    __shared__ double red[4];
    double s = threadIdx.x < n ? part[threadIdx.x] : 0.0;
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) *out = (red[0] + red[1]) + (red[2] + red[3]);
}

__device__ __forceinline__ float kkt_violation(float g, float b, float lambda)
{
    float v;
    if (b == 0.f) v = fmaxf(fabsf(g) - lambda, 0.f);
    else v = fabsf(g - copysignf(lambda, b));
    if (!(v == v)) v = __uint_as_float(0x7F800000u);         // NaN counts as an infinite violation
    return v;
}

// Optimality violation of eq. (1) per column and its maximum.  Workgroups stride over the
// columns and keep a running maximum; one integer atomicMax per workgroup at the end (float bits
// of a non-negative number are order-preserving), so the result is deterministic and the single
// result word is not hammered once per column.
template <int TPC, bool VEC4>
__global__ __launch_bounds__(256) void k_kkt(const float *__restrict__ X, int64_t N, int64_t J,
                                             const float *__restrict__ r, const float *__restrict__ beta, float lambda,
                                             float *__restrict__ g_out, RoundScalars *__restrict__ sc)
{
    __shared__ float red[4];
    __shared__ float vm[4];
    constexpr int CPB = 256 / TPC;
    float vmax = 0.f;
    for (int64_t j0 = (int64_t)blockIdx.x * CPB; j0 < J; j0 += (int64_t)gridDim.x * CPB) {
        const int64_t j = j0 + threadIdx.x / TPC;
        if (TPC == 64 && j >= J) break;         // whole wavefront; TPC = 256 has one column per workgroup
        const float g = column_dot<TPC, VEC4>(X + j * N, r, N, threadIdx.x % TPC, red);
        if (threadIdx.x % TPC == 0) {
            if (g_out) g_out[j] = g;
            vmax = fmaxf(vmax, kkt_violation(g, beta[j], lambda));
        }
        if (TPC > 64) __syncthreads();          // red[] is reused by the next column
    }
    if ((threadIdx.x & 63) == 0) vm[threadIdx.x >> 6] = vmax;
    __syncthreads();
    if (threadIdx.x == 0)
        atomicMax(&sc->kkt_max_bits, __float_as_uint(fmaxf(fmaxf(vm[0], vm[1]), fmaxf(vm[2], vm[3]))));
}

// The same pass for 2048 < N <= 1024*NR with 16-byte aligned columns: a persistent workgroup keeps
// its slice of r in registers (NR float4 per thread) and streams columns two at a time, so X is
// the only HBM/L2 traffic and one block-level reduction serves two columns.
template <int NR>
__global__ __launch_bounds__(256) void k_kkt_stream(const float *__restrict__ X, int64_t N, int64_t J,
                                                    const float *__restrict__ r, const float *__restrict__ beta,
                                                    float lambda, float *__restrict__ g_out,
                                                    RoundScalars *__restrict__ sc)
{
    __shared__ float red[2][4];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int64_t n4 = N >> 2;
    float4 rr[NR];
#pragma unroll
    for (int q = 0; q < NR; ++q) {
        const int64_t i = (int64_t)q * 256 + t;
        rr[q] = i < n4 ? reinterpret_cast<const float4 *>(r)[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float vmax = 0.f;
    for (int64_t j0 = (int64_t)blockIdx.x * 2; j0 < J; j0 += (int64_t)gridDim.x * 2) {
        const bool two = j0 + 1 < J;
        const float4 *xa = reinterpret_cast<const float4 *>(X + j0 * N);
        const float4 *xb = reinterpret_cast<const float4 *>(X + (two ? j0 + 1 : j0) * N);
        float4 va[NR], vb[NR];
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            const int64_t i = (int64_t)q * 256 + t;
            const int64_t ii = i < n4 ? i : n4 - 1;             // clamped: rr is zero there
            va[q] = xa[ii];
            vb[q] = xb[ii];
        }
        float sa = 0.f, sb = 0.f;
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            sa += va[q].x * rr[q].x + va[q].y * rr[q].y + va[q].z * rr[q].z + va[q].w * rr[q].w;
            sb += vb[q].x * rr[q].x + vb[q].y * rr[q].y + vb[q].z * rr[q].z + vb[q].w * rr[q].w;
        }
        sa = wave_sum(sa);
        sb = wave_sum(sb);
        if (lane == 0) { red[0][wave] = sa; red[1][wave] = sb; }
        __syncthreads();
        if (t < 2 && (t == 0 || two)) {
            const float g = (red[t][0] + red[t][1]) + (red[t][2] + red[t][3]);
            const int64_t j = j0 + t;
            if (g_out) g_out[j] = g;
            vmax = fmaxf(vmax, kkt_violation(g, beta[j], lambda));
        }
        __syncthreads();
    }
    if (t < 2 && vmax > 0.f) atomicMax(&sc->kkt_max_bits, __float_as_uint(vmax));
}

__global__ __launch_bounds__(256) void k_init_state(const float *__restrict__ y, int64_t N, int64_t Npad, int64_t J,
                                                    float c_init, int zero_state,
                                                    float *__restrict__ beta, float *__restrict__ dbeta,
                                                    float *__restrict__ r, uint32_t *__restrict__ hist,
                                                    uint32_t *__restrict__ scalars_words, int n_scalar_words)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    // histograms and round scalars start at zero (the sampler's last kernel re-zeroes them every round)
    if (blockIdx.x == 0) {
        for (int i = threadIdx.x; i < 2 * kHistBins; i += 256) hist[i] = 0u;
        for (int i = threadIdx.x; i < n_scalar_words; i += 256) scalars_words[i] = 0u;
    }
    // the padding of r stays zero for good: kernels that work on whole 64-row groups rely on it
    // squared loss: r = y - X 0; logistic loss: the state vector is -X 0
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < Npad; i += stride)
        r[i] = (i < N && !zero_state) ? y[i] : 0.f;
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < J; j += stride) { beta[j] = 0.f; dbeta[j] = c_init; }
}

__global__ void k_clear_kkt(RoundScalars *sc) { sc->kkt_max_bits = 0u; }

// ---------------------------------------------------------------------------------------------
hipError_t launch_dots_dense(strads_lasso *h)
{
    const RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    const float *r = dots_vector(h);
    const int32_t *kept = h->at<int32_t>(h->ws.kept);
    const bool wide = h->cfg.n > 2048;
    const unsigned grid = wide ? (unsigned)((h->L + 1) / 2) : (unsigned)((h->L + 3) / 4);
#define STRADS_DOTS_ARGS dim3(grid), dim3(256), 0, h->stream, h->cfg.x, h->cfg.n, kept, sc, r, h->cfg.lambda, h->step_scale, h->at<float>(h->ws.beta), h->at<float>(h->ws.dbeta), h->at<float>(h->ws.z), h->at<float>(h->ws.delta)
    if (wide) {
        if (h->vec4) hipLaunchKernelGGL((k_dots_update_pair<true>), STRADS_DOTS_ARGS);
        else hipLaunchKernelGGL((k_dots_update_pair<false>), STRADS_DOTS_ARGS);
    } else {
        if (h->vec4) hipLaunchKernelGGL((k_dots_update<64, true>), STRADS_DOTS_ARGS);
        else hipLaunchKernelGGL((k_dots_update<64, false>), STRADS_DOTS_ARGS);
    }
#undef STRADS_DOTS_ARGS
    return launch_status(h->stream);
}

CandDots cand_dots_args(strads_lasso *h)
{
    CandDots cd;
    cd.L = h->L;
    cd.wide = h->cfg.n > 2048 ? 1 : 0;
    cd.r = dots_vector(h);
    cd.lambda = h->cfg.lambda;
    cd.step = h->step_scale;
    cd.beta = h->at<float>(h->ws.beta);
    cd.zc = h->at<float>(h->ws.zc);
    cd.dc = h->at<float>(h->ws.dc);
    cd.nbc = h->at<float>(h->ws.nbc);
    return cd;
}

hipError_t launch_dots_cand(strads_lasso *h)
{
    const bool wide = h->cfg.n > 2048;
    const unsigned grid = wide ? (unsigned)((h->L + 1) / 2) : (unsigned)((h->L + 3) / 4);
    const CandDots cd = cand_dots_args(h);
#define STRADS_DOTS_CAND_ARGS dim3(grid), dim3(256), 0, h->stream, h->cfg.x, h->cfg.n, h->at<int32_t>(h->ws.cand), cd
    if (wide) {
        if (h->vec4) hipLaunchKernelGGL((k_dots_cand_pair<true>), STRADS_DOTS_CAND_ARGS);
        else hipLaunchKernelGGL((k_dots_cand_pair<false>), STRADS_DOTS_CAND_ARGS);
    } else {
        if (h->vec4) hipLaunchKernelGGL((k_dots_cand<64, true>), STRADS_DOTS_CAND_ARGS);
        else hipLaunchKernelGGL((k_dots_cand<64, false>), STRADS_DOTS_CAND_ARGS);
    }
#undef STRADS_DOTS_CAND_ARGS
    return launch_status(h->stream);
}

int residual_groups(int64_t n, int32_t l)
{
    const int64_t rowblocks = (n + 1023) / 1024;
    int64_t G = 2048 / rowblocks;
    if (G > kMaxResidualGroups) G = kMaxResidualGroups;
    if (G > l) G = l;
    if (G < 1) G = 1;
    return (int)G;
}

hipError_t launch_residual_dense(strads_lasso *h, bool want_next_keys, bool *next_keys_done)
{
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    *next_keys_done = false;
    // one kernel where one fits the shape: long, 16-byte aligned columns and more than 1024 candidates take
    // 256 rows per workgroup (it needs N / 256 workgroups to be enough to fill the chip); lists of at most
    // 4096 take 64 rows per workgroup; what is left (long lists over short columns) is done in two stages
    const bool rows = h->vec4 && h->cfg.n >= 32768 && h->L > 1024;
    if (h->residual_fused && (rows || h->L <= kFusedResidualMaxL)) {
        const unsigned res_blocks = rows ? (unsigned)((h->cfg.n / 4 + 63) / 64) : (unsigned)((h->cfg.n + 63) / 64);
        unsigned key_blocks = 0;
        if (want_next_keys && h->n_lanes == 1) {
            key_blocks = (unsigned)((h->Js + 4095) / 4096);         // four keys per thread, at most 256 workgroups
            if (key_blocks > 256u) key_blocks = 256u;
            *next_keys_done = true;
        }
        if (rows)
            hipLaunchKernelGGL(k_residual_rows, dim3(res_blocks + key_blocks), dim3(1024), (size_t)h->Lpad * 8, h->stream,
                               h->cfg.x, h->cfg.n, h->at<int32_t>(h->ws.kept), h->at<float>(h->ws.delta), sc,
                               h->at<float>(h->ws.r), h->Lpad, res_blocks, keys_args(h));
        else
            hipLaunchKernelGGL(k_residual_fused, dim3(res_blocks + key_blocks), dim3(1024), 0, h->stream,
                               h->cfg.x, h->cfg.n, h->at<int32_t>(h->ws.kept), h->at<float>(h->ws.delta), sc,
                               h->at<float>(h->ws.r), h->Lpad, res_blocks, keys_args(h));
        return launch_status(h->stream);
    }
    const int G = residual_groups(h->cfg.n, h->L);
    const dim3 grid((unsigned)((h->cfg.n + 1023) / 1024), (unsigned)G);
    float *part = h->at<float>(h->ws.rpart);
    if (h->vec4)
        hipLaunchKernelGGL(k_residual_partial<true>, grid, dim3(256), 0, h->stream, h->cfg.x, h->cfg.n, h->Npad,
                           h->at<int32_t>(h->ws.kept), h->at<float>(h->ws.delta), sc, part);
    else
        hipLaunchKernelGGL(k_residual_partial<false>, grid, dim3(256), 0, h->stream, h->cfg.x, h->cfg.n, h->Npad,
                           h->at<int32_t>(h->ws.kept), h->at<float>(h->ws.delta), sc, part);
    const hipError_t e = hipGetLastError();
    return e != hipSuccess ? e : launch_residual_apply(h, G, want_next_keys, next_keys_done);
}

hipError_t launch_residual_apply(strads_lasso *h, int groups, bool want_next_keys, bool *next_keys_done)
{
    const unsigned res_blocks = (unsigned)((h->cfg.n + 255) / 256);
    unsigned key_blocks = 0;
    *next_keys_done = false;
    if (want_next_keys && h->n_lanes == 1) {
        key_blocks = (unsigned)((h->Js + 1023) / 1024);             // four keys per thread, at most 256 workgroups
        if (key_blocks > 256u) key_blocks = 256u;
        *next_keys_done = true;
    }
    hipLaunchKernelGGL(k_residual_apply, dim3(res_blocks + key_blocks), dim3(256), 0, h->stream,
                       h->at<float>(h->ws.rpart), groups, h->cfg.n, h->Npad, h->at<float>(h->ws.r), res_blocks,
                       keys_args(h));
    return launch_status(h->stream);
}

hipError_t launch_objective(strads_lasso *h)
{
    double *part = h->at<double>(h->ws.objpart);
    if (h->cfg.loss == STRADS_LOSS_LOGISTIC)
        hipLaunchKernelGGL(k_objective_logistic_partial, dim3(kObjBlocks), dim3(256), 0, h->stream, h->cfg.y,
                           h->at<float>(h->ws.r), h->cfg.n, h->at<float>(h->ws.beta), h->cfg.j,
                           (double)h->cfg.lambda, part);
    else
        hipLaunchKernelGGL(k_objective_partial, dim3(kObjBlocks), dim3(256), 0, h->stream, h->at<float>(h->ws.r),
                           h->cfg.n, h->at<float>(h->ws.beta), h->cfg.j, (double)h->cfg.lambda, part);
    hipLaunchKernelGGL(k_objective_final, dim3(1), dim3(256), 0, h->stream, part, kObjBlocks,
                       h->at<double>(h->ws.objout));
    return launch_status(h->stream);
}

hipError_t launch_kkt_dense(strads_lasso *h, float *g_or_null)
{
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    hipLaunchKernelGGL(k_clear_kkt, dim3(1), dim3(1), 0, h->stream, sc);
    const bool wide = h->cfg.n > 2048;
    if (wide && h->vec4 && h->cfg.n <= 16 * 1024) {
        // persistent: 8 workgroups per compute unit
        int64_t g = (h->cfg.j + 1) / 2;
        if (g > 256 * 8) g = 256 * 8;
        const int nr = (int)((h->cfg.n / 4 + 255) / 256);
#define STRADS_KKT_STREAM(NR) hipLaunchKernelGGL((k_kkt_stream<NR>), dim3((unsigned)g), dim3(256), 0, h->stream, h->cfg.x, h->cfg.n, h->cfg.j, dots_vector(h), h->at<float>(h->ws.beta), h->cfg.lambda, g_or_null, sc)
        if (nr <= 4) STRADS_KKT_STREAM(4);
        else if (nr <= 8) STRADS_KKT_STREAM(8);
        else if (nr <= 12) STRADS_KKT_STREAM(12);
        else STRADS_KKT_STREAM(16);
#undef STRADS_KKT_STREAM
        return launch_status(h->stream);
    }
    int64_t gk = wide ? h->cfg.j : (h->cfg.j + 3) / 4;
    // Long columns: about 16 columns per workgroup, dispatched as compute units become free (32 workgroups' worth
    // of columns per resident workgroup: the XCDs of a chip do not work through them at the same speed, and with
    // two workgroups per slot, 244 columns each, the pass took 2 % longer).  Short columns: a few workgroups per
    // compute unit, each striding over the columns.
    const int64_t cap = wide ? 256 * 256 : 256 * 16;
    if (gk > cap) gk = cap;
    const unsigned grid = (unsigned)gk;
#define STRADS_KKT(TPC, V) hipLaunchKernelGGL((k_kkt<TPC, V>), dim3(grid), dim3(256), 0, h->stream, h->cfg.x, h->cfg.n, h->cfg.j, dots_vector(h), h->at<float>(h->ws.beta), h->cfg.lambda, g_or_null, sc)
    if (wide) { if (h->vec4) STRADS_KKT(256, true); else STRADS_KKT(256, false); }
    else      { if (h->vec4) STRADS_KKT(64, true);  else STRADS_KKT(64, false); }
#undef STRADS_KKT
    return launch_status(h->stream);
}

hipError_t launch_logistic_weights(strads_lasso *h)
{
    hipLaunchKernelGGL(k_logistic_weights, dim3((unsigned)((h->Npad + 255) / 256)), dim3(256), 0, h->stream, h->cfg.y,
                       h->at<float>(h->ws.r), h->cfg.n, h->Npad, h->at<float>(h->ws.w));
    return launch_status(h->stream);
}

hipError_t launch_clear_kkt(strads_lasso *h)
{
    hipLaunchKernelGGL(k_clear_kkt, dim3(1), dim3(1), 0, h->stream, h->at<RoundScalars>(h->ws.scalars));
    return launch_status(h->stream);
}

hipError_t launch_init_state(strads_lasso *h)
{
    hipLaunchKernelGGL(k_init_state, dim3(1024), dim3(256), 0, h->stream, h->cfg.y, h->cfg.n, h->Npad, h->cfg.j,
                       h->cfg.c_init, h->cfg.loss == STRADS_LOSS_LOGISTIC ? 1 : 0,
                       h->at<float>(h->ws.beta), h->at<float>(h->ws.dbeta), h->at<float>(h->ws.r),
                       h->at<uint32_t>(h->ws.hist), h->at<uint32_t>(h->ws.scalars), (int)(sizeof(RoundScalars) / 4));
    return launch_status(h->stream);
}

// The update of eq. (2) has no 1 / ||x_j||^2 factor because columns are standardised to unit l2 norm: a
// precondition the library states and, in a debug build, checks when a handle is created.  One wavefront
// per column (grid-stride), the sum of squares in fp32 (fp64 across the wavefront); a column off by more
// than 1e-3 sets bit 1 of bad_input.
__global__ __launch_bounds__(256) void k_check_unit_norm(int32_t layout, const float *__restrict__ x, int64_t N, int64_t J,
                                                         const int32_t *__restrict__ row_idx,
                                                         const int64_t *__restrict__ col_ptr,
                                                         const float *__restrict__ col_mean,
                                                         const float *__restrict__ col_scale, uint32_t *__restrict__ bad)
{
    const int lane = threadIdx.x & 63;
    const int64_t words = (N + 63) / 64 * 4;
    for (int64_t j = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); j < J; j += (int64_t)gridDim.x * 4) {
        double s = 0.0;
        if (layout == STRADS_LAYOUT_DENSE_COLMAJOR) {
            const float *c = x + j * N;
            for (int64_t i = lane; i < N; i += 64) s += (double)c[i] * (double)c[i];
        } else if (layout == STRADS_LAYOUT_CSC) {
            for (int64_t p = col_ptr[j] + lane; p < col_ptr[j + 1]; p += 64) s += (double)x[p] * (double)x[p];
        } else {
            const uint32_t *w = reinterpret_cast<const uint32_t *>(x) + j * words;
            const float m = col_mean[j], sc = col_scale[j];
            for (int64_t i = lane; i < N; i += 64) {
                const float v = __fmul_rn(__fsub_rn((float)((w[i >> 4] >> (2 * (i & 15))) & 3u), m), sc);
                s += (double)v * (double)v;
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off);
        if (lane == 0 && !(fabs(s - 1.0) <= 1e-3)) atomicOr(bad, 2u);
    }
}

hipError_t update_prepare()
{
    // the long-list residual kernel keeps the mover list (up to 8192 columns and changes) in dynamic LDS
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_residual_rows),
                               hipFuncAttributeMaxDynamicSharedMemorySize, STRADS_MAX_L_PRIME * 8);
}

hipError_t launch_check_unit_norm(strads_lasso *h)
{
    const int64_t want = (h->cfg.j + 3) / 4;
    hipLaunchKernelGGL(k_check_unit_norm, dim3((unsigned)(want < 8192 ? want : 8192)), dim3(256), 0, h->stream,
                       h->cfg.layout, h->cfg.x, h->cfg.n, h->cfg.j, h->cfg.row_idx, h->cfg.col_ptr, h->cfg.col_mean,
                       h->cfg.col_scale, &h->at<RoundScalars>(h->ws.scalars)->bad_input);
    return launch_status(h->stream);
}

} // namespace strads
