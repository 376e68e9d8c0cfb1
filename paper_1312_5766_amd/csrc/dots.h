// Device helpers shared by the kernels that take x_j^T r over a dense column and apply eq. (2).
// Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace strads {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
    return v;                                   // lane 0 holds the sum
}

// dot product of one column with r by TPC threads (TPC = 64: one wavefront, 256: a workgroup)
template <int TPC, bool VEC4>
__device__ __forceinline__ float column_dot(const float *__restrict__ x, const float *__restrict__ r, int64_t N,
                                            int t, float *red /* TPC/64 floats of LDS, TPC > 64 only */)
{
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (VEC4) {
        const float4 *x4 = reinterpret_cast<const float4 *>(x);
        const float4 *r4 = reinterpret_cast<const float4 *>(r);
        const int64_t n4 = N >> 2;
        int64_t i = t;
        for (; i + 3 * TPC < n4; i += 4 * TPC) {
            const float4 a0 = x4[i], a1 = x4[i + TPC], a2 = x4[i + 2 * TPC], a3 = x4[i + 3 * TPC];
            const float4 b0 = r4[i], b1 = r4[i + TPC], b2 = r4[i + 2 * TPC], b3 = r4[i + 3 * TPC];
            s0 += a0.x * b0.x + a0.y * b0.y + a0.z * b0.z + a0.w * b0.w;
            s1 += a1.x * b1.x + a1.y * b1.y + a1.z * b1.z + a1.w * b1.w;
            s2 += a2.x * b2.x + a2.y * b2.y + a2.z * b2.z + a2.w * b2.w;
            s3 += a3.x * b3.x + a3.y * b3.y + a3.z * b3.z + a3.w * b3.w;
        }
        for (; i < n4; i += TPC) {
            const float4 a = x4[i], b = r4[i];
            s0 += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
        }
    } else {
        for (int64_t i = t; i < N; i += TPC) s0 += x[i] * r[i];
    }
    float s = wave_sum((s0 + s1) + (s2 + s3));
    if (TPC > 64) {
        if ((t & 63) == 0) red[t >> 6] = s;
        __syncthreads();
        s = 0.f;
        if (t == 0) for (int w = 0; w < TPC / 64; ++w) s += red[w];
    }
    return s;                                   // valid in thread 0 of the group
}

// Two columns at once by a workgroup of 256 threads: every piece of r is loaded once and used for both
// columns, which takes a third off the requests to the L2 (r lives there; X comes from HBM).  Each
// column's sum is formed exactly as column_dot<256, VEC4> forms it (same partial sums, same order), so
// the two routes give the same bits.  Results in sa, sb, valid in thread 0.
template <bool VEC4>
__device__ __forceinline__ void column_dot2(const float *__restrict__ xa, const float *__restrict__ xb,
                                            const float *__restrict__ r, int64_t N, int t, float (*red)[4],
                                            float &sa, float &sb)
{
    constexpr int TPC = 256;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f, b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
    if (VEC4) {
        const float4 *xa4 = reinterpret_cast<const float4 *>(xa);
        const float4 *xb4 = reinterpret_cast<const float4 *>(xb);
        const float4 *r4 = reinterpret_cast<const float4 *>(r);
        const int64_t n4 = N >> 2;
        int64_t i = t;
        for (; i + 3 * TPC < n4; i += 4 * TPC) {
            const float4 p0 = xa4[i], p1 = xa4[i + TPC], p2 = xa4[i + 2 * TPC], p3 = xa4[i + 3 * TPC];
            const float4 q0 = xb4[i], q1 = xb4[i + TPC], q2 = xb4[i + 2 * TPC], q3 = xb4[i + 3 * TPC];
            const float4 v0 = r4[i], v1 = r4[i + TPC], v2 = r4[i + 2 * TPC], v3 = r4[i + 3 * TPC];
            a0 += p0.x * v0.x + p0.y * v0.y + p0.z * v0.z + p0.w * v0.w;
            a1 += p1.x * v1.x + p1.y * v1.y + p1.z * v1.z + p1.w * v1.w;
            a2 += p2.x * v2.x + p2.y * v2.y + p2.z * v2.z + p2.w * v2.w;
            a3 += p3.x * v3.x + p3.y * v3.y + p3.z * v3.z + p3.w * v3.w;
            b0 += q0.x * v0.x + q0.y * v0.y + q0.z * v0.z + q0.w * v0.w;
            b1 += q1.x * v1.x + q1.y * v1.y + q1.z * v1.z + q1.w * v1.w;
            b2 += q2.x * v2.x + q2.y * v2.y + q2.z * v2.z + q2.w * v2.w;
            b3 += q3.x * v3.x + q3.y * v3.y + q3.z * v3.z + q3.w * v3.w;
        }
        for (; i < n4; i += TPC) {
            const float4 p = xa4[i], q = xb4[i], v = r4[i];
            a0 += p.x * v.x + p.y * v.y + p.z * v.z + p.w * v.w;
            b0 += q.x * v.x + q.y * v.y + q.z * v.z + q.w * v.w;
        }
    } else {
        for (int64_t i = t; i < N; i += TPC) { const float v = r[i]; a0 += xa[i] * v; b0 += xb[i] * v; }
    }
    const float wa = wave_sum((a0 + a1) + (a2 + a3)), wb = wave_sum((b0 + b1) + (b2 + b3));
    if ((t & 63) == 0) { red[0][t >> 6] = wa; red[1][t >> 6] = wb; }
    __syncthreads();
    sa = sb = 0.f;
    if (t == 0)
        for (int w = 0; w < TPC / 64; ++w) { sa += red[0][w]; sb += red[1][w]; }
}

__device__ __forceinline__ float soft_threshold(float a, float lambda)
{
    const float m = fabsf(a) - lambda;
    return m > 0.f ? copysignf(m, a) : 0.f;
}

// The update candidate position c would make from the vector r: zc[c] = x_j^T r,
// nbc[c] = S(zc * step + beta_j, lambda * step) (step = 1: eq. (2) as printed), dc[c] = nbc - beta_j.
// Nothing of the solver state is written.  One group of TPC threads per candidate, 256 / TPC
// candidates per workgroup `block`.
struct CandDots {
    int32_t L;                  // candidates; 0: none wanted
    int32_t wide;               // 1: a workgroup per candidate, 0: a wavefront per candidate
    const float *r;
    float lambda, step;
    const float *beta;
    float *zc, *dc, *nbc;
};

template <int TPC, bool VEC4>
__device__ __forceinline__ void cand_dots_block(const float *__restrict__ X, int64_t N,
                                                const int32_t *__restrict__ cand, const CandDots &cd, int block,
                                                float *red)
{
    constexpr int CPB = 256 / TPC;
    const int c = block * CPB + (int)threadIdx.x / TPC;
    if (c >= cd.L) return;                      // TPC = 256: whole workgroup; TPC = 64: whole wavefront
    const int32_t j = cand[c];
    const float b = cd.beta[j];                 // requested with the column, not after the reduction
    const float s = column_dot<TPC, VEC4>(X + (int64_t)j * N, cd.r, N, (int)threadIdx.x % TPC, red);
    if (threadIdx.x % TPC == 0) {
        const float nb = soft_threshold(s * cd.step + b, cd.lambda * cd.step);
        cd.zc[c] = s;
        cd.nbc[c] = nb;
        cd.dc[c] = nb - b;
    }
}

// The same for candidate positions 2*block and 2*block + 1 by one workgroup (long columns, stand-alone kernel).
template <bool VEC4>
__device__ __forceinline__ void cand_dots_pair(const float *__restrict__ X, int64_t N,
                                               const int32_t *__restrict__ cand, const CandDots &cd, int block,
                                               float (*red)[4])
{
    const int c0 = 2 * block;
    if (c0 >= cd.L) return;
    const bool two = c0 + 1 < cd.L;
    const int32_t ja = cand[c0], jb = cand[two ? c0 + 1 : c0];
    const float ba = cd.beta[ja], bb = cd.beta[jb];
    float sa, sb;
    column_dot2<VEC4>(X + (int64_t)ja * N, X + (int64_t)jb * N, cd.r, N, (int)threadIdx.x, red, sa, sb);
    if (threadIdx.x == 0) {
        const float na = soft_threshold(sa * cd.step + ba, cd.lambda * cd.step);
        cd.zc[c0] = sa;
        cd.nbc[c0] = na;
        cd.dc[c0] = na - ba;
        if (two) {
            const float nb = soft_threshold(sb * cd.step + bb, cd.lambda * cd.step);
            cd.zc[c0 + 1] = sb;
            cd.nbc[c0 + 1] = nb;
            cd.dc[c0 + 1] = nb - bb;
        }
    }
}

} // namespace strads
