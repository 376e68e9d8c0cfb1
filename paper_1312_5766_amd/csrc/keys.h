// Step 1's sampling keys: device code shared by the sampler's kernels and by the kernel that makes
// the next round's key pass early.  Not part of the public ABI.
#pragma once

#include "strads_internal.h"

namespace strads {

// ---------------------------------------------------------------------------------------------
// random numbers and the specified log2
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                        uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c0;
}

// log2 of a positive normal float: exponent by bit extraction, mantissa folded into
// [sqrt(1/2), sqrt(2)], then e + f*Q(f) with a fixed degree-8 Q in Horner form.
__device__ __forceinline__ float log2_spec(float x)
{
    const uint32_t bits = __float_as_uint(x);
    int e = (int)(bits >> 23) - 127;
    const uint32_t man = bits & 0x007FFFFFu;
    uint32_t mb;
    if (man > 0x003504F3u) { mb = man | 0x3F000000u; e += 1; }
    else                   { mb = man | 0x3F800000u; }
    const float f = __fsub_rn(__uint_as_float(mb), 1.0f);
    float q = 0x1.f841dcp-4f;
    q = __fmaf_rn(q, f, -0x1.a59aeap-3f);
    q = __fmaf_rn(q, f, 0x1.ba8738p-3f);
    q = __fmaf_rn(q, f, -0x1.e9d1e6p-3f);
    q = __fmaf_rn(q, f, 0x1.26d01cp-2f);
    q = __fmaf_rn(q, f, -0x1.715994p-2f);
    q = __fmaf_rn(q, f, 0x1.ec73dep-2f);
    q = __fmaf_rn(q, f, -0x1.715474p-1f);
    q = __fmaf_rn(q, f, 0x1.715476p+0f);
    return __fmaf_rn(f, q, (float)e);
}

// weight of coordinate j in the draw: (delta beta)^2 + eta (Theorem 1), |delta beta| + eta
// (Algorithm 1 as printed) or 1 (the uniform draw of the comparison schedulers of Section 5.1)
__device__ __forceinline__ float priority_weight(float dbeta, float eta, int priority)
{
    if (priority == STRADS_PRIORITY_LINEAR) return __fadd_rn(fabsf(dbeta), eta);
    if (priority == STRADS_PRIORITY_UNIFORM) return 1.0f;
    return __fmaf_rn(dbeta, dbeta, eta);
}

__device__ __forceinline__ float priority_key(float dbeta, float eta, uint64_t seed, uint64_t t, uint32_t j,
                                              int priority)
{
    const float w = priority_weight(dbeta, eta, priority);
    const uint32_t x = philox4x32_10_word0(j, 0u, (uint32_t)t, (uint32_t)(t >> 32), (uint32_t)seed,
                                           (uint32_t)(seed >> 32));
    const float u = __fmul_rn((float)(2u * (x >> 9) + 1u), 0x1.0p-24f);   // odd multiple of 2^-24, exact
    const float e = -log2_spec(u);
    const float key = __fsub_rn(log2_spec(w), log2_spec(e));
    return __fadd_rn(key, 0.0f);                                          // -0 -> +0
}

// order-preserving map float -> uint32 (larger float <=> larger integer)
__device__ __forceinline__ uint32_t orderable(float key)
{
    const uint32_t b = __float_as_uint(key);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// ---------------------------------------------------------------------------------------------
// pass 1 of the selection: keys + histogram of their top 11 bits
// ---------------------------------------------------------------------------------------------
// Js coordinates of scheduler shard `shard` out of `shards`: position i of the shard is coordinate
// j = i * shards + shard (one shard: j = i).  Keys are stored by position; the random number and
// delta beta are those of coordinate j.  The round index is the shard's device-side counter,
// advanced by the shard's last sampler kernel.
struct KeysArgs {
    const float *dbeta;
    uint32_t Js, shards, shard;
    float eta;
    uint64_t seed;
    const RoundScalars *sc;
    int priority;
    uint32_t *keys, *hist0;
};

// block `bid` of `nblocks` workgroups (any width up to 1024 threads) that share the pass
__device__ __forceinline__ void keys_hist_block(const KeysArgs &ka, uint32_t bid, uint32_t nblocks)
{
    __shared__ uint32_t lh[kHistBins];
    const uint64_t t = ka.sc->next_round;
    for (int i = threadIdx.x; i < kHistBins; i += blockDim.x) lh[i] = 0;
    __syncthreads();
    for (uint32_t i = bid * blockDim.x + threadIdx.x; i < ka.Js; i += nblocks * blockDim.x) {
        const uint32_t j = i * ka.shards + ka.shard;
        const uint32_t ok = orderable(priority_key(ka.dbeta[j], ka.eta, ka.seed, t, j, ka.priority));
        ka.keys[i] = ok;
        atomicAdd(&lh[ok >> 21], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kHistBins; i += blockDim.x)
        if (lh[i]) atomicAdd(&ka.hist0[i], lh[i]);
}

} // namespace strads
