// Step 1 of SAP for the Lasso (Section 2.1, Step 1; Algorithm 1's draw of the set U of P'
// coefficients; Theorem 1's weight): draw P' distinct coordinates with probability
// proportional to w_j = (delta beta_j)^2 + eta.
//
// Successive sampling without replacement is done with the Gumbel-top-k identity: the P'
// largest of  key_j = log2 w_j - log2(-log2 u_j),  u_j uniform in (0,1), ARE such a draw, in
// draw order.  u_j comes from a counter-based generator (Philox-4x32-10, Salmon et al., SC'11)
// keyed by (seed, round, j), so a draw never depends on the launch shape.  The fp32 key
// arithmetic is specified operation by operation (correctly rounded IEEE add / fma only), which
// makes the key bits, and with them the candidate list, reproducible on any IEEE machine.
//
// Selection of the P' largest (key desc, j asc) out of J: MSB-first radix select on the
// order-preserving 32-bit image of the key, two 11-bit histogram passes, then everything
// strictly above the 22-bit boundary prefix is appended to the output and the few keys on the
// boundary prefix are resolved and everything is sorted by one workgroup in LDS.
#include "strads_internal.h"
#include "keys.h"

namespace strads {

// ---------------------------------------------------------------------------------------------
// block helpers (256-thread workgroups unless stated)
// ---------------------------------------------------------------------------------------------
// In a histogram whose bins are ordered ascending, find the bin that holds the K-th largest
// element: above(bin) < K <= above(bin) + hist[bin].  All threads of the workgroup (256 or more)
// call it; results are returned to all.  tmp: 6 uint32 of LDS.  Thread t owns bins 8t..8t+7; the suffix sums over the
// per-thread totals are taken inside each wavefront with lane shifts, then across the four
// wavefronts through LDS (two barriers in all).
__device__ void find_bin_desc(const uint32_t *__restrict__ hist, uint32_t K, uint32_t *tmp, uint32_t &bin,
                              uint32_t &above)
{
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const bool owner = t < 256;                 // wider workgroups: the other threads only meet the barriers
    uint32_t loc[8];
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { loc[i] = owner ? hist[8 * t + i] : 0u; s += loc[i]; }
    uint32_t suf = s;                           // inclusive suffix sum over the lanes of this wavefront
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t v = __shfl_down(suf, d);
        if (lane + d < 64) suf += v;
    }
    if (owner && lane == 0) tmp[wave] = suf;    // total of this wavefront
    if (t == 0) { tmp[4] = 0; tmp[5] = 0; }
    __syncthreads();
    if (owner) {
        uint32_t higher = 0;                    // totals of the wavefronts holding higher bins
#pragma unroll
        for (int w = 1; w < 4; ++w) if (w > wave) higher += tmp[w];
        uint32_t ab = higher + suf - s;         // elements in bins above this thread's 8 bins
#pragma unroll
        for (int i = 7; i >= 0; --i) {
            if (ab < K && K <= ab + loc[i]) { tmp[4] = 8 * t + i; tmp[5] = ab; }
            ab += loc[i];
        }
    }
    __syncthreads();
    bin = tmp[4];
    above = tmp[5];
    __syncthreads();
}

// Append one 64-bit item per flagged lane to a global list; one atomic per wavefront.
__device__ __forceinline__ void wave_append(bool flag, uint64_t item, uint64_t *__restrict__ list,
                                            uint32_t *__restrict__ counter)
{
    const uint64_t m = __ballot(flag);
    if (m == 0) return;
    const int lane = __lane_id();
    uint32_t base = 0;
    if (lane == __ffsll((long long)m) - 1) base = atomicAdd(counter, (uint32_t)__popcll(m));
    base = __shfl(base, __ffsll((long long)m) - 1);
    if (flag) list[base + __popcll(m & ((1ull << lane) - 1ull))] = item;
}

// ---------------------------------------------------------------------------------------------
// pass 1: keys + histogram of the top 11 bits
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_keys_hist(KeysArgs ka)
{
    keys_hist_block(ka, blockIdx.x, gridDim.x);
}

__global__ __launch_bounds__(256) void k_keys_only(const float *__restrict__ dbeta, uint32_t J, float eta,
                                                   uint64_t seed, uint64_t t, int priority,
                                                   float *__restrict__ keys)
{
    for (uint32_t j = blockIdx.x * 256u + threadIdx.x; j < J; j += gridDim.x * 256u)
        keys[j] = priority_key(dbeta[j], eta, seed, t, j, priority);
}

// pass 2: histogram of the next 11 bits among keys in the boundary bin of pass 1
__global__ __launch_bounds__(1024) void k_hist2(const uint32_t *__restrict__ keys, uint32_t J, uint32_t L,
                                               const uint32_t *__restrict__ hist0, uint32_t *__restrict__ hist1,
                                               RoundScalars *__restrict__ sc)
{
    __shared__ uint32_t lh[kHistBins];
    __shared__ uint32_t tmp[258];
    // The thread's first keys are requested before the boundary bin is looked up (which takes a trip to
    // memory for the histogram and two barriers), so that the two latencies overlap.
    constexpr int kEarly = 4;
    const uint32_t stride = gridDim.x * blockDim.x;
    uint32_t early[kEarly];
#pragma unroll
    for (int q = 0; q < kEarly; ++q) {
        const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x + q * stride;
        early[q] = j < J ? keys[j] : 0u;
    }
    uint32_t b0, above;
    find_bin_desc(hist0, L, tmp, b0, above);
    if (blockIdx.x == 0 && threadIdx.x == 0) { sc->bin0 = b0; sc->rem1 = L - above; }
    for (int i = threadIdx.x; i < kHistBins; i += blockDim.x) lh[i] = 0;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kEarly; ++q) {
        const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x + q * stride;
        if (j < J && (early[q] >> 21) == b0) atomicAdd(&lh[(early[q] >> 10) & 0x7FFu], 1u);
    }
    for (uint32_t j = blockIdx.x * blockDim.x + threadIdx.x + kEarly * stride; j < J; j += stride) {
        const uint32_t ok = keys[j];
        if ((ok >> 21) == b0) atomicAdd(&lh[(ok >> 10) & 0x7FFu], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kHistBins; i += blockDim.x)
        if (lh[i]) atomicAdd(&hist1[i], lh[i]);
}

constexpr int kCollectPerThread = 16;

// pass 3: everything strictly above the 22-bit boundary prefix is selected; keys on the prefix
// go to the boundary list.  Items are (orderable key << 32) | (2^32-1 - j): all distinct, and
// larger item <=> (larger key, then smaller j).  Keys are indexed by position in the scheduler
// shard; the item carries the coordinate itself (position * shards + shard).
//
// Every appended item needs a slot from one of two device-wide counters, and atomics on one
// address are served one after the other (roughly 8 ns each), so a workgroup looks at
// 256 * kCollectPerThread keys, counts first, and reserves its slots with ONE atomic per list.
__global__ __launch_bounds__(256) void k_collect(const uint32_t *__restrict__ keys, uint32_t J, uint32_t shards,
                                                 uint32_t shard, const uint32_t *__restrict__ hist1,
                                                 RoundScalars *__restrict__ sc, uint64_t *__restrict__ sel,
                                                 uint64_t *__restrict__ bnd)
{
    __shared__ uint32_t tmp[258];
    __shared__ uint32_t wtot[2][4], wbase[2][4];
    const int lane = __lane_id(), wave = threadIdx.x >> 6;
    const uint32_t base = (blockIdx.x * 256u + (threadIdx.x & ~63u)) * kCollectPerThread + (threadIdx.x & 63u);
    // the keys are requested before the boundary prefix is looked up, so that the two trips to memory overlap
    uint32_t okv[kCollectPerThread];
#pragma unroll
    for (int q = 0; q < kCollectPerThread; ++q) {
        const uint32_t j = base + q * 64u;
        okv[q] = j < J ? keys[j] : 0u;
    }
    const uint32_t b0 = sc->bin0, rem1 = sc->rem1;
    uint32_t b1, above;
    find_bin_desc(hist1, rem1, tmp, b1, above);
    const uint32_t p22 = (b0 << 11) | b1;
    if (blockIdx.x == 0 && threadIdx.x == 0) { sc->prefix22 = p22; sc->rem2 = rem1 - above; }
    uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
    for (int q = 0; q < kCollectPerThread; ++q) {
        const uint32_t j = base + q * 64u;
        const uint32_t p = okv[q] >> 10;
        n_gt += (j < J && p > p22) ? 1u : 0u;
        n_eq += (j < J && p == p22) ? 1u : 0u;
    }
    // wavefront-level inclusive scan of the per-lane counts, then one reservation per workgroup
    uint32_t off_gt = n_gt, off_eq = n_eq;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t a = __shfl_up(off_gt, d), b = __shfl_up(off_eq, d);
        if (lane >= d) { off_gt += a; off_eq += b; }
    }
    if (lane == 63) { wtot[0][wave] = off_gt; wtot[1][wave] = off_eq; }
    __syncthreads();
    if (threadIdx.x < 2) {
        const int l = threadIdx.x;
        const uint32_t t0 = wtot[l][0], t1 = wtot[l][1], t2 = wtot[l][2], t3 = wtot[l][3];
        const uint32_t tot = t0 + t1 + t2 + t3;
        uint32_t b = 0;
        if (tot) b = atomicAdd(l == 0 ? &sc->n_sel : &sc->n_bnd, tot);
        wbase[l][0] = b; wbase[l][1] = b + t0; wbase[l][2] = b + t0 + t1; wbase[l][3] = b + t0 + t1 + t2;
    }
    __syncthreads();
    uint32_t base_gt = wbase[0][wave] + off_gt - n_gt;
    uint32_t base_eq = wbase[1][wave] + off_eq - n_eq;
#pragma unroll
    for (int q = 0; q < kCollectPerThread; ++q) {
        const uint32_t j = base + q * 64u;
        const uint32_t p = okv[q] >> 10;
        const uint64_t item = ((uint64_t)okv[q] << 32) | (uint64_t)(0xFFFFFFFFu - (j * shards + shard));
        if (j < J && p > p22) sel[base_gt++] = item;
        if (j < J && p == p22) bnd[base_eq++] = item;
    }
}

// ---------------------------------------------------------------------------------------------
// final: one workgroup of 1024 threads
// ---------------------------------------------------------------------------------------------
__device__ void bitonic_sort_desc(uint64_t *a, uint32_t n /* power of two */)
{
    const uint32_t tid = threadIdx.x;
    for (uint32_t k = 2; k <= n; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = tid; i < n; i += 1024u) {
                const uint32_t p = i ^ j;
                if (p > i) {
                    const uint64_t x = a[i], y = a[p];
                    const bool desc = (i & k) == 0;
                    if (desc ? (x < y) : (x > y)) { a[i] = y; a[p] = x; }
                }
            }
            __syncthreads();
        }
    }
}

// The value that lane (l ^ J) of the wavefront holds, for J a power of two below 64, without a
// trip through LDS: quad permutes and row mirrors of the data-parallel move for J < 16 (an
// exclusive-or of the lane number with 7 or 15 is a mirror; two of them compose to J = 4 and 8),
// the row and half-wave swap instructions of gfx950 for J = 16 and 32.
template <int J> __device__ __forceinline__ uint32_t lane_xor(uint32_t v)
{
    constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kQuadXor3 = 0x1B, kRowMirror = 0x140, kHalfMirror = 0x141;
    if constexpr (J == 1) {
        return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, kQuadXor1, 0xF, 0xF, false);
    } else if constexpr (J == 2) {
        return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, kQuadXor2, 0xF, 0xF, false);
    } else if constexpr (J == 4) {
        const int t = __builtin_amdgcn_mov_dpp((int)v, kHalfMirror, 0xF, 0xF, false);
        return (uint32_t)__builtin_amdgcn_mov_dpp(t, kQuadXor3, 0xF, 0xF, false);
    } else if constexpr (J == 8) {
        const int t = __builtin_amdgcn_mov_dpp((int)v, kRowMirror, 0xF, 0xF, false);
        return (uint32_t)__builtin_amdgcn_mov_dpp(t, kHalfMirror, 0xF, 0xF, false);
    } else if constexpr (J == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        return (__lane_id() & 16) ? r[0] : r[1];
    } else {
        static_assert(J == 32, "lane_xor: J is a power of two below 64");
        const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return (__lane_id() & 32) ? r[0] : r[1];
    }
}

// One compare-exchange step of the bitonic network (merge width k, partner distance J < 64).
// Items are distinct or equal padding, so "take the partner's item" is one comparison.
template <int J> __device__ __forceinline__ uint64_t bitonic_step_in_wave(uint64_t x, uint32_t i, uint32_t k)
{
    const uint64_t y = ((uint64_t)lane_xor<J>((uint32_t)(x >> 32)) << 32) | lane_xor<J>((uint32_t)x);
    const bool take_max = ((i & k) == 0) == ((i & (uint32_t)J) == 0);   // lower index of a descending pair keeps the larger
    return ((x < y) == take_max) ? y : x;
}

template <int JMAX> __device__ __forceinline__ uint64_t bitonic_merge_in_wave(uint64_t x, uint32_t i, uint32_t k)
{
    if constexpr (JMAX >= 32) x = bitonic_step_in_wave<32>(x, i, k);
    if constexpr (JMAX >= 16) x = bitonic_step_in_wave<16>(x, i, k);
    if constexpr (JMAX >= 8) x = bitonic_step_in_wave<8>(x, i, k);
    if constexpr (JMAX >= 4) x = bitonic_step_in_wave<4>(x, i, k);
    if constexpr (JMAX >= 2) x = bitonic_step_in_wave<2>(x, i, k);
    return bitonic_step_in_wave<1>(x, i, k);
}

// Bitonic sort, descending, of up to 1024 items held one per thread (1024 threads): exchanges
// with a partner less than 64 lanes away stay in the vector registers (lane_xor), the ten longer
// strides go through LDS, alternating between two buffers so that one barrier per step is enough.
// Returns the item that belongs at position threadIdx.x.
constexpr uint32_t kRegSortLdsItems = 2048;
__device__ uint64_t bitonic_sort_desc_1024(uint64_t x, uint64_t *xch /* kRegSortLdsItems items of LDS */)
{
    const uint32_t i = threadIdx.x;
    x = bitonic_merge_in_wave<1>(x, i, 2);
    x = bitonic_merge_in_wave<2>(x, i, 4);
    x = bitonic_merge_in_wave<4>(x, i, 8);
    x = bitonic_merge_in_wave<8>(x, i, 16);
    x = bitonic_merge_in_wave<16>(x, i, 32);
    x = bitonic_merge_in_wave<32>(x, i, 64);
    uint32_t half = 0;
    for (uint32_t k = 128; k <= 1024u; k <<= 1) {
        for (uint32_t j = k >> 1; j >= 64u; j >>= 1) {
            uint64_t *buf = xch + half;
            half ^= 1024u;                                // the step after the next reuses this buffer: its
            buf[i] = x;                                   // readers have passed the barrier in between
            __syncthreads();
            const uint64_t y = buf[i ^ j];
            const bool take_max = ((i & k) == 0) == ((i & j) == 0);
            x = ((x < y) == take_max) ? y : x;
        }
        x = bitonic_merge_in_wave<32>(x, i, k);
    }
    __syncthreads();                                      // callers may reuse xch at once
    return x;
}

constexpr uint32_t kRegSortMax = 1024;
constexpr uint32_t kRankMax = 192;      // boundary lists up to this length are ranked by counting

// exclusive rank of a flagged thread among the flagged threads of a 1024-thread block
__device__ __forceinline__ uint32_t block_rank(bool flag, uint32_t *wave_tot /* 17 */, uint32_t &total)
{
    const int lane = __lane_id(), wave = threadIdx.x >> 6;
    const uint64_t m = __ballot(flag);
    if (lane == 0) wave_tot[wave] = (uint32_t)__popcll(m);
    __syncthreads();
    uint32_t before = 0, tot = 0;
    for (int w = 0; w < 16; ++w) { const uint32_t c = wave_tot[w]; if (w < wave) before += c; tot += c; }
    __syncthreads();
    total = tot;
    return before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}

__global__ __launch_bounds__(1024) void k_finalize(RoundScalars *__restrict__ sc, uint64_t *__restrict__ sel,
                                                   uint64_t *__restrict__ bnd, uint32_t L, uint32_t Lpad,
                                                   uint32_t cap, uint32_t shards, int32_t *__restrict__ cand,
                                                   uint32_t *__restrict__ hist)
{
    extern __shared__ uint64_t lds[];
    __shared__ uint32_t h8[256];
    __shared__ uint32_t wt[17];
    __shared__ uint32_t pick[2];
    const uint32_t tid = threadIdx.x;
    uint32_t n_sel = sc->n_sel, nb = sc->n_bnd, need = sc->rem2;
    // what the collect pass selected outright is final: this thread's item of it is requested now, so that
    // its trip to memory overlaps the work on the boundary list (steps A and B only append behind it)
    const uint32_t n_sel_collected = n_sel;
    const uint64_t early_item = sel[tid];         // (any value past the collected part; the buffer holds 2 x 8192 items)

    // A. (rare) boundary list longer than the LDS sort can hold: peel 8-bit digits below the
    //    22-bit prefix until it fits.  Items are distinct, so this always terminates.
    int shift = 42;
    while (nb > cap && shift > 0) {
        const int width = shift < 8 ? shift : 8;
        shift -= width;
        const uint32_t dmask = (1u << width) - 1u;
        if (tid < 256) h8[tid] = 0;
        __syncthreads();
        for (uint32_t i = tid; i < nb; i += 1024u) atomicAdd(&h8[(uint32_t)(bnd[i] >> shift) & dmask], 1u);
        __syncthreads();
        if (tid == 0) {
            uint32_t ab = 0; int d = (int)dmask;
            for (; d > 0; --d) { if (need <= ab + h8[d]) break; ab += h8[d]; }
            pick[0] = (uint32_t)d; pick[1] = ab;
        }
        __syncthreads();
        const uint32_t d = pick[0], ab = pick[1];
        uint32_t w_eq = 0, w_gt = n_sel;
        for (uint32_t s = 0; s < nb; s += 1024u) {
            const uint32_t i = s + tid;
            const uint64_t v = i < nb ? bnd[i] : 0ull;
            const uint32_t dg = (uint32_t)(v >> shift) & dmask;
            const bool gt = i < nb && dg > d, eq = i < nb && dg == d;
            uint32_t tg, te;
            const uint32_t rg = block_rank(gt, wt, tg);
            const uint32_t re = block_rank(eq, wt, te);   // block_rank's barriers also order the reads above
            if (gt) sel[w_gt + rg] = v;
            if (eq) bnd[w_eq + re] = v;                    // w_eq + re <= s + tid: already read
            w_gt += tg; w_eq += te;
            __syncthreads();
        }
        n_sel += ab; need -= ab; nb = w_eq;
        __syncthreads();
    }

    // B. take the `need` largest boundary items
    if (nb == need) {
        for (uint32_t i = tid; i < nb; i += 1024u) sel[n_sel + i] = bnd[i];
    } else if (nb <= kRankMax) {
        // few items (the usual case with a 22-bit prefix): an item's rank is the number of larger
        // items, counted against all of them through LDS broadcasts; items are distinct, so the
        // ranks 0..need-1 are exactly the wanted ones.  Step C puts everything in order anyway.
        if (tid < nb) lds[tid] = bnd[tid];
        __syncthreads();
        if (tid < nb) {
            const uint64_t x = lds[tid];
            uint32_t rank = 0;
            for (uint32_t i = 0; i < nb; ++i) rank += lds[i] > x ? 1u : 0u;
            if (rank < need) sel[n_sel + rank] = x;
        }
    } else if (nb <= kRegSortMax) {
        const uint64_t v = bitonic_sort_desc_1024(tid < nb ? bnd[tid] : 0ull, lds);
        if (tid < need) sel[n_sel + tid] = v;
    } else {
        uint32_t p2 = 1; while (p2 < nb) p2 <<= 1;
        for (uint32_t i = tid; i < p2; i += 1024u) lds[i] = i < nb ? bnd[i] : 0ull;
        __syncthreads();
        bitonic_sort_desc(lds, p2);
        for (uint32_t i = tid; i < need; i += 1024u) sel[n_sel + i] = lds[i];
    }
    __threadfence_block();
    __syncthreads();

    // C. sort the L selected items: descending item = draw order
    if (L <= kRegSortMax) {
        const uint64_t mine = tid < n_sel_collected ? early_item : (tid < L ? sel[tid] : 0ull);
        const uint64_t v = bitonic_sort_desc_1024(mine, lds);
        if (tid < Lpad) cand[tid] = tid < L ? (int32_t)(0xFFFFFFFFu - (uint32_t)v) : 0;
    }
    // longer lists are put in order by k_sort_chunks + k_merge_rank, spread over many workgroups

    // D. leave the histograms and per-round scalars clean for the next round
    for (uint32_t i = tid; i < 2u * kHistBins; i += 1024u) hist[i] = 0;
    // (gram_next: the 256-wide tile kernel's queue position; the kernel that adds its tile slots resets it as
    // well, this covers a round that was cut short between the two)
    if (tid == 0) { sc->n_sel = 0; sc->n_bnd = 0; sc->near_rho_pairs = 0; sc->gram_next = 0u; sc->next_round += shards; }
}

// Draw order for lists longer than 1024 items, in two kernels.  (1) every workgroup sorts one
// chunk of 1024 items (descending) in registers.  (2) the items are distinct, so the final
// position of an item is the number of items greater than it: its position inside its own sorted
// chunk plus, for every other chunk, the count found by binary search.  All chunks sit in LDS.
__global__ __launch_bounds__(1024) void k_sort_chunks(const uint64_t *__restrict__ sel, uint32_t L,
                                                      uint64_t *__restrict__ sorted)
{
    __shared__ uint64_t xch[kRegSortLdsItems];
    const uint32_t i = blockIdx.x * 1024u + threadIdx.x;
    sorted[i] = bitonic_sort_desc_1024(i < L ? sel[i] : 0ull, xch);     // zeros (padding) sort last
}

__global__ __launch_bounds__(256) void k_merge_rank(const uint64_t *__restrict__ sorted, uint32_t L, uint32_t Lpad,
                                                    uint32_t n_chunks, int32_t *__restrict__ cand)
{
    extern __shared__ uint64_t all[];             // [n_chunks * 1024]
    const uint32_t n = n_chunks * 1024u;
    for (uint32_t i = threadIdx.x; i < n; i += 256u) all[i] = sorted[i];
    __syncthreads();
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= n) return;
    const uint64_t x = all[i];
    if (x != 0ull) {
        uint32_t rank = i & 1023u;
        const uint32_t own = i >> 10;
        for (uint32_t c = 0; c < n_chunks; ++c) {
            if (c == own) continue;
            const uint64_t *a = all + c * 1024u;  // descending: count of elements > x = first index with a[idx] < x
            uint32_t lo = 0, hi = 1024;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (a[mid] > x) lo = mid + 1; else hi = mid;
            }
            rank += lo;
        }
        cand[rank] = (int32_t)(0xFFFFFFFFu - (uint32_t)x);
    }
    if (i >= L && i < Lpad) cand[i] = 0;          // padding slots of the candidate list
}

// ---------------------------------------------------------------------------------------------
// Workgroup width and count of the two histogram passes.  Every workgroup flushes its LDS histogram
// with global atomics, so there are at most 256 of them; when that cap binds, the workgroups get
// wider instead (up to 1024 threads), so that a thread's share stays at a few keys and each
// compute unit has enough wavefronts to cover the memory latency.
static inline int sampler_threads(int64_t J)
{
    int t = 256;
    while (t < 1024 && (J + (int64_t)t * 4 - 1) / ((int64_t)t * 4) > 256) t *= 2;
    return t;
}

static inline int sampler_grid(int64_t J)
{
    const int64_t per = (int64_t)sampler_threads(J) * 4;
    int64_t b = (J + per - 1) / per;
    if (b < 1) b = 1;
    if (b > 256) b = 256;
    return (int)b;
}

// (also run whenever the solver state is set from outside: a CSC range error reported for the old state is dropped)
__global__ void k_set_next_round(RoundScalars *sc, unsigned long long t) { sc->next_round = t; sc->overflow = 0u; }

hipError_t launch_set_next_round(strads_lasso *h, hipStream_t stream, int64_t next_round)
{
    hipLaunchKernelGGL(k_set_next_round, dim3(1), dim3(1), 0, stream, h->at<RoundScalars>(h->ws.scalars),
                       (unsigned long long)next_round);
    return launch_status(stream);
}

KeysArgs keys_args(strads_lasso *h)
{
    KeysArgs ka;
    ka.dbeta = h->at<float>(h->ws.dbeta);
    ka.Js = (uint32_t)h->Js;
    ka.shards = (uint32_t)h->n_lanes;
    ka.shard = (uint32_t)h->lane_id;
    ka.eta = h->cfg.eta;
    ka.seed = h->cfg.seed;
    ka.sc = h->at<RoundScalars>(h->ws.scalars);
    ka.priority = h->cfg.priority;
    ka.keys = h->at<uint32_t>(h->ws.keys);
    ka.hist0 = h->at<uint32_t>(h->ws.hist);
    return ka;
}

hipError_t launch_sampler(strads_lasso *h, bool keys_done)
{
    const uint32_t J = (uint32_t)h->Js, L = (uint32_t)h->L;      // this shard's coordinates
    const uint32_t S = (uint32_t)h->n_lanes, sh = (uint32_t)h->lane_id;
    const int g = sampler_grid(h->Js);
    uint32_t *keys = h->at<uint32_t>(h->ws.keys);
    uint32_t *hist = h->at<uint32_t>(h->ws.hist);
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    uint64_t *sel = h->at<uint64_t>(h->ws.sel), *bnd = h->at<uint64_t>(h->ws.bnd);
    const int bt = sampler_threads(h->Js);
    // (keys_done: the previous round's last kernel has already made this pass, see launch_residual_dense)
    if (!keys_done) hipLaunchKernelGGL(k_keys_hist, dim3(g), dim3(bt), 0, h->stream, keys_args(h));
    hipLaunchKernelGGL(k_hist2, dim3(g), dim3(bt), 0, h->stream, keys, J, L, hist, hist + kHistBins, sc);
    const unsigned gc = (unsigned)((h->Js + 256 * kCollectPerThread - 1) / (256 * kCollectPerThread));
    hipLaunchKernelGGL(k_collect, dim3(gc), dim3(256), 0, h->stream, keys, J, S, sh, hist + kHistBins, sc, sel, bnd);
    // LDS of the final kernel: the two exchange buffers of the register sort, or the boundary
    // list (at most `cap` items, padded to a power of two) when that is longer.  Kept small so the
    // kernel can share a compute unit with another shard's Gram workgroups.
    const uint32_t cap = (uint32_t)h->select_cap;
    uint32_t items = kRegSortLdsItems;
    while (items < cap) items <<= 1;
    const size_t lds = (size_t)items * sizeof(uint64_t);
    hipLaunchKernelGGL(k_finalize, dim3(1), dim3(1024), lds, h->stream, sc, sel, bnd, L, (uint32_t)h->Lpad, cap, S,
                       h->at<int32_t>(h->ws.cand), hist);
    if (L > kRegSortMax) {
        const uint32_t n_chunks = (L + 1023u) / 1024u;
        uint64_t *sorted = sel + STRADS_MAX_L_PRIME;          // second half of the selection buffer
        hipLaunchKernelGGL(k_sort_chunks, dim3(n_chunks), dim3(1024), 0, h->stream, sel, L, sorted);
        hipLaunchKernelGGL(k_merge_rank, dim3(n_chunks * 4u), dim3(256), (size_t)n_chunks * 1024u * 8u, h->stream,
                           sorted, L, (uint32_t)h->Lpad, n_chunks, h->at<int32_t>(h->ws.cand));
    }
    return launch_status(h->stream);
}

hipError_t launch_keys_only(strads_lasso *h, int64_t round, float *keys)
{
    hipLaunchKernelGGL(k_keys_only, dim3(sampler_grid(h->cfg.j)), dim3(256), 0, h->stream,
                       h->at<float>(h->ws.dbeta), (uint32_t)h->cfg.j, h->cfg.eta, h->cfg.seed, (uint64_t)round,
                       h->cfg.priority, keys);
    return launch_status(h->stream);
}

hipError_t sampler_prepare()
{
    hipError_t e0 = hipFuncSetAttribute(reinterpret_cast<const void *>(k_merge_rank),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, STRADS_MAX_L_PRIME * 8);
    if (e0 != hipSuccess) return e0;
    // the final kernel sorts up to 16384 64-bit items in LDS (128 KiB): raise its dynamic-LDS limit
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_finalize),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STRADS_MAX_L_PRIME * 8);
}

} // namespace strads
