// Step 2 of SAP for the Lasso, first half (Section 2.1, Step 2; Algorithm 1's constraint on
// B_1): the dependencies d(x_a, x_b) = |x_a^T x_b| between the P' candidates, i.e. the Gram
// matrix of the gathered columns X_S, and from it one bit per pair: "conflict" iff NOT |g| < rho.
//
// This is a dense contraction (L' x N times N x L'), so it runs on the matrix cores:
// v_mfma_f32_32x32x2_f32, fp32 in, fp32 accumulate.  A workgroup of 4 wavefronts owns one
// 128 x 128 output tile of the upper triangle and one slice of the row (K) range; each
// wavefront holds a 64 x 64 sub-tile as 2 x 2 MFMA accumulators.  Columns of X are contiguous
// along K, so both operand panels are staged K-contiguous in LDS with coalesced 16-byte loads,
// double-buffered, and read back 16 bytes per lane: lane (i, h) of a wavefront reads
// k = 8*s + 4*h .. +3 of column i and feeds component c to the c-th of four MFMAs.  The MFMA
// sums over its two k-slots, and the assignment of k values to slots is the same for both
// operands, so any such assignment yields the same dot products.
//
// K-slices are written as fp32 partial tiles and summed in fixed order by the mask kernel, so
// results do not depend on scheduling.
#include "strads_internal.h"

namespace strads {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kPad = 4;                         // LDS row padding, floats
constexpr int kRow = kGramKT + kPad;            // LDS row stride, floats
constexpr int kPanel = kGramTile * kRow;        // floats per operand panel per stage

// 4 consecutive K values of one column, zero beyond kend.  No branch: the address is clamped into
// the column and the value is selected, so the main loop stays one straight-line block.
template <bool VEC4>
__device__ __forceinline__ float4 load_k4(const float *__restrict__ col, int64_t k, int64_t kend)
{
    if (VEC4) {
        const bool in = k < kend;                             // kend and k are multiples of 4 here
        const float4 v = *reinterpret_cast<const float4 *>(col + (in ? k : kend - 4));
        return in ? v : make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
        float4 v;
        const int64_t last = kend - 1;
        v.x = col[k + 0 <= last ? k + 0 : last]; v.x = (k + 0 <= last) ? v.x : 0.f;
        v.y = col[k + 1 <= last ? k + 1 : last]; v.y = (k + 1 <= last) ? v.y : 0.f;
        v.z = col[k + 2 <= last ? k + 2 : last]; v.z = (k + 2 <= last) ? v.z : 0.f;
        v.w = col[k + 3 <= last ? k + 3 : last]; v.w = (k + 3 <= last) ? v.w : 0.f;
        return v;
    }
}

// grid.x = T(T+1)/2 * split (T = Lpad/128): upper-triangular tiles only, K-slice fastest.
// Software pipeline per LDS stage st (32 K values): registers hold stage st+1 (fetched one stage
// ago), they are written to the other LDS buffer, the fetch of stage st+2 is issued, then stage st
// is multiplied out of LDS; one barrier per stage.
template <bool VEC4>
__global__ __launch_bounds__(256, 2) void k_gram_tiles(const float *__restrict__ X, int64_t N,
                                                       const int32_t *__restrict__ cand, int32_t L, int32_t Lpad,
                                                       int32_t T, int32_t split, int64_t kchunk,
                                                       float *__restrict__ P)
{
    const int32_t s = blockIdx.x % split;
    int32_t u = blockIdx.x / split;             // index into the row-major upper triangle
    int32_t ta = 0;
    while (u >= T - ta) { u -= T - ta; ++ta; }
    const int32_t tb = ta + u;

    extern __shared__ float smem[];             // [2 stages][A panel | B panel]
    const int tid = threadIdx.x;
    const int64_t kbeg = (int64_t)s * kchunk;
    const int64_t kend = (kbeg + kchunk < N) ? kbeg + kchunk : N;
    const int nstage = (int)((kend - kbeg + kGramKT - 1) / kGramKT);

    // this thread stages 4 A-columns and 4 B-columns: column (it*32 + tid/8), floats (tid%8)*4..+3.
    // Columns past the candidate count are clamped to the last candidate: their products land in
    // rows/columns >= L of the tile, which nobody reads.
    const int crow = tid >> 3, kq = (tid & 7) * 4;
    const float *col[8];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        int ia = ta * kGramTile + it * 32 + crow, ib = tb * kGramTile + it * 32 + crow;
        ia = ia < L ? ia : L - 1;
        ib = ib < L ? ib : L - 1;
        col[it] = X + (int64_t)cand[ia] * N;
        col[4 + it] = X + (int64_t)cand[ib] * N;
    }

    float4 R[8];
    auto fetch = [&](int st) {
        const int64_t k = kbeg + (int64_t)st * kGramKT + kq;
#pragma unroll
        for (int i = 0; i < 8; ++i) R[i] = load_k4<VEC4>(col[i], k, kend);
    };
    auto stash = [&](int buf) {
        float *pa = smem + buf * 2 * kPanel, *pb = pa + kPanel;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            *reinterpret_cast<float4 *>(pa + (it * 32 + crow) * kRow + kq) = R[it];
            *reinterpret_cast<float4 *>(pb + (it * 32 + crow) * kRow + kq) = R[4 + it];
        }
    };

    const int wave = tid >> 6, lane = tid & 63;
    const int wr = wave >> 1, wc = wave & 1;    // 64x64 sub-tile of this wavefront
    const int li = lane & 31, lh = lane >> 5;

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int offa = (wr * 64 + li) * kRow + lh * 4;
    const int offb = kPanel + (wc * 64 + li) * kRow + lh * 4;
    auto compute = [&](int buf) {
        const float *pa = smem + buf * 2 * kPanel + offa;
        const float *pb = smem + buf * 2 * kPanel + offb;
#pragma unroll
        for (int ks = 0; ks < kGramKT / 8; ++ks) {
            const float4 a0 = *reinterpret_cast<const float4 *>(pa + ks * 8);
            const float4 a1 = *reinterpret_cast<const float4 *>(pa + 32 * kRow + ks * 8);
            const float4 b0 = *reinterpret_cast<const float4 *>(pb + ks * 8);
            const float4 b1 = *reinterpret_cast<const float4 *>(pb + 32 * kRow + ks * 8);
            const float av0[4] = {a0.x, a0.y, a0.z, a0.w}, av1[4] = {a1.x, a1.y, a1.z, a1.w};
            const float bv0[4] = {b0.x, b0.y, b0.z, b0.w}, bv1[4] = {b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0[c], bv0[c], acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0[c], bv1[c], acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av1[c], bv0[c], acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av1[c], bv1[c], acc[1][1], 0, 0, 0);
            }
        }
    };

    fetch(0);
    stash(0);
    if (nstage > 1) fetch(1);
    __syncthreads();
    int st = 0;
    for (; st + 2 < nstage; ++st) {             // steady state: no conditionals inside
        stash((st + 1) & 1);
        fetch(st + 2);
        compute(st & 1);
        __syncthreads();
    }
    if (st + 1 < nstage) {
        stash((st + 1) & 1);
        compute(st & 1);
        __syncthreads();
        ++st;
    }
    compute(st & 1);

    // accumulator layout of the 32x32 MFMA: register v of lane (li, lh) holds
    // row 8*(v/4) + 4*lh + (v%4), column li of the 32x32 block.
    float *out = P + (int64_t)s * Lpad * Lpad;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int colo = tb * kGramTile + wc * 64 + b * 32 + li;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = ta * kGramTile + wr * 64 + a * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                out[(int64_t)row * Lpad + colo] = acc[a][b][v];
            }
        }
}

// Sum the K-slices in slice order and emit the conflict bits (and, optionally, the fp32 Gram).
// One thread per (row a, column b) with b in the tiles at or right of a's diagonal tile; 64
// consecutive b per wavefront make one 64-bit mask word.
__global__ __launch_bounds__(256) void k_gram_mask(const float *__restrict__ P, int32_t split, int32_t L,
                                                   int32_t Lpad, float rho, uint64_t *__restrict__ mask,
                                                   float *__restrict__ gram, int32_t *__restrict__ near_pairs)
{
    const int32_t a = blockIdx.y;
    const int32_t b = blockIdx.x * 256 + threadIdx.x;
    const int32_t first = (a / kGramTile) * kGramTile;      // first column of a's diagonal tile
    if (b < first || b >= Lpad) return;                     // uniform per wavefront (both are multiples of 64)
    float g = 0.f;
    const int64_t plane = (int64_t)Lpad * Lpad;
    for (int32_t s = 0; s < split; ++s) g += P[s * plane + (int64_t)a * Lpad + b];
    const bool live = a < L && b < L && a != b;
    const float ag = fabsf(g);
    const bool conflict = live && !(ag < rho);
    const uint64_t w = __ballot(conflict);
    if ((threadIdx.x & 63) == 0) mask[(int64_t)a * (Lpad / 64) + (b >> 6)] = w;
    if (near_pairs) {
        const bool nr = live && b > a && fabsf(ag - rho) <= 1e-6f;
        const uint64_t m = __ballot(nr);
        if (m && (threadIdx.x & 63) == 0) atomicAdd(near_pairs, (int32_t)__popcll(m));
    }
    if (gram) {
        gram[(int64_t)a * Lpad + b] = g;
        if (b >= first + kGramTile) gram[(int64_t)b * Lpad + a] = g;   // mirror the tiles right of the diagonal
    }
}

// Conflict bits from a caller-supplied full Gram (stage entry for parity tests).
__global__ __launch_bounds__(256) void k_mask_from_gram(const float *__restrict__ G, int32_t L, int32_t Lpad,
                                                        float rho, uint64_t *__restrict__ mask)
{
    const int32_t a = blockIdx.y;
    const int32_t b = blockIdx.x * 256 + threadIdx.x;
    if (b >= Lpad) return;                                  // whole wavefronts: Lpad is a multiple of 64
    const bool live = a < L && b < L && a != b;
    const float g = live ? G[(int64_t)a * L + b] : 0.f;
    const uint64_t w = __ballot(live && !(fabsf(g) < rho));
    if ((threadIdx.x & 63) == 0) mask[(int64_t)a * (Lpad / 64) + (b >> 6)] = w;
}

int gram_split_auto(int64_t n, int32_t lpad)
{
    // Workgroups = upper-triangular tiles x K-slices.  Two workgroups are resident per compute
    // unit (LDS), so the launch runs in rounds of 512.  With few tiles, slice K as far as a slice
    // still has 2 LDS stages, to get enough workgroups in flight to cover memory latency; with
    // many tiles, pick the slice count that wastes the least of the last round, preferring fewer
    // slices (less partial-sum traffic) among near-equals.
    const int64_t T = lpad / kGramTile;
    const int64_t tiles = T * (T + 1) / 2;
    int64_t max_split = n / (2 * kGramKT);
    if (max_split > 64) max_split = 64;
    if (max_split < 1) max_split = 1;
    if (tiles * max_split <= 512) return (int)max_split;
    int64_t best = 1;
    double best_eff = 0.0;
    for (int64_t s = 1; s <= max_split && (s == 1 || tiles * s <= 4 * 512); ++s) {
        const int64_t wg = tiles * s;
        const int64_t rounds = (wg + 511) / 512;
        const double eff = (double)wg / (double)(rounds * 512);
        if (eff > best_eff + 0.02) { best_eff = eff; best = s; }
    }
    return (int)best;
}

hipError_t launch_gram_dense(strads_lasso *h, int part)
{
    const int32_t T = h->Lpad / kGramTile;
    int32_t split = h->split_user > 0 ? h->split_user : gram_split_auto(h->cfg.n, h->Lpad);
    if (split > h->split_max) split = h->split_max;
    int64_t kchunk = (h->cfg.n + split - 1) / split;
    kchunk = ((kchunk + kGramKT - 1) / kGramKT) * kGramKT;
    split = (int32_t)((h->cfg.n + kchunk - 1) / kchunk);
    const size_t lds = 2 * 2 * kPanel * sizeof(float);
    float *P = h->at<float>(h->ws.partial);
    const dim3 grid((unsigned)(T * (T + 1) / 2 * split));
    if (part == 1) {
        RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
        hipLaunchKernelGGL(k_gram_mask, dim3((h->Lpad + 255) / 256, h->Lpad), dim3(256), 0, h->stream, P, split,
                           h->L, h->Lpad, h->cfg.rho, h->at<uint64_t>(h->ws.mask),
                           h->cfg.keep_gram ? h->at<float>(h->ws.gram) : nullptr, &sc->near_rho_pairs);
        return hipGetLastError();
    }
    if (h->vec4)
        hipLaunchKernelGGL(k_gram_tiles<true>, grid, dim3(256), lds, h->stream, h->cfg.x, h->cfg.n,
                           h->at<int32_t>(h->ws.cand), h->L, h->Lpad, T, split, kchunk, P);
    else
        hipLaunchKernelGGL(k_gram_tiles<false>, grid, dim3(256), lds, h->stream, h->cfg.x, h->cfg.n,
                           h->at<int32_t>(h->ws.cand), h->L, h->Lpad, T, split, kchunk, P);
    return hipGetLastError();
}

hipError_t launch_mask_from_gram(strads_lasso *h, const float *gram, int32_t l)
{
    hipLaunchKernelGGL(k_mask_from_gram, dim3((h->Lpad + 255) / 256, h->Lpad), dim3(256), 0, h->stream, gram, l,
                       h->Lpad, h->cfg.rho, h->at<uint64_t>(h->ws.mask));
    return hipGetLastError();
}

hipError_t gram_prepare()
{
    const int lds = 2 * 2 * kPanel * (int)sizeof(float);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_gram_tiles<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_gram_tiles<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

} // namespace strads
