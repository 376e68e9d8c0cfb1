// Step 2 of SAP for the Lasso, first half (Section 2.1, Step 2; Algorithm 1's constraint on
// B_1): the dependencies d(x_a, x_b) = |x_a^T x_b| between the P' candidates, i.e. the Gram
// matrix of the gathered columns X_S, and from it one bit per pair: "conflict" iff NOT |g| < rho.
//
// This is a dense contraction (L' x N times N x L'), so it runs on the matrix cores:
// v_mfma_f32_32x32x2_f32, fp32 in, fp32 accumulate.  A workgroup of 4 wavefronts owns one
// 128 x 128 output tile of the upper triangle and one slice of the row (K) range.  Columns of X
// are contiguous along K, so operand panels are staged K-contiguous in LDS with coalesced 16-byte
// loads, double-buffered, and read back 16 bytes per lane: lane (i, h) of a wavefront reads
// k = 8*s + 4*h .. +3 of column i and feeds component c to the c-th of four MFMAs.  The MFMA
// sums over its two k-slots, and the assignment of k values to slots is the same for both
// operands, so any such assignment yields the same dot products.
//
//   * Off-diagonal tiles: each wavefront holds a 64 x 64 sub-tile as 2 x 2 MFMA accumulators.
//   * Diagonal tiles (both operands are the same 128 columns): only one panel is staged and only
//     the 10 of 16 32x32 blocks on or above the diagonal are computed -- wavefronts 0 and 3 take
//     the two 64 x 64 diagonal sub-tiles (3 blocks each), wavefronts 1 and 2 one row of two
//     blocks each of the off-diagonal sub-tile -- and blocks above the diagonal are also stored
//     mirrored, so the tile is complete in memory.  A diagonal tile costs 3/4 of an off-diagonal
//     one per K step, so it gets proportionally longer K slices (fewer of them).
//
// Accumulators live in the accumulation registers (AGPRs): loads returning into the ordinary
// vector registers then do not compete with the matrix pipe for register-file ports.
//
// K-slices are written as fp32 partial tiles and summed in fixed order by the mask kernel, so
// results do not depend on scheduling.
#include "strads_internal.h"
#include "dots.h"
#include <string.h>
#include <algorithm>
#include <type_traits>
#include <utility>
#include <vector>

namespace strads {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kPad = 4;                         // LDS row padding, floats
constexpr int kRow = kGramKT + kPad;            // LDS row stride, floats
constexpr int kPanel = kGramTile * kRow;        // floats per operand panel per stage
constexpr int kGramSlots = 256 * kGramOcc;      // resident workgroups on 256 compute units
constexpr int kKQ = kGramKT / 4;                // 16-byte pieces of one column per stage
constexpr int kColsPerPass = 256 / kKQ;         // columns the 256 threads stage in one pass
constexpr int kPasses = kGramTile / kColsPerPass;   // passes per 128-column panel

// D += A * B on the matrix core with the accumulator pinned to the AGPR file.
__device__ __forceinline__ void mfma32(floatx16 &acc, float a, float b)
{
    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// The compiler does not see inside the MFMA statements above, so it cannot count the cycles the
// last of them needs before its result may be read: wait them out (a 32x32x2 MFMA takes 16
// passes of 4 cycles).
__device__ __forceinline__ void mfma_drain()
{
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
}

// 4 consecutive K values of one column, zero beyond kend.  The address is clamped into the
// column and the value is selected.
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

// How the columns of X reach the kernel.
enum { kLoadScalar = 0, kLoadVec4 = 1, kLoadGeno2 = 2 };

// Packed genotype design: per-column mean and scale, words per column (see STRADS_LAYOUT_GENO2).
struct GenoCols {
    const float *mean, *scale;
    int64_t words;
};

// Staging of NPAN panels of 128 columns, one stage of kGramKT rows at a time: fetch() brings a
// stage from global memory into registers, stash() writes it K-contiguous into an LDS stage
// ([panel][128 rows of kRow floats]).
//   fp32 designs: a thread holds kPasses float4 per panel: column (it*kColsPerPass + tid/kKQ),
//     floats (tid%kKQ)*4..+3.
//   packed genotypes: a thread holds one 32-bit word (16 rows) per panel: column tid/2, rows
//     16*(tid%2)..+15 of the stage; stash() decodes it to fp32 as fl(fl(g - mean) * scale), both
//     operations rounded separately as the layout defines them.
// Columns past the candidate count are clamped to the last candidate: their products land in
// rows/columns >= L of the tile, which nobody reads.
template <int LOAD, int NPAN>
struct PanelLoader {
    int64_t kbeg, kend;
    // fp32
    const float *col[NPAN * kPasses];
    float4 R[NPAN * kPasses];
    int crow, kq;
    // packed genotypes
    const uint32_t *wp[NPAN];
    uint32_t W[NPAN];
    int valid[NPAN];
    float mean[NPAN], scale[NPAN];

    __device__ __forceinline__ void init(const float *__restrict__ X, int64_t N, const int32_t *__restrict__ cand,
                                         int32_t L, const int32_t (&tile)[NPAN], const GenoCols &gc, int64_t kb,
                                         int64_t ke)
    {
        kbeg = kb;
        kend = ke;
        const int tid = threadIdx.x;
        if (LOAD == kLoadGeno2) {
            static_assert(LOAD != kLoadGeno2 || kGramKT == 32, "the genotype loader stages 32 rows at a time");
            const uint32_t *Xw = reinterpret_cast<const uint32_t *>(X);
#pragma unroll
            for (int p = 0; p < NPAN; ++p) {
                int i = tile[p] * kGramTile + (tid >> 1);
                i = i < L ? i : L - 1;
                const int64_t j = cand[i];
                wp[p] = Xw + j * gc.words + kb / 16 + (tid & 1);
                mean[p] = gc.mean[j];
                scale[p] = gc.scale[j];
                W[p] = 0u;
                valid[p] = 0;
            }
        } else {
            crow = tid / kKQ;
            kq = (tid % kKQ) * 4;
#pragma unroll
            for (int p = 0; p < NPAN; ++p)
#pragma unroll
                for (int it = 0; it < kPasses; ++it) {
                    int i = tile[p] * kGramTile + it * kColsPerPass + crow;
                    i = i < L ? i : L - 1;
                    col[p * kPasses + it] = X + (int64_t)cand[i] * N;
                }
        }
    }

    // stages 0 .. nfull()-1 lie entirely inside the slice and can be fetched without clamping
    __device__ __forceinline__ int nfull() const
    {
        return LOAD == kLoadScalar ? 0 : (int)((kend - kbeg) / kGramKT);
    }

    __device__ __forceinline__ void fetch(int st)
    {
        if (LOAD == kLoadGeno2) {
            const int64_t row0 = kbeg + (int64_t)st * kGramKT + 16 * (threadIdx.x & 1);
            const int64_t left = kend - row0;                 // rows of this word inside the slice
            const int v = left >= 16 ? 16 : (left > 0 ? (int)left : 0);
#pragma unroll
            for (int p = 0; p < NPAN; ++p) {
                W[p] = v > 0 ? wp[p][2 * st] : 0u;            // a word that starts inside the column exists in full
                valid[p] = v;
            }
        } else {
            const int64_t k = kbeg + (int64_t)st * kGramKT + kq;
#pragma unroll
            for (int i = 0; i < NPAN * kPasses; ++i) R[i] = load_k4<LOAD == kLoadVec4>(col[i], k, kend);
        }
    }

    __device__ __forceinline__ void fetch_full(int st)
    {
        if (LOAD == kLoadGeno2) {
#pragma unroll
            for (int p = 0; p < NPAN; ++p) { W[p] = wp[p][2 * st]; valid[p] = 16; }
        } else {
            const int64_t k = kbeg + (int64_t)st * kGramKT + kq;
#pragma unroll
            for (int i = 0; i < NPAN * kPasses; ++i) R[i] = *reinterpret_cast<const float4 *>(col[i] + k);
        }
    }

    // packed genotypes: entries q, q+4, q+8, q+12 of a word are the four bytes of (word >> 2q) & 0x03030303
    template <bool FULL>
    __device__ __forceinline__ void stash_geno(float *stage) const
    {
        const int tid = threadIdx.x;
#pragma unroll
        for (int p = 0; p < NPAN; ++p) {
            float *dst = stage + p * kPanel + (tid >> 1) * kRow + 16 * (tid & 1);
            const float m = mean[p], sc = scale[p];
            float x[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t t = (W[p] >> (2 * q)) & 0x03030303u;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float g = (float)((t >> (8 * c)) & 0xFFu);
                    const float val = __fmul_rn(__fsub_rn(g, m), sc);
                    x[4 * c + q] = FULL || 4 * c + q < valid[p] ? val : 0.f;
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4 *>(dst + 4 * q) = make_float4(x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]);
        }
    }

    __device__ __forceinline__ void stash(float *stage) const
    {
        if (LOAD == kLoadGeno2) {
            stash_geno<false>(stage);
        } else {
#pragma unroll
            for (int p = 0; p < NPAN; ++p)
#pragma unroll
                for (int it = 0; it < kPasses; ++it)
                    *reinterpret_cast<float4 *>(stage + p * kPanel + (it * kColsPerPass + crow) * kRow + kq) =
                        R[p * kPasses + it];
        }
    }

    // a stage brought in by fetch_full(): no row of it lies past the slice
    __device__ __forceinline__ void stash_full(float *stage) const
    {
        if (LOAD == kLoadGeno2) stash_geno<true>(stage);
        else stash(stage);
    }
};

// store one 32x32 accumulator block: register v of lane (li, lh) holds row 8*(v/4) + 4*lh + (v%4),
// column li of the block
__device__ __forceinline__ void store_block(float *__restrict__ out, int32_t Lpad, int row0, int col0,
                                            const floatx16 &acc, int li, int lh)
{
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = row0 + 8 * (v >> 2) + 4 * lh + (v & 3);
        out[(int64_t)row * Lpad + col0 + li] = acc[v];
    }
}

// the same block written transposed: 4 consecutive registers are 4 consecutive columns of the
// transposed block, i.e. one 16-byte store
__device__ __forceinline__ void store_block_t(float *__restrict__ out, int32_t Lpad, int row0, int col0,
                                              const floatx16 &acc, int li, int lh)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float4 v4 = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
        *reinterpret_cast<float4 *>(out + (int64_t)(col0 + li) * Lpad + row0 + 8 * q + 4 * lh) = v4;
    }
}

// Off-diagonal tile (ta < tb).  Software pipeline per LDS stage st (32 K values): registers hold
// stage st+1 (fetched one stage ago), they are written to the other LDS buffer, the fetch of stage
// st+2 is issued, then stage st is multiplied out of LDS; one barrier per stage.
template <int LOAD>
__device__ __forceinline__ void gram_tile_off(const float *__restrict__ X, int64_t N,
                                              const int32_t *__restrict__ cand, const GramShape &g,
                                              const GenoCols &gc, int32_t ta, int32_t tb, int32_t s,
                                              float *__restrict__ P, float *smem)
{
    const int tid = threadIdx.x;
    const int64_t kbeg = (int64_t)s * g.kchunk_off;
    const int64_t kend = (kbeg + g.kchunk_off < N) ? kbeg + g.kchunk_off : N;
    const int nstage = (int)((kend - kbeg + kGramKT - 1) / kGramKT);

    PanelLoader<LOAD, 2> ld;
    const int32_t tiles[2] = {ta, tb};
    ld.init(X, N, cand, g.L, tiles, gc, kbeg, kend);
    auto fetch = [&](int st) { ld.fetch(st); };
    auto fetch_full = [&](int st) { ld.fetch_full(st); };
    auto stash = [&](int buf) { ld.stash(smem + buf * 2 * kPanel); };
    auto stash_full = [&](int buf) { ld.stash_full(smem + buf * 2 * kPanel); };
    const int nfull = ld.nfull();

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
    // Operands of one 8-row K step: lane (li, lh) reads k = 8*ks + 4*lh .. +3 of its two A columns
    // and two B columns.  The operands of step ks+1 are requested before the MFMAs of step ks are
    // issued, and those of a stage's first step before the stage's LDS writes and global loads, so
    // that LDS latency is never waited for with an empty matrix pipe.
    struct Ops { float4 a0, a1, b0, b1; };
    auto read_ops = [&](int buf, int ks) {
        const float *pa = smem + buf * 2 * kPanel + offa + ks * 8;
        const float *pb = smem + buf * 2 * kPanel + offb + ks * 8;
        Ops o;
        o.a0 = *reinterpret_cast<const float4 *>(pa);
        o.a1 = *reinterpret_cast<const float4 *>(pa + 32 * kRow);
        o.b0 = *reinterpret_cast<const float4 *>(pb);
        o.b1 = *reinterpret_cast<const float4 *>(pb + 32 * kRow);
        return o;
    };
    auto mma = [&](const Ops &o) {
        const float av0[4] = {o.a0.x, o.a0.y, o.a0.z, o.a0.w}, av1[4] = {o.a1.x, o.a1.y, o.a1.z, o.a1.w};
        const float bv0[4] = {o.b0.x, o.b0.y, o.b0.z, o.b0.w}, bv1[4] = {o.b1.x, o.b1.y, o.b1.z, o.b1.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            mfma32(acc[0][0], av0[c], bv0[c]);
            mfma32(acc[0][1], av0[c], bv1[c]);
            mfma32(acc[1][0], av1[c], bv0[c]);
            mfma32(acc[1][1], av1[c], bv1[c]);
        }
    };
    // One stage: multiply stage `buf` out of LDS.  Its first operands are in `cur` already; `between` runs
    // after the MFMAs of the first K step have been issued (the next stage's LDS writes and the global
    // loads of the stage after: whatever they wait for is then waited for behind a full matrix pipe).
    // The stage's one barrier sits before its LAST K step, not after it: by then every wavefront has
    // written its share of the next stage (and nobody reads that buffer any more: its last operands
    // were requested a step earlier), so the first operands of the next stage are requested right
    // after the barrier and arrive while the last step's 16 MFMAs run: neither the barrier nor the LDS
    // round trip after it is waited for with an empty matrix pipe.  `more`: another stage follows.
    auto stage = [&](int buf, Ops &cur, bool more, auto between) {
#pragma unroll
        for (int ks = 0; ks < kGramKT / 8; ++ks) {
            Ops next = cur;
            if (ks + 1 < kGramKT / 8) {
                next = read_ops(buf, ks + 1);
            } else if (more) {
                __syncthreads();
                next = read_ops(buf ^ 1, 0);
            }
            mma(cur);
            if (ks == 0) between();
            cur = next;
        }
    };

    fetch(0);
    stash(0);
    if (nstage > 1) fetch(1);
    __syncthreads();
    Ops cur = read_ops(0, 0);
    int st = 0;
    for (; st + 2 < nfull; ++st)                // steady state
        stage(st & 1, cur, true, [&] { stash_full((st + 1) & 1); fetch_full(st + 2); });
    for (; st + 2 < nstage; ++st)               // a ragged last stage is fetched with clamping
        stage(st & 1, cur, true, [&] { stash((st + 1) & 1); fetch(st + 2); });
    if (st + 1 < nstage) {
        stage(st & 1, cur, true, [&] { stash((st + 1) & 1); });
        ++st;
    }
    stage(st & 1, cur, false, [] {});
    mfma_drain();

    float *out = P + (int64_t)s * g.Lpad * g.Lpad;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
            store_block(out, g.Lpad, ta * kGramTile + wr * 64 + a * 32, tb * kGramTile + wc * 64 + b * 32,
                        acc[a][b], li, lh);
}

// Diagonal tile: one panel of 128 columns; 32-column groups p < q (< r) of this wavefront:
//   wavefront 0: (0,0) (0,1) (1,1)      wavefront 3: (2,2) (2,3) (3,3)
//   wavefront 1: (0,2) (0,3)            wavefront 2: (1,2) (1,3)
template <int LOAD>
__device__ __forceinline__ void gram_tile_diag(const float *__restrict__ X, int64_t N,
                                               const int32_t *__restrict__ cand, const GramShape &g,
                                               const GenoCols &gc, int32_t ta, int32_t s, float *__restrict__ P,
                                               float *smem)
{
    const int tid = threadIdx.x;
    const int64_t kbeg = (int64_t)s * g.kchunk_diag;
    const int64_t kend = (kbeg + g.kchunk_diag < N) ? kbeg + g.kchunk_diag : N;
    const int nstage = (int)((kend - kbeg + kGramKT - 1) / kGramKT);

    PanelLoader<LOAD, 1> ld;
    const int32_t tiles[1] = {ta};
    ld.init(X, N, cand, g.L, tiles, gc, kbeg, kend);
    auto fetch = [&](int st) { ld.fetch(st); };
    auto fetch_full = [&](int st) { ld.fetch_full(st); };
    auto stash = [&](int buf) { ld.stash(smem + buf * 2 * kPanel); };
    auto stash_full = [&](int buf) { ld.stash_full(smem + buf * 2 * kPanel); };
    const int nfull = ld.nfull();

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int li = lane & 31, lh = lane >> 5;
    const bool sym = wave == 0 || wave == 3;            // uniform per wavefront
    const int gp = wave == 0 ? 0 : wave == 3 ? 2 : wave - 1;    // 0, 0, 1, 2
    const int gq = wave == 0 ? 1 : wave == 3 ? 3 : 2;           // 1, 2, 2, 3
    const int gr = 3;                                           // rect wavefronts only

    floatx16 acc[3];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;

    const int offp = (gp * 32 + li) * kRow + lh * 4;
    const int offq = (gq * 32 + li) * kRow + lh * 4;
    const int offr = (gr * 32 + li) * kRow + lh * 4;
    // The whole pipeline once for the wavefronts with a symmetric share (SYM) and once for the others: the
    // two use the accumulators and operands differently, and a choice made inside the K loop would cost
    // register moves in every step.
    auto run = [&](auto symc) {
        constexpr bool SYM = decltype(symc)::value;
        // operands of one 8-row K step: 4 K values of this lane's column in groups p, q (and r)
        struct Ops { float4 p, q, r; };
        auto read_ops = [&](int buf, int ks) {
            const float *base = smem + buf * 2 * kPanel + ks * 8;
            Ops o;
            o.p = *reinterpret_cast<const float4 *>(base + offp);
            o.q = *reinterpret_cast<const float4 *>(base + offq);
            if (SYM) o.r = o.q;
            else o.r = *reinterpret_cast<const float4 *>(base + offr);
            return o;
        };
        auto mma = [&](const Ops &o) {
            const float pv[4] = {o.p.x, o.p.y, o.p.z, o.p.w}, qv[4] = {o.q.x, o.q.y, o.q.z, o.q.w};
            const float rv[4] = {o.r.x, o.r.y, o.r.z, o.r.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (SYM) {
                    mfma32(acc[0], pv[c], pv[c]);
                    mfma32(acc[1], pv[c], qv[c]);
                    mfma32(acc[2], qv[c], qv[c]);
                } else {
                    mfma32(acc[0], pv[c], qv[c]);
                    mfma32(acc[1], pv[c], rv[c]);
                }
            }
        };
        // one stage, as in gram_tile_off: operands one K step ahead, the stage's barrier before its last step
        auto stage = [&](int buf, Ops &cur, bool more, auto between) {
#pragma unroll
            for (int ks = 0; ks < kGramKT / 8; ++ks) {
                Ops next = cur;
                if (ks + 1 < kGramKT / 8) {
                    next = read_ops(buf, ks + 1);
                } else if (more) {
                    __syncthreads();
                    next = read_ops(buf ^ 1, 0);
                }
                mma(cur);
                if (ks == 0) between();
                cur = next;
            }
        };

        fetch(0);
        stash(0);
        if (nstage > 1) fetch(1);
        __syncthreads();
        Ops cur = read_ops(0, 0);
        int st = 0;
        for (; st + 2 < nfull; ++st)
            stage(st & 1, cur, true, [&] { stash_full((st + 1) & 1); fetch_full(st + 2); });
        for (; st + 2 < nstage; ++st)
            stage(st & 1, cur, true, [&] { stash((st + 1) & 1); fetch(st + 2); });
        if (st + 1 < nstage) {
            stage(st & 1, cur, true, [&] { stash((st + 1) & 1); });
            ++st;
        }
        stage(st & 1, cur, false, [] {});
        mfma_drain();
    };
    if (sym) run(std::true_type{});
    else run(std::false_type{});

    float *out = P + (int64_t)s * g.Lpad * g.Lpad;
    const int t0 = ta * kGramTile;
    if (sym) {
        store_block(out, g.Lpad, t0 + gp * 32, t0 + gp * 32, acc[0], li, lh);
        store_block(out, g.Lpad, t0 + gp * 32, t0 + gq * 32, acc[1], li, lh);
        store_block_t(out, g.Lpad, t0 + gp * 32, t0 + gq * 32, acc[1], li, lh);
        store_block(out, g.Lpad, t0 + gq * 32, t0 + gq * 32, acc[2], li, lh);
    } else {
        store_block(out, g.Lpad, t0 + gp * 32, t0 + gq * 32, acc[0], li, lh);
        store_block_t(out, g.Lpad, t0 + gp * 32, t0 + gq * 32, acc[0], li, lh);
        store_block(out, g.Lpad, t0 + gp * 32, t0 + gr * 32, acc[1], li, lh);
        store_block_t(out, g.Lpad, t0 + gp * 32, t0 + gr * 32, acc[1], li, lh);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Long candidate lists over 16-byte aligned fp32 columns: 256 x 256 output tiles.
//
// A global load instruction costs the matrix pipe the same however little it brings (measured: the 128 x 128
// kernel above takes 12 % less time when its loads are left out, whether they would have hit the L2 or not),
// and a 256 x 256 tile needs half as many of them per MFMA; they also write LDS themselves
// (global_load_lds_dwordx4), so that no data passes through the vector registers on its way there.  A workgroup
// of 8 wavefronts (two per SIMD, one workgroup per compute unit: two LDS stages of 512 columns take 128 KB)
// owns the tile; wavefront (wr, wc) holds rows 128 wr .. +127 and columns 64 wc .. +63 of it as 4 x 2 MFMA
// accumulators (128 AGPRs).
//
// Work is handed out from a queue.  One workgroup per compute unit and a few hundred tiles of 1500 stages
// do not divide evenly, and the eight XCDs of one chip do not run at the same speed (measured: up to 5 %
// between the slowest and the fastest under this load, differently from box to box), so equal shares would
// leave most of the chip waiting for its slowest part.  The (tile, stage range) items of the queue shrink as
// the queue empties -- whole tiles while more than a tile per workgroup is left, then a 256th of what is left,
// down to 32 stages -- and a workgroup that has finished an item takes the next with one atomic increment
// (guided self-scheduling).  An item is written to a tile slot of its own (256 x 256 floats); the slots of a
// tile are consecutive, in K order, and the mask kernel adds them in that order, so the sum does not depend
// on which workgroup computed what or when.  The queue is computed on the host when the handle is created.
//
// A tile on the diagonal stages its 256 columns once and multiplies only the 36 of its 64 32 x 32 blocks on or
// above the diagonal, dealt out to the wavefronts so that no SIMD gets more than 10 (an off-diagonal tile: 16);
// the queue's item sizes count a stage of a diagonal tile as 10/16 of a stage accordingly.  Blocks above the diagonal
// of a 128 x 128 diagonal square are also stored mirrored, as the mask kernel expects that square complete.
constexpr int kBigTile = 256;
constexpr int32_t kJobBlock = 8;                        // tiles per side of a block of jobs that share panels in one L2
constexpr int kBigThreads = 512;
constexpr int kBigLdsBytes = 2 * 2 * kBigTile * kGramKT * (int)sizeof(float);   // two stages of two 256-column panels
constexpr int kBigColsPerPass = kBigThreads / kKQ;      // columns the 512 threads stage in one pass
constexpr int kBigPasses = kBigTile / kBigColsPerPass;  // passes per panel
constexpr int kBigSlot = kBigTile * kBigTile;           // floats per tile slot
constexpr int kBigWorkgroups = 256;                     // one per compute unit
constexpr int kBigMinStages = 32;                       // shortest item of the queue

struct BigPiece {
    int32_t ta, tb;         // tile (256-column groups), ta <= tb
    int32_t sbeg, send;     // stages [sbeg, send) of kGramKT rows each
    int32_t slot;           // tile slot the item is written to
    int32_t pad_[3];
};

// 16 bytes per lane from global memory straight into LDS: lane l's piece lands at lds + 16 l (lds: the same for
// the whole wavefront).  Issued as an assembly statement that sets M0 (the LDS base) itself, with the waits
// placed by hand (dma_wait before the barrier that publishes the data); through the compiler's builtin for the
// same instruction the kernel was measured 2.7 % slower.
__device__ __forceinline__ void dma16(const float *g, const float *lds_uniform)
{
    const uint32_t l = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const float *)lds_uniform;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(l), "v"(g) : "memory", "m0");
}
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// One item of the queue: stages [sbeg, send) of tile (ta, tb), written to the item's tile slot.
// The panels come from global memory straight into LDS.  An LDS stage is [panel][256 columns][32 floats],
// unpadded (a wavefront's 64 pieces of one load instruction are 8 columns x 128 bytes in a row); the 16-byte quads
// of a column are stored permuted, quad q of column c at position q ^ (c & 7), so that the 32 lanes that read the
// same quad of 32 consecutive columns spread over all banks.  Two stages are in LDS (128 KB); a stage's loads are
// requested as early as its buffer is free, a whole stage before they are needed.
// BOTH, RIGHT: which of the wavefront's blocks are multiplied (see k_gram_tiles256); compile-time, because a
// choice made at run time around the MFMA statements makes the compiler copy accumulators between registers
// right behind them, and it does not know how long their results take.
// LATE: when the wavefront requests its share of the next data.  0: stage st+2 into the buffer of stage st right
// after stage st's barrier; otherwise stage st+1 into the other buffer behind the first MFMAs of stage st.  The
// two wavefronts of a SIMD differ in this, so that one of them feeds the matrix pipe while the other issues its
// loads (all at once: +2.5 %; a K step later than this: +0.3 %; two K steps later: +2.5 %, the data then arrive
// late for the barrier).
template <bool DIAG, uint32_t BOTH, uint32_t RIGHT, int LATE = 0>
__device__ __forceinline__ void gram_piece256(const float *__restrict__ X, int64_t N,
                                              const int32_t *__restrict__ cand, int32_t L, int32_t Lpad,
                                              const BigPiece pc, int ra, int cb, float *__restrict__ P, float *smem)
{
    constexpr int NPAN = DIAG ? 1 : 2;
    constexpr int NLD = NPAN * kBigPasses;
    constexpr int kRowD = kGramKT;                      // floats per column per stage, no padding
    constexpr int kPanelD = kBigTile * kRowD;
    constexpr int kStageD = NPAN * kPanelD;
    constexpr bool EARLY = LATE == 0;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t kbeg = (int64_t)pc.sbeg * kGramKT;
    const int64_t kend = (int64_t)pc.send * kGramKT < N ? (int64_t)pc.send * kGramKT : N;
    const int nstage = pc.send - pc.sbeg;
    const int nfull = (int)((kend - kbeg) / kGramKT);

    // staging: thread -> column (it * 64 + tid / 8) of each panel; it brings the quad that belongs at position
    // tid % 8 of that column
    const int crow = tid / kKQ, pq = tid % kKQ;
    const int kq = (pq ^ (crow & 7)) * 4;
    const float *col[NLD];
#pragma unroll
    for (int p = 0; p < NPAN; ++p)
#pragma unroll
        for (int it = 0; it < kBigPasses; ++it) {
            int i = (p == 0 ? pc.ta : pc.tb) * kBigTile + it * kBigColsPerPass + crow;
            i = i < L ? i : L - 1;
            col[p * kBigPasses + it] = X + (int64_t)cand[i] * N;
        }
    auto dma = [&](int st, int buf) {                   // a stage that lies entirely inside the item's rows
        const int64_t k = kbeg + (int64_t)st * kGramKT + kq;
#pragma unroll
        for (int p = 0; p < NPAN; ++p)
#pragma unroll
            for (int it = 0; it < kBigPasses; ++it)
                dma16(col[p * kBigPasses + it] + k,
                      smem + buf * kStageD + p * kPanelD + (it * kBigColsPerPass + wave * 8) * kRowD);
    };
    auto bring = [&](int st, int buf) {                 // any stage: a ragged one goes through registers
        if (st < nfull) { dma(st, buf); return; }
        const int64_t k = kbeg + (int64_t)st * kGramKT + kq;
        float4 R[NLD];
#pragma unroll
        for (int i = 0; i < NLD; ++i) R[i] = load_k4<true>(col[i], k, kend);
#pragma unroll
        for (int p = 0; p < NPAN; ++p)
#pragma unroll
            for (int it = 0; it < kBigPasses; ++it)
                *reinterpret_cast<float4 *>(smem + buf * kStageD + p * kPanelD +
                                            (it * kBigColsPerPass + crow) * kRowD + pq * 4) = R[p * kBigPasses + it];
    };

    const int lane = tid & 63;
    const int li = lane & 31, lh = lane >> 5;
    constexpr uint32_t both = BOTH, right = RIGHT;

    floatx16 acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // where lane (li, lh) finds k = 8 ks + 4 lh .. +3 of column (32 r + li): quad 2 ks + lh sits at position
    // (2 ks + lh) ^ (li & 7)
    int sw[kGramKT / 8];
#pragma unroll
    for (int ks = 0; ks < kGramKT / 8; ++ks) sw[ks] = ((2 * ks + lh) ^ (li & 7)) * 4;
    const int offa = (ra * 32 + li) * kRowD;
    const int offb = (DIAG ? 0 : kPanelD) + (cb * 32 + li) * kRowD;
    struct Ops { float4 a[4], b[2]; };
    auto read_a = [&](int buf, int ks, int a) {
        return *reinterpret_cast<const float4 *>(smem + buf * kStageD + offa + a * 32 * kRowD + sw[ks]);
    };
    auto read_b = [&](int buf, int ks, int b) {
        return *reinterpret_cast<const float4 *>(smem + buf * kStageD + offb + b * 32 * kRowD + sw[ks]);
    };
    auto mma_row = [&](int a, const float4 &av4, const float4 (&bv4)[2]) {
        const float av[4] = {av4.x, av4.y, av4.z, av4.w};
        const float b0[4] = {bv4[0].x, bv4[0].y, bv4[0].z, bv4[0].w}, b1[4] = {bv4[1].x, bv4[1].y, bv4[1].z, bv4[1].w};
        if (both >> a & 1u) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                mfma32(acc[a][0], av[c], b0[c]);
                mfma32(acc[a][1], av[c], b1[c]);
            }
        } else if (right >> a & 1u) {
#pragma unroll
            for (int c = 0; c < 4; ++c) mfma32(acc[a][1], av[c], b1[c]);
        }
    };
    // One stage.  Its barrier sits before its last K step; a wavefront arrives there with its own loads into
    // the next stage's buffer landed.  `between` runs behind the first eight MFMAs of the last K step (early
    // wavefronts: the barrier has just freed this stage's buffer) or of K step 1 (late ones).
    auto stage = [&](int buf, Ops &cur, bool more, auto between) {
#pragma unroll
        for (int ks = 0; ks < kGramKT / 8; ++ks) {
            const bool last = ks + 1 == kGramKT / 8;
            if (last && more) { dma_wait(); __syncthreads(); }
            const bool ahead = !last || more;
            const int nbuf = last ? buf ^ 1 : buf, nks = last ? 0 : ks + 1;
            float4 bn[2] = {cur.b[0], cur.b[1]};
            if (ahead) { bn[0] = read_b(nbuf, nks, 0); bn[1] = read_b(nbuf, nks, 1); }
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                mma_row(a, cur.a[a], cur.b);
                if (ahead) cur.a[a] = read_a(nbuf, nks, a);
                if (ks == (EARLY ? kGramKT / 8 - 1 : 0) && a == 0) between();
            }
            cur.b[0] = bn[0];
            cur.b[1] = bn[1];
        }
    };

    bring(0, 0);
    if (EARLY && nstage > 1) bring(1, 1);
    dma_wait();
    __syncthreads();
    Ops cur;
#pragma unroll
    for (int a = 0; a < 4; ++a) cur.a[a] = read_a(0, 0, a);
#pragma unroll
    for (int b = 0; b < 2; ++b) cur.b[b] = read_b(0, 0, b);
    int st = 0;
    for (; st + 2 < nfull; ++st)                // steady state
        stage(st & 1, cur, true, [&] { if (EARLY) dma(st + 2, st & 1); else dma(st + 1, (st & 1) ^ 1); });
    for (; st + 1 < nstage; ++st)               // the last stages: what is left to bring may be ragged or nothing
        stage(st & 1, cur, true, [&] {
            if (EARLY) { if (st + 2 < nstage) bring(st + 2, st & 1); }
            else bring(st + 1, (st & 1) ^ 1);
        });
    stage(st & 1, cur, false, [] {});
    mfma_drain();

    float *out = P + (int64_t)pc.slot * kBigSlot;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int rb = ra + a, cbk = cb + b;
            const bool mine = (both >> a & 1u) || (b == 1 && (right >> a & 1u));
            if (!mine || pc.ta * kBigTile + rb * 32 >= Lpad || pc.tb * kBigTile + cbk * 32 >= Lpad) continue;
            store_block(out, kBigTile, rb * 32, cbk * 32, acc[a][b], li, lh);
            if (DIAG && rb != cbk && rb / 4 == cbk / 4) store_block_t(out, kBigTile, rb * 32, cbk * 32, acc[a][b], li, lh);
        }
}

__global__ __launch_bounds__(kBigThreads, 1) void k_gram_tiles256(const float *__restrict__ X, int64_t N,
                                                                  const int32_t *__restrict__ cand, int32_t L,
                                                                  int32_t Lpad, const BigPiece *__restrict__ items,
                                                                  int32_t n_items, uint32_t *__restrict__ next,
                                                                  float *__restrict__ P)
{
    // [2 stages][A panel | B panel]; aligned for 16-byte LDS accesses whatever else the kernel keeps in LDS
    extern __shared__ __align__(16) float smem[];
    __shared__ uint32_t taken;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // every workgroup ends by drawing an index past the queue: the counter stops at n_items + gridDim.x and
    // the mask kernel, which runs next on the stream, puts it back to zero
    for (;;) {
        if (threadIdx.x == 0) taken = atomicAdd(next, 1u);
        __syncthreads();
        const uint32_t it = taken;              // uniform
        if (it >= (uint32_t)n_items) break;
        const BigPiece pc = items[it];
        // 32-column blocks of tile column tb that hold candidates: 8, fewer in the last tile column
        const int nbv = L - pc.tb * kBigTile >= kBigTile ? 8 : (L - pc.tb * kBigTile + 31) / 32;
        const bool half = nbv <= 4;
        if (pc.ta != pc.tb && nbv <= 2) {
            // 256 rows x 64 columns: wavefront w takes rows 32 w .. +31, two blocks
            gram_piece256<false, 0x1u, 0u>(X, N, cand, L, Lpad, pc, wave, 0, P, smem);
        } else if (pc.ta != pc.tb && !half) {
            // wavefront (wr, wc) = (wave / 4, wave % 4): rows 128 wr .. +127, columns 64 wc .. +63, all eight blocks
            // The two wavefronts of a SIMD (w and w + 4) stage at different K steps of a stage, so that one of them
            // feeds the matrix pipe while the other issues its LDS writes and global loads (-1.4 %).
            if (wave < 4) gram_piece256<false, 0xFu, 0u, 0>(X, N, cand, L, Lpad, pc, 0, wave * 2, P, smem);
            else gram_piece256<false, 0xFu, 0u, 2>(X, N, cand, L, Lpad, pc, 4, (wave & 3) * 2, P, smem);
        } else if (pc.ta != pc.tb) {
            // 256 rows x 128 columns: wavefront (wave / 2, wave % 2) takes rows 64 (wave / 2) .. +63 and columns
            // 64 (wave % 2) .. +63, four blocks each
            gram_piece256<false, 0x3u, 0u>(X, N, cand, L, Lpad, pc, (wave >> 1) * 2, (wave & 1) * 2, P, smem);
        } else if (half) {
            // the corner tile with at most 128 columns: one diagonal 128 x 128 square, 10 blocks (3 if 64 columns)
            if (wave == 3 && nbv > 2) gram_piece256<true, 0x7u, 0x8u>(X, N, cand, L, Lpad, pc, 0, 2, P, smem);
            else if (wave == 7) gram_piece256<true, 0x1u, 0x2u>(X, N, cand, L, Lpad, pc, 0, 0, P, smem);
            else gram_piece256<true, 0u, 0u>(X, N, cand, L, Lpad, pc, 0, 0, P, smem);
        } else {
            // On the diagonal only the 36 blocks with row block <= column block are needed; they are dealt out so
            // that the two wavefronts of a SIMD (w and w + 4) have 8, 8, 10 and 10 of them between them:
            //   w0 / w4: rows 0-3 x cols 6,7 (a = 0,1 / a = 2,3)      w1 / w5: rows 0-3 x cols 4,5 (a = 0,1 / a = 2,3)
            //   w2: rows 4-7 x cols 6,7 (7 blocks)   w6: rows 4-7 x cols 4,5 (3)
            //   w3: rows 0-3 x cols 2,3 (7 blocks)   w7: rows 0-3 x cols 0,1 (3)
            switch (wave) {
            case 0: gram_piece256<true, 0x3u, 0u>(X, N, cand, L, Lpad, pc, 0, 6, P, smem); break;
            case 1: gram_piece256<true, 0x3u, 0u>(X, N, cand, L, Lpad, pc, 0, 4, P, smem); break;
            case 4: gram_piece256<true, 0xCu, 0u>(X, N, cand, L, Lpad, pc, 0, 6, P, smem); break;
            case 5: gram_piece256<true, 0xCu, 0u>(X, N, cand, L, Lpad, pc, 0, 4, P, smem); break;
            case 2: gram_piece256<true, 0x7u, 0x8u>(X, N, cand, L, Lpad, pc, 4, 6, P, smem); break;
            case 3: gram_piece256<true, 0x7u, 0x8u>(X, N, cand, L, Lpad, pc, 0, 2, P, smem); break;
            case 6: gram_piece256<true, 0x1u, 0x2u>(X, N, cand, L, Lpad, pc, 4, 4, P, smem); break;
            default: gram_piece256<true, 0x1u, 0x2u>(X, N, cand, L, Lpad, pc, 0, 0, P, smem); break;
            }
        }
        __syncthreads();                        // the next item reuses the LDS stages, and `taken`
    }
}

// One job = one (tile, K-slice) pair.  Jobs are numbered with the off-diagonal tiles of the upper
// triangle first (K-slice fastest), then the diagonal tiles.
template <int LOAD>
__device__ __forceinline__ void gram_job(const float *__restrict__ X, int64_t N, const int32_t *__restrict__ cand,
                                         const GramShape &g, const GenoCols &gc, int32_t job, float *__restrict__ P,
                                         float *smem)
{
    const int32_t n_off = g.T * (g.T - 1) / 2 * g.split_off;
    if (job < n_off) {
        const int32_t s = job % g.split_off;
        int32_t u = job / g.split_off;          // index into the row-major strict upper triangle
        int32_t ta = 0;
        while (u >= g.T - 1 - ta) { u -= g.T - 1 - ta; ++ta; }
        gram_tile_off<LOAD>(X, N, cand, g, gc, ta, ta + 1 + u, s, P, smem);
    } else {
        const int32_t d = job - n_off;
        gram_tile_diag<LOAD>(X, N, cand, g, gc, d / g.split_diag, d % g.split_diag, P, smem);
    }
}

// Static dependencies: the decomposition is known on the host; the first n_jobs workgroups take one job
// each.  jobtab (may be NULL) says which, see gram_job_table.
//
// Workgroups past n_jobs (there are some when cd.L > 0; fp32 designs only) compute every candidate's
// x_j^T r and tentative update.  They are dispatched last, into the slots the tile jobs leave free
// while the last of them finish, they are bound by memory where the tiles are bound by the matrix
// cores, and they read columns the tiles have just pulled on chip: for a short candidate list this
// hides the whole pass, and the kernel that would otherwise make it after the filter is not needed.
template <int LOAD>
__global__ __launch_bounds__(256, kGramOcc) void k_gram_tiles(const float *__restrict__ X, int64_t N,
                                                       const int32_t *__restrict__ cand, GramShape g,
                                                       GenoCols gc, const int32_t *__restrict__ jobtab,
                                                       float *__restrict__ P, int32_t n_jobs, CandDots cd)
{
    extern __shared__ __align__(16) float smem[];             // [2 stages][A panel | B panel]
    if ((int32_t)blockIdx.x >= n_jobs) {
        if constexpr (LOAD != kLoadGeno2) {
            const int block = (int)blockIdx.x - n_jobs;
            if (cd.wide) cand_dots_block<256, LOAD == kLoadVec4>(X, N, cand, cd, block, smem);
            else cand_dots_block<64, LOAD == kLoadVec4>(X, N, cand, cd, block, smem);
        }
        return;
    }
    const int32_t job = jobtab ? jobtab[blockIdx.x] : (int32_t)blockIdx.x;
    gram_job<LOAD>(X, N, cand, g, gc, job, P, smem);
}

// ---------------------------------------------------------------------------------------------------------
// Short columns under a long candidate list (e.g. 2000 candidates over 500 rows): 64 x 64 tiles over the whole
// row range, conflict bits straight from the accumulators.
//
// With few rows there is little to split along K, and the 128 x 128 tiles of such a list are fewer than the
// chip's compute units: the K-slices that fill the chip then cost a partial tile per slice and a second kernel
// that sums them.  Here a workgroup of 4 wavefronts owns a 64 x 64 tile of the upper triangle (diagonal tiles in
// full) for all N rows, each wavefront one 32 x 32 block in a single MFMA accumulator (consecutive MFMAs into the
// same accumulator issue back to back), and writes the tile's conflict bits itself: a wavefront ballot over an
// accumulator register is 32 columns of two rows, i.e. two halves of 64-bit mask words.  The sums run over K
// in one order, so nothing depends on scheduling here either.  The staging, the operand reads one K step ahead
// and the place of the stage's barrier are those of the 128 x 128 kernel.
// (Measured at 2000 candidates over 500 rows, 528 tiles: 37 us, of which 8 us are launch, first fetch and the
// epilogue; with no loads, LDS traffic or barriers in the loop it is 31 us, because 528 equal workgroups leave some
// SIMDs three wavefronts to run where most have two.  The tile kernel with K-slices plus the sum of the slices
// takes 50 us there.)
constexpr int kDirTile = 64;
constexpr int kDirPanel = kDirTile * kRow;                      // floats per operand panel per stage
constexpr int kDirLdsBytes = 2 * 2 * kDirPanel * (int)sizeof(float);

// Staging of the two 64-column panels of a tile, one stage of kGramKT rows at a time (see PanelLoader).
//   fp32 designs: a thread holds two float4 per panel: column (it * 32 + tid / 8), floats (tid % 8) * 4 .. +3.
//   packed genotypes: threads 0..127 stage the first panel, the others the second; a thread holds one 32-bit
//     word (16 rows): column (tid % 128) / 2, rows 16 * (tid % 2) .. +15 of the stage.
template <int LOAD>
struct DirectLoader {
    int64_t kend;
    const float *col[4];
    float4 R[4];
    int crow, kq;
    const uint32_t *wp;
    uint32_t W;
    int valid, gpanel, gcol, ghalf;
    float mean, scale;

    __device__ __forceinline__ void init(const float *__restrict__ X, int64_t N, const int32_t *__restrict__ cand,
                                         int32_t L, int32_t ta, int32_t tb, const GenoCols &gc)
    {
        kend = N;
        const int tid = threadIdx.x;
        if (LOAD == kLoadGeno2) {
            gpanel = tid >> 7; gcol = (tid & 127) >> 1; ghalf = tid & 1;
            int i = (gpanel ? tb : ta) * kDirTile + gcol;
            i = i < L ? i : L - 1;
            const int64_t j = cand[i];
            wp = reinterpret_cast<const uint32_t *>(X) + j * gc.words + ghalf;
            mean = gc.mean[j];
            scale = gc.scale[j];
            W = 0u;
            valid = 0;
        } else {
            crow = tid >> 3;
            kq = (tid & 7) * 4;
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int it = 0; it < 2; ++it) {
                    int i = (p ? tb : ta) * kDirTile + it * 32 + crow;
                    i = i < L ? i : L - 1;
                    col[p * 2 + it] = X + (int64_t)cand[i] * N;
                }
        }
    }

    __device__ __forceinline__ void fetch(int st)
    {
        if (LOAD == kLoadGeno2) {
            const int64_t left = kend - ((int64_t)st * kGramKT + 16 * ghalf);     // rows of this word inside the column
            valid = left >= 16 ? 16 : (left > 0 ? (int)left : 0);
            W = valid > 0 ? wp[2 * st] : 0u;
        } else {
            const int64_t k = (int64_t)st * kGramKT + kq;
#pragma unroll
            for (int i = 0; i < 4; ++i) R[i] = load_k4<LOAD == kLoadVec4>(col[i], k, kend);
        }
    }

    __device__ __forceinline__ void stash(float *stage) const
    {
        if (LOAD == kLoadGeno2) {
            float *dst = stage + gpanel * kDirPanel + gcol * kRow + 16 * ghalf;
            float x[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {       // entries q, q+4, q+8, q+12 of a word are the bytes of (word >> 2q) & 0x03030303
                const uint32_t t = (W >> (2 * q)) & 0x03030303u;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float g = (float)((t >> (8 * c)) & 0xFFu);
                    const float val = __fmul_rn(__fsub_rn(g, mean), scale);
                    x[4 * c + q] = 4 * c + q < valid ? val : 0.f;
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4 *>(dst + 4 * q) = make_float4(x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]);
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int it = 0; it < 2; ++it)
                    *reinterpret_cast<float4 *>(stage + p * kDirPanel + (it * 32 + crow) * kRow + kq) = R[p * 2 + it];
        }
    }
};

// Workgroups past n_jobs take the candidates' x_j^T r, as in k_gram_tiles.
template <int LOAD>
__global__ __launch_bounds__(256) void k_gram_direct(const float *__restrict__ X, int64_t N,
                                                     const int32_t *__restrict__ cand, int32_t L, int32_t Lpad,
                                                     GenoCols gc, float rho, uint64_t *__restrict__ mask,
                                                     float *__restrict__ gram, int32_t *__restrict__ near_pairs,
                                                     int32_t n_jobs, CandDots cd)
{
    extern __shared__ __align__(16) float smem[];             // [2 stages][A panel | B panel]
    if ((int32_t)blockIdx.x >= n_jobs) {
        if constexpr (LOAD != kLoadGeno2) {
            const int block = (int)blockIdx.x - n_jobs;
            if (cd.wide) cand_dots_block<256, LOAD == kLoadVec4>(X, N, cand, cd, block, smem);
            else cand_dots_block<64, LOAD == kLoadVec4>(X, N, cand, cd, block, smem);
        }
        return;
    }
    // tile (ta, tb), ta <= tb, of the upper triangle in row-major order
    const int32_t T = Lpad / kDirTile;
    int32_t u = (int32_t)blockIdx.x, ta = 0;
    for (int32_t n = T; u >= n; --n) { u -= n; ++ta; }         // uniform
    const int32_t tb = ta + u;
    const int tid = threadIdx.x;
    const int nstage = (int)((N + kGramKT - 1) / kGramKT);

    DirectLoader<LOAD> ld;
    ld.init(X, N, cand, L, ta, tb, gc);

    const int wave = tid >> 6, lane = tid & 63;
    const int wr = wave >> 1, wc = wave & 1;    // 32 x 32 block of this wavefront
    const int li = lane & 31, lh = lane >> 5;
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const int offa = (wr * 32 + li) * kRow + lh * 4;
    const int offb = kDirPanel + (wc * 32 + li) * kRow + lh * 4;
    struct Ops { float4 a, b; };
    auto read_ops = [&](int buf, int ks) {
        Ops o;
        o.a = *reinterpret_cast<const float4 *>(smem + buf * 2 * kDirPanel + offa + ks * 8);
        o.b = *reinterpret_cast<const float4 *>(smem + buf * 2 * kDirPanel + offb + ks * 8);
        return o;
    };
    auto mma = [&](const Ops &o) {
        mfma32(acc, o.a.x, o.b.x);
        mfma32(acc, o.a.y, o.b.y);
        mfma32(acc, o.a.z, o.b.z);
        mfma32(acc, o.a.w, o.b.w);
    };
    auto stage = [&](int buf, Ops &cur, bool more, auto between) {
#pragma unroll
        for (int ks = 0; ks < kGramKT / 8; ++ks) {
            Ops next = cur;
            if (ks + 1 < kGramKT / 8) {
                next = read_ops(buf, ks + 1);
            } else if (more) {
                __syncthreads();
                next = read_ops(buf ^ 1, 0);
            }
            mma(cur);
            if (ks == 0) between();
            cur = next;
        }
    };
    ld.fetch(0);
    ld.stash(smem);
    if (nstage > 1) ld.fetch(1);
    __syncthreads();
    Ops cur = read_ops(0, 0);
    int st = 0;
    for (; st + 2 < nstage; ++st)
        stage(st & 1, cur, true, [&] { ld.stash(smem + ((st + 1) & 1) * 2 * kDirPanel); ld.fetch(st + 2); });
    if (st + 1 < nstage) {
        stage(st & 1, cur, true, [&] { ld.stash(smem + ((st + 1) & 1) * 2 * kDirPanel); });
        ++st;
    }
    stage(st & 1, cur, false, [] {});
    mfma_drain();

    // register v of lane (li, lh) holds row 8 * (v / 4) + 4 * lh + (v % 4), column li of the block: the ballot
    // over register v is columns 0..31 of row 8 * (v / 4) + (v % 4) in its low half and of the row 4 below in
    // its high half
    const int32_t row0 = ta * kDirTile + wr * 32, b = tb * kDirTile + wc * 32 + li;
    uint32_t *m32 = reinterpret_cast<uint32_t *>(mask);       // (little-endian halves of the 64-bit words)
    uint32_t n_near = 0;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int32_t a = row0 + 8 * (v >> 2) + 4 * lh + (v & 3);
        const bool live = a < L && b < L && a != b;
        const float ag = fabsf(acc[v]);
        const uint64_t bal = __ballot(live && !(ag < rho));
        if (near_pairs) n_near += (uint32_t)__popcll(__ballot(live && b > a && fabsf(ag - rho) <= 1e-6f));
        if (li == 0) m32[((int64_t)a * (Lpad / 64) + tb) * 2 + wc] = lh ? (uint32_t)(bal >> 32) : (uint32_t)bal;
    }
    if (near_pairs && n_near && lane == 0) atomicAdd(near_pairs, (int32_t)n_near);
    if (gram) {
        store_block(gram, Lpad, row0, tb * kDirTile + wc * 32, acc, li, lh);
        if (ta != tb) store_block_t(gram, Lpad, row0, tb * kDirTile + wc * 32, acc, li, lh);
    }
}

// Dynamic dependencies: the Gram of the movers only.  Their number is known on the device alone,
// so the launch has a fixed number of resident workgroups, which read the decomposition the mover
// kernel chose.  Each takes the job with its own number first; when there are more jobs than workgroups the
// rest are taken in order from a counter (`next`, zeroed by the mover kernel), because the XCDs of a chip do
// not run at the same speed and equal shares would wait for the slowest.
template <int LOAD>
__global__ __launch_bounds__(256, kGramOcc) void k_gram_tiles_dyn(const float *__restrict__ X, int64_t N,
                                                           const int32_t *__restrict__ mcand,
                                                           const GramShape *__restrict__ gdev, GenoCols gc,
                                                           float *__restrict__ P, uint32_t *__restrict__ next)
{
    extern __shared__ __align__(16) float smem[];
    __shared__ uint32_t taken;
    const GramShape g = *gdev;
    const int32_t total = g.T * (g.T - 1) / 2 * g.split_off + g.T * g.split_diag;
    int32_t job = blockIdx.x;
    while (job < total) {
        gram_job<LOAD>(X, N, mcand, g, gc, job, P, smem);
        if (total <= (int32_t)gridDim.x) break; // every job had a workgroup of its own
        if (threadIdx.x == 0) taken = atomicAdd(next, 1u);
        __syncthreads();                        // also: the next job reuses the LDS panels
        job = (int32_t)gridDim.x + (int32_t)taken;
        __syncthreads();                        // `taken` is written again after the next job
    }
}

// bit k of a 16-bit value -> bit 4k of the result
__device__ __forceinline__ uint64_t spread_every_4th(uint64_t x)
{
    x = (x | (x << 24)) & 0x000000FF000000FFull;
    x = (x | (x << 12)) & 0x000F000F000F000Full;
    x = (x | (x << 6)) & 0x0303030303030303ull;
    x = (x | (x << 3)) & 0x1111111111111111ull;
    return x;
}

// Sum the K-slices in slice order and emit the conflict bits (and, optionally, the fp32 Gram).
// A thread owns 4 consecutive columns b of one row a (16-byte loads of every slice), a wavefront
// 256 columns = four 64-bit mask words, assembled from one ballot per column-in-thread; only
// columns in the tiles at or right of a's diagonal tile exist.  gdev != NULL: the shape is read
// from device memory (dynamic dependencies) and the grid strides over it.
__global__ __launch_bounds__(256) void k_gram_mask(const float *__restrict__ P, GramShape gh,
                                                   const GramShape *__restrict__ gdev, float rho,
                                                   uint64_t *__restrict__ mask, float *__restrict__ gram,
                                                   int32_t *__restrict__ near_pairs)
{
    const GramShape g = gdev ? *gdev : gh;
    const int32_t L = g.L, Lpad = g.Lpad;
    const int64_t plane = (int64_t)Lpad * Lpad;
    const int lane = threadIdx.x & 63;
    for (int32_t a = blockIdx.y; a < Lpad; a += gridDim.y) {
        const int32_t first = (a / kGramTile) * kGramTile;  // first column of a's diagonal tile
        for (int32_t b0 = (blockIdx.x * 256 + (threadIdx.x & ~63)) * 4; b0 < Lpad; b0 += gridDim.x * 1024) {
            // b0: first column of this wavefront's 256; Lpad is a multiple of 128, so a wavefront is
            // either fully inside or half inside (its first 128 columns)
            if (b0 + 256 <= first) continue;                // uniform per wavefront
            const int32_t b = b0 + 4 * lane;
            const bool have = b >= first && b < Lpad;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (have) {
                const int32_t split = b < first + kGramTile ? g.split_diag : g.split_off;
                const float *p = P + (int64_t)a * Lpad + b;
                int32_t s = 0;
                for (; s + 7 < split; s += 8) {             // eight slices in flight, added in slice order
                    float4 q[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) q[u] = *reinterpret_cast<const float4 *>(p + (s + u) * plane);
#pragma unroll
                    for (int u = 0; u < 8; ++u) { v[0] += q[u].x; v[1] += q[u].y; v[2] += q[u].z; v[3] += q[u].w; }
                }
                for (; s < split; ++s) {
                    const float4 q = *reinterpret_cast<const float4 *>(p + s * plane);
                    v[0] += q.x; v[1] += q.y; v[2] += q.z; v[3] += q.w;
                }
            }
            uint64_t B[4];
            uint32_t n_near = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool live = have && a < L && b + c < L && a != b + c;
                const float ag = fabsf(v[c]);
                B[c] = __ballot(live && !(ag < rho));
                if (near_pairs) n_near += (uint32_t)__popcll(__ballot(live && b + c > a && fabsf(ag - rho) <= 1e-6f));
            }
            if (lane < 4) {
                const int32_t wb = b0 + 64 * lane;          // first column of mask word `lane` of this wavefront
                if (wb >= first && wb < Lpad) {
                    uint64_t w = 0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) w |= spread_every_4th((B[c] >> (16 * lane)) & 0xFFFFull) << c;
                    mask[(int64_t)a * (Lpad / 64) + (wb >> 6)] = w;
                }
            }
            if (near_pairs && n_near && lane == 0) atomicAdd(near_pairs, (int32_t)n_near);
            if (gram && have) {
                *reinterpret_cast<float4 *>(gram + (int64_t)a * Lpad + b) = make_float4(v[0], v[1], v[2], v[3]);
                if (b >= first + kGramTile) {               // mirror the tiles right of the diagonal
#pragma unroll
                    for (int c = 0; c < 4; ++c) gram[(int64_t)(b + c) * Lpad + a] = v[c];
                }
            }
        }
    }
}

// Rows per wavefront of k_gram_mask256 (measured at 8000 candidates, 470 MB of tile slots: 2 rows 80 us, 4 rows
// 86 us, 8 rows 106 us; one row per wavefront, with workgroups for the tiles left of the diagonal too, 212 us).
constexpr int kMaskRows = 2;
constexpr int kMaskGroups = kBigTile / (4 * kMaskRows);     // workgroups per tile

// Conflict bits (and, optionally, the fp32 Gram) from the tile slots the 256-wide tile kernel wrote.  A
// workgroup takes 4 * kMaskRows consecutive rows of one tile on or right of the diagonal (they are consecutive
// in every slot of the tile), a wavefront kMaskRows of them, a thread 4 consecutive columns of each; the
// slots are added in slot order, those of four slots and all the wavefront's rows in flight at once, and a row's
// four 64-bit mask words are assembled from one ballot per column-in-thread.  First slot and slot count of a
// tile are looked up in slots256 ([T2 * T2] first slots, then [T2 * T2] counts).  The kernel also puts the tile
// kernel's queue position back to zero for the next round, and marks the chunks of 64 rows that have a conflict
// bit in a word the greedy walk's row holders use (chunk_nz, see k_filter).
__global__ __launch_bounds__(256) void k_gram_mask256(const float *__restrict__ P, GramShape g, float rho,
                                                      uint64_t *__restrict__ mask, float *__restrict__ gram,
                                                      int32_t *__restrict__ near_pairs,
                                                      const int32_t *__restrict__ slots256, int32_t T2,
                                                      uint32_t *__restrict__ queue_next, uint32_t *__restrict__ chunk_nz)
{
    constexpr int R = kMaskRows;
    if (blockIdx.x == 0 && threadIdx.x == 0) *queue_next = 0u;
    // last tile row first (the tiles at the end of the queue are the ones cut into the most items): tile row
    // T2 - 1 has one tile on or right of the diagonal, tile row tr has T2 - tr
    int32_t u = (int32_t)blockIdx.x / kMaskGroups, tr = T2 - 1;
    for (int32_t n = 1; u >= n; ++n) { u -= n; --tr; }      // uniform
    const int32_t tc = tr + u;
    const int lane = threadIdx.x & 63;
    const int32_t a0 = tr * kBigTile + (((int32_t)blockIdx.x % kMaskGroups) * 4 + (int32_t)(threadIdx.x >> 6)) * R;
    const int32_t L = g.L, Lpad = g.Lpad;
    if (a0 >= Lpad) return;                                 // whole wavefronts: R divides 128, and so does Lpad's step
    const int32_t first = (a0 / kGramTile) * kGramTile;     // first column of these rows' 128-wide diagonal tile
    const int32_t b0 = tc * kBigTile, b = b0 + 4 * lane;
    const bool have = b >= first && b < Lpad;
    float4 v[R];
#pragma unroll
    for (int i = 0; i < R; ++i) v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (have) {
        const int32_t tile = tr * T2 + tc;
        const int32_t split = slots256[T2 * T2 + tile];
        const float *p = P + (int64_t)slots256[tile] * kBigSlot + (a0 % kBigTile) * kBigTile + 4 * lane;
        constexpr int64_t plane = kBigSlot;
        int32_t s = 0;
        for (; s + 3 < split; s += 4) {
            float4 q[4][R];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < R; ++i)
                    q[t][i] = *reinterpret_cast<const float4 *>(p + (s + t) * plane + i * kBigTile);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    v[i].x += q[t][i].x; v[i].y += q[t][i].y; v[i].z += q[t][i].z; v[i].w += q[t][i].w;
                }
        }
        for (; s < split; ++s) {
            float4 q[R];
#pragma unroll
            for (int i = 0; i < R; ++i) q[i] = *reinterpret_cast<const float4 *>(p + s * plane + i * kBigTile);
#pragma unroll
            for (int i = 0; i < R; ++i) { v[i].x += q[i].x; v[i].y += q[i].y; v[i].z += q[i].z; v[i].w += q[i].w; }
        }
    }
    uint32_t n_near = 0;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int32_t a = a0 + i;
        const float vc[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
        uint64_t B[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool live = have && a < L && b + c < L && a != b + c;
            const float ag = fabsf(vc[c]);
            B[c] = __ballot(live && !(ag < rho));
            if (near_pairs) n_near += (uint32_t)__popcll(__ballot(live && b + c > a && fabsf(ag - rho) <= 1e-6f));
        }
        if (lane < 4) {
            const int32_t wb = b0 + 64 * lane;              // first column of mask word `lane` of this row
            if (wb >= first && wb < Lpad) {
                uint64_t w = 0;
#pragma unroll
                for (int c = 0; c < 4; ++c) w |= spread_every_4th((B[c] >> (16 * lane)) & 0xFFFFull) << c;
                mask[(int64_t)a * (Lpad / 64) + (wb >> 6)] = w;
                // a word that the greedy walk's row holders use (see k_filter): mark the row's chunk of 64
                if (w != 0 && (wb >> 6) >= (a >> 6) + 2) chunk_nz[a >> 6] = 1u;
            }
        }
        if (gram && have) {
            *reinterpret_cast<float4 *>(gram + (int64_t)a * Lpad + b) = v[i];
            if (b >= first + kGramTile) {                   // mirror the tiles right of the diagonal
#pragma unroll
                for (int c = 0; c < 4; ++c) gram[(int64_t)(b + c) * Lpad + a] = vc[c];
            }
        }
    }
    if (near_pairs && n_near && lane == 0) atomicAdd(near_pairs, (int32_t)n_near);
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

// K-slices of a diagonal tile for a given off-diagonal slice count: the fewest slices whose
// cost (3/4 of an off-diagonal tile per K stage) exceeds an off-diagonal workgroup's by at most
// one stage.
__host__ __device__ static inline int diag_split_for(int64_t stages, int split_off)
{
    const int64_t off_len = (stages + split_off - 1) / split_off;
    int sd = 1;
    while (sd < split_off && 3 * ((stages + sd - 1) / sd) > 4 * (off_len + 1)) ++sd;
    return sd;
}

// Number of K-slices per off-diagonal tile.
// Workgroups = off-diagonal tiles x K-slices + diagonal tiles x their (fewer) K-slices.  Two
// workgroups are resident per compute unit (LDS), so the launch runs in rounds of kGramSlots.  The cost
// of a choice, in K stages of an off-diagonal workgroup: rounds x (stages per slice + a fixed
// prologue/epilogue allowance) + the partial-sum traffic it causes.
__host__ __device__ static inline int gram_split_choose(int64_t n, int32_t lpad)
{
    const int64_t T = lpad / kGramTile;
    const int64_t stages = (n + kGramKT - 1) / kGramKT;
    const int64_t n_off = T * (T - 1) / 2;
    if (T < 1) return 1;
    // at most 64 slices.  (More slices for one or two tiles were tried: at one tile and N = 50000 the tile
    // kernel goes from 60 us to 21-32 us with 160-200 workgroups, but the sum over the slices in the mask
    // kernel grows as fast, and at 261 workgroups both kernels take 105 us.)
    int64_t max_split = stages / 2;
    if (max_split > 64) max_split = 64;
    if (max_split < 1) max_split = 1;
    int best = 1;
    double best_cost = 1e300;
    for (int s = 1; s <= max_split; ++s) {
        const int sd = diag_split_for(stages, s);
        const int64_t wg = n_off * s + T * sd;
        const int64_t rounds = (wg + kGramSlots - 1) / kGramSlots;
        const int64_t len = (stages + s - 1) / s;
        // about 96 rows' worth of K per workgroup for first fetch and tile store; the partial tiles of
        // 512 workgroups (32 MiB written, then read by the mask kernel) cost about 64 rows' worth
        const double cost = (double)rounds * (double)(len + 96 / kGramKT) + (64.0 / kGramKT) * (double)wg / 512.0;
        if (cost < best_cost * 0.995) { best_cost = cost; best = s; }
    }
    return best;
}

int gram_split_auto(int64_t n, int32_t lpad) { return gram_split_choose(n, lpad); }

// L columns over N rows -> tiles, slices and slice lengths.  split_off_wanted = 0: automatic.
__host__ __device__ static inline GramShape gram_shape_for(int64_t n, int32_t L, int32_t split_off_wanted,
                                                           int32_t split_cap)
{
    GramShape g;
    g.L = L;
    g.Lpad = (L + kGramTile - 1) / kGramTile * kGramTile;
    g.T = g.Lpad / kGramTile;
    g.pad_ = 0;
    const int64_t stages = (n + kGramKT - 1) / kGramKT;
    int32_t so = split_off_wanted > 0 ? split_off_wanted : (g.T > 0 ? gram_split_choose(n, g.Lpad) : 1);
    if (so > split_cap) so = split_cap;
    if (so > stages) so = (int32_t)stages;
    if (so < 1) so = 1;
    const int64_t len = (stages + so - 1) / so;
    so = (int32_t)((stages + len - 1) / len);               // drop empty slices
    int32_t sd = diag_split_for(stages, so);
    const int64_t dlen = (stages + sd - 1) / sd;
    sd = (int32_t)((stages + dlen - 1) / dlen);
    g.split_off = so;
    g.split_diag = sd;
    g.kchunk_off = len * kGramKT;
    g.kchunk_diag = dlen * kGramKT;
    return g;
}

// The queue of the 256-wide route: the tiles of the upper triangle in blocks of 8 x 8 (neighbours in the queue
// share panels), each cut into equal items, shorter from tile to tile.  An item is at most a 256th (one
// workgroup's share) of the work that comes after its tile in the queue, measured in off-diagonal stages (a
// stage of a diagonal tile keeps the busiest SIMD busy for 10 MFMA blocks, of a tile in a last tile column of
// 128 columns for 8, of any other for 16), but at least kBigMinStages stages and at most the tile.  Slots are
// numbered in queue order, so a tile's items have consecutive slots in K order.
// first / count ([T2 * T2], may be NULL): first slot and number of slots of every tile.
static std::vector<BigPiece> gram256_queue(int64_t n, int32_t lpad, int32_t *first, int32_t *count)
{
    const int32_t T2 = (lpad + kBigTile - 1) / kBigTile;
    const int64_t S = (n + kGramKT - 1) / kGramKT;
    const bool half_last = T2 * kBigTile > lpad;
    auto weight = [&](int32_t ta, int32_t tb) {
        return ta == tb ? (int64_t)10 : (half_last && tb == T2 - 1 ? (int64_t)8 : (int64_t)16);
    };
    std::vector<BigPiece> tiles;
    int64_t left = 0;                                   // what is left of the job, in 16ths of an off-diagonal stage
    for (int32_t bi = 0; bi * kJobBlock < T2; ++bi)
        for (int32_t bj = bi; bj * kJobBlock < T2; ++bj)
            for (int32_t ta = bi * kJobBlock; ta < (bi + 1) * kJobBlock && ta < T2; ++ta)
                for (int32_t tb = bj * kJobBlock; tb < (bj + 1) * kJobBlock && tb < T2; ++tb)
                    if (ta <= tb) {
                        tiles.push_back(BigPiece{ta, tb, 0, 0, 0, {0, 0, 0}});
                        left += weight(ta, tb) * S;
                    }
    if (first) for (int32_t i = 0; i < T2 * T2; ++i) first[i] = count[i] = 0;
    std::vector<BigPiece> queue;
    for (const BigPiece &t : tiles) {
        const int64_t w = weight(t.ta, t.tb);
        if (first) first[t.ta * T2 + t.tb] = (int32_t)queue.size();
        // items of this tile: equal parts no longer than a 256th of what will be left after the tile
        int64_t len = (left - w * S) / kBigWorkgroups / w;
        if (len < kBigMinStages) len = kBigMinStages;
        const int64_t parts = (S + len - 1) / len;
        for (int64_t k = 0; k < parts; ++k) {
            const int64_t s0 = S * k / parts, s1 = S * (k + 1) / parts;
            queue.push_back(BigPiece{t.ta, t.tb, (int32_t)s0, (int32_t)s1, (int32_t)queue.size(), {0, 0, 0}});
            if (count) ++count[t.ta * T2 + t.tb];
        }
        left -= w * S;
    }
    return queue;
}

int32_t gram256_items(int64_t n, int32_t lpad) { return (int32_t)gram256_queue(n, lpad, nullptr, nullptr).size(); }

// Shapes that take the 256-wide route by default (fp32 columns, Algorithm 1's dependency rule; the caller
// checks the 16-byte alignment of X): lists longer than the short-list route serves, and shorter ones whose Gram
// gives every workgroup at least 180 stages' worth of work (measured: 4096 candidates over 50000 rows 6.0 ms
// against 6.4 ms with 128-wide tiles, 2048 candidates 1.63 against 1.71 ms; 4096 over 10000 rows a tie; below
// that the 128-wide kernel with its K-slices wins).
bool gram256_default(int64_t n, int32_t lpad, int32_t layout, int32_t deps)
{
    if (layout != STRADS_LAYOUT_DENSE_COLMAJOR || deps != STRADS_DEPS_STATIC || n < 4096 || n % 4 != 0) return false;
    if (lpad > kShortList) return true;
    const int64_t T2 = (lpad + kBigTile - 1) / kBigTile, S = (n + kGramKT - 1) / kGramKT;
    const int64_t work = (T2 * (T2 - 1) / 2 * 16 + T2 * 10) * S / 16;      // in stages of an off-diagonal tile
    return work >= (int64_t)180 * kBigWorkgroups;
}

// Where the 64 x 64 tiles that write the conflict bits themselves (k_gram_direct) are the default: columns short
// enough that a tile's whole row range is a short job, and a list long enough that such tiles fill the chip.
// (Measured, tiles + sum of the K-slices against this kernel, in us: 256 rows x 1024 candidates 22 / 13, x 4096
// 95 / 54; 500 x 1024 27 / 18, x 2000 50 / 36, x 4096 134 / 93; 1000 x 1024 35 / 29, x 1536 49 / 46, x 4096 217 / 172;
// 2000 x 1024 44 / 50, x 2000 113 / 117, x 3072 214 / 188, x 4096 362 / 324.)
bool gram_direct_default(int64_t n, int32_t lpad)
{
    const int64_t T = lpad / kDirTile;
    return (n <= 1024 && T >= 16) || (n <= 2048 && T >= 48);
}

// Bytes of the route's tables in the workspace: the queue, then first slot and slot count per tile.
size_t gram256_table_bytes(int64_t n, int32_t lpad)
{
    const size_t T2 = (size_t)((lpad + kBigTile - 1) / kBigTile);
    return sizeof(BigPiece) * (size_t)gram256_items(n, lpad) + 2 * sizeof(int32_t) * T2 * T2;
}

// Host image of those tables; returns the number of items.
int32_t gram256_tables(int64_t n, int32_t lpad, void *out)
{
    const int32_t T2 = (lpad + kBigTile - 1) / kBigTile;
    std::vector<int32_t> first((size_t)T2 * T2), count((size_t)T2 * T2);
    const std::vector<BigPiece> q = gram256_queue(n, lpad, first.data(), count.data());
    char *o = reinterpret_cast<char *>(out);
    memcpy(o, q.data(), sizeof(BigPiece) * q.size());
    memcpy(o + sizeof(BigPiece) * q.size(), first.data(), sizeof(int32_t) * first.size());
    memcpy(o + sizeof(BigPiece) * q.size() + sizeof(int32_t) * first.size(), count.data(), sizeof(int32_t) * count.size());
    return (int32_t)q.size();
}

// The queue as plain integers for the host-side plan call: items5[i] = (ta, tb, sbeg, send, slot).
int32_t gram256_plan_host(int64_t n, int32_t lpad, int32_t cap, int32_t *items5, int32_t *first, int32_t *count)
{
    const std::vector<BigPiece> q = gram256_queue(n, lpad, first, count);
    for (size_t i = 0; i < q.size() && i < (size_t)cap; ++i) {
        items5[5 * i + 0] = q[i].ta; items5[5 * i + 1] = q[i].tb; items5[5 * i + 2] = q[i].sbeg;
        items5[5 * i + 3] = q[i].send; items5[5 * i + 4] = q[i].slot;
    }
    return (int32_t)q.size();
}

size_t gram_partial_floats(int64_t n, int32_t lpad, bool dynamic)
{
    if (!dynamic) {
        size_t need = (size_t)gram_split_choose(n, lpad) * lpad * lpad;
        if (gram256_default(n, lpad, STRADS_LAYOUT_DENSE_COLMAJOR, STRADS_DEPS_STATIC)) {
            const size_t slots = (size_t)gram256_items(n, lpad) * kBigSlot;      // one tile slot per queue item
            if (slots > need) need = slots;
        }
        return need;
    }
    size_t most = 0;                                        // any mover count up to lpad
    for (int32_t l = kGramTile; l <= lpad; l += kGramTile) {
        const size_t need = (size_t)gram_split_choose(n, l) * l * l;
        if (need > most) most = need;
    }
    return most;
}

static GramShape gram_shape(const strads_lasso *h)
{
    return gram_shape_for(h->cfg.n, h->L, h->split_user, h->split_max);
}

// Which job the workgroup with a given blockIdx.x takes.  Workgroups are dealt to the chip's eight XCDs
// in turn (workgroup b runs on XCD b mod 8), each XCD has its own L2, and a job streams the rows of its
// K-slice of two 128-column panels (one for a diagonal tile).  What two jobs can share in an L2 is a panel
// they have in common, read at about the same time over the same rows.  So the jobs are put in an order in
// which neighbours share as much as possible, and every XCD gets a consecutive eighth of that order (the
// 64 workgroups it holds at a time are then neighbours):
//   * first by the first row of the job's K-slice: with many slices (a short candidate list) an XCD then
//     works on one or two slices of all tiles, and a panel row crosses the fabric once or twice, not eight times;
//   * within a slice by blocks of 8 x 8 tiles (block row, block column, then tile row, tile column; a
//     diagonal tile sits where its row and column meet): the 64 tiles of a block need 16 panels between
//     them, where 64 consecutive tiles of one tile row need 65.  What this buys is modest, because the
//     workgroups of an XCD do not stay in step over the thousands of stages of a long slice: for 8000
//     candidates over 50000 rows the L2 miss rate of the launch falls from 45 % to 36 % of requests, and the
//     kernel, which is bound by the matrix pipe, takes the same time.
size_t gram_job_table_entries(int64_t n, int32_t lpad)
{
    const size_t T = (size_t)(lpad / kGramTile);
    return (T * (T - 1) / 2 + T) * (size_t)gram_split_choose(n, lpad);      // any smaller slice count fits
}

int32_t gram_job_table(const strads_lasso *h, int32_t *out)
{
    const GramShape g = gram_shape(h);
    const int32_t n_off = g.T * (g.T - 1) / 2 * g.split_off;
    const int32_t total = n_off + g.T * g.split_diag;
    struct Key { int64_t kbeg; int32_t bi, bj, ta, tb, job; };
    std::vector<Key> order((size_t)total);
    {
        int32_t job = 0;
        for (int32_t ta = 0; ta < g.T; ++ta)                 // the numbering gram_job decodes
            for (int32_t tb = ta + 1; tb < g.T; ++tb)
                for (int32_t sl = 0; sl < g.split_off; ++sl, ++job)
                    order[(size_t)job] = Key{(int64_t)sl * g.kchunk_off, ta / kJobBlock, tb / kJobBlock, ta, tb, job};
        for (int32_t ta = 0; ta < g.T; ++ta)
            for (int32_t sl = 0; sl < g.split_diag; ++sl, ++job)
                order[(size_t)job] = Key{(int64_t)sl * g.kchunk_diag, ta / kJobBlock, ta / kJobBlock, ta, ta, job};
    }
    std::sort(order.begin(), order.end(), [](const Key &a, const Key &b) {
        if (a.kbeg != b.kbeg) return a.kbeg < b.kbeg;
        if (a.bi != b.bi) return a.bi < b.bi;
        if (a.bj != b.bj) return a.bj < b.bj;
        if (a.ta != b.ta) return a.ta < b.ta;
        if (a.tb != b.tb) return a.tb < b.tb;
        return a.job < b.job;
    });
    const int32_t kXcds = 8, base = total / kXcds, rem = total % kXcds;
    for (int32_t b = 0; b < total; ++b) {
        const int32_t x = b % kXcds, q = b / kXcds;
        const int32_t first = x * base + (x < rem ? x : rem);               // jobs of the XCDs before x
        out[b] = order[(size_t)(first + q)].job;
    }
    return total;
}

// Dynamic dependencies: list the movers (candidates whose tentative change is not zero) in draw
// order and look up the decomposition of their Gram.  One workgroup of 1024 threads walks the
// candidate positions 1024 at a time (coalesced reads, wavefront ballots for the ordered offsets).
__global__ __launch_bounds__(1024) void k_movers(const float *__restrict__ dc, const int32_t *__restrict__ cand,
                                                 int32_t L, const GramShape *__restrict__ table, int32_t lpad_fixed,
                                                 int32_t *__restrict__ mpos, int32_t *__restrict__ mcand,
                                                 RoundScalars *__restrict__ sc, GramShape *__restrict__ gout)
{
    __shared__ uint32_t wtot[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t base = 0;
    for (int32_t a0 = 0; a0 < L; a0 += 1024) {          // 1024 positions at a time, in order
        const int32_t a = a0 + tid;
        const bool mv = a < L && dc[a] != 0.f;
        const int32_t j = mv ? cand[a] : 0;
        const uint64_t m = __ballot(mv);
        if (lane == 0) wtot[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) { const uint32_t v = wtot[w]; if (w < wave) before += v; total += v; }
        if (mv) {
            const uint32_t idx = base + before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            mpos[idx] = a;
            mcand[idx] = j;
        }
        base += total;
        __syncthreads();                                // wtot is reused by the next pass
    }
    if (tid == 0) {
        // dense designs: the decomposition depends on the mover count only through the number of
        // tiles, and the host tabulated it per tile count when the handle was created.  CSC designs
        // have no tiles: only the count is needed, the conflict rows keep the full row width.
        GramShape g;
        if (table) {
            g = table[(base + kGramTile - 1) / kGramTile];
        } else {
            g.Lpad = lpad_fixed; g.T = lpad_fixed / kGramTile; g.split_off = g.split_diag = 1; g.pad_ = 0;
            g.kchunk_off = g.kchunk_diag = 0;
        }
        g.L = (int32_t)base;
        sc->n_movers = (int32_t)base;
        sc->gram_next = 0u;                     // the mover Gram's job counter (k_gram_tiles_dyn)
        *gout = g;
    }
}

void gram_shape_table(int64_t n, int32_t lpad, GramShape *out)
{
    for (int32_t t = 0; t <= lpad / kGramTile; ++t) out[t] = gram_shape_for(n, t * kGramTile, 0, 64);
}

hipError_t launch_movers(strads_lasso *h)
{
    const bool tiled = h->cfg.layout != STRADS_LAYOUT_CSC;      // dense and packed designs share the tile kernel
    hipLaunchKernelGGL(k_movers, dim3(1), dim3(1024), 0, h->stream, h->at<float>(h->ws.dc),
                       h->at<int32_t>(h->ws.cand), h->L, tiled ? h->at<GramShape>(h->ws.dtable) : nullptr,
                       tiled ? 0 : h->Lpad, h->at<int32_t>(h->ws.mpos),
                       h->at<int32_t>(h->ws.mcand), h->at<RoundScalars>(h->ws.scalars),
                       h->at<GramShape>(h->ws.dshape));
    return launch_status(h->stream);
}

// L x L image (row-major) of the mover Gram for parity checks: x_a^T x_b where both candidate
// positions a and b are movers, 0 elsewhere.
__global__ __launch_bounds__(256) void k_scatter_mover_gram(const float *__restrict__ gram,
                                                            const GramShape *__restrict__ gdev,
                                                            const int32_t *__restrict__ mpos, int32_t L,
                                                            float *__restrict__ out)
{
    const int32_t m = gdev->L, Lpad = gdev->Lpad;
    for (int32_t i = blockIdx.y; i < m; i += gridDim.y)
        for (int32_t k = blockIdx.x * 256 + threadIdx.x; k < m; k += gridDim.x * 256)
            out[(int64_t)mpos[i] * L + mpos[k]] = gram[(int64_t)i * Lpad + k];
}

hipError_t launch_scatter_mover_gram(strads_lasso *h, float *out)
{
    hipError_t e = hipMemsetAsync(out, 0, (size_t)h->L * h->L * 4, h->stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_scatter_mover_gram, dim3(4, 1024), dim3(256), 0, h->stream, h->at<float>(h->ws.gram),
                       h->at<GramShape>(h->ws.dshape), h->at<int32_t>(h->ws.mpos), h->L, out);
    return launch_status(h->stream);
}

hipError_t launch_gram_dense(strads_lasso *h, int part)
{
    const bool dynamic = h->cfg.deps == STRADS_DEPS_DYNAMIC;
    const GramShape g = gram_shape(h);
    const GramShape *gdev = dynamic ? h->at<GramShape>(h->ws.dshape) : nullptr;
    const size_t lds = 2 * 2 * kPanel * sizeof(float);
    float *P = h->at<float>(h->ws.partial);
    const bool big = !dynamic && h->big_items > 0;          // 256-wide tiles (see k_gram_tiles256)
    const BigPiece *items = reinterpret_cast<const BigPiece *>(h->base + h->ws.big_tables);
    RoundScalars *sc = h->at<RoundScalars>(h->ws.scalars);
    const bool direct = !dynamic && gram_direct_on(h);      // 64 x 64 tiles straight to conflict bits (see k_gram_direct)
    if (part == 1) {
        float *gram = h->cfg.keep_gram ? h->at<float>(h->ws.gram) : nullptr;
        if (direct) return hipSuccess;                      // the tile kernel has written the mask
        if (big) {
            const int32_t T2 = (h->Lpad + kBigTile - 1) / kBigTile;
            hipLaunchKernelGGL(k_gram_mask256, dim3((unsigned)(T2 * (T2 + 1) / 2 * kMaskGroups)), dim3(256), 0, h->stream, P, g,
                               h->cfg.rho, h->at<uint64_t>(h->ws.mask), gram, &sc->near_rho_pairs,
                               reinterpret_cast<const int32_t *>(items + h->big_items), T2, &sc->gram_next, sc->chunk_nz);
            return launch_status(h->stream);
        }
        dim3 grid((h->Lpad + 1023) / 1024, h->Lpad);       // 1024 columns of one row per workgroup
        if (dynamic) { if (grid.x > 2) grid.x = 2; if (grid.y > 2048) grid.y = 2048; }
        hipLaunchKernelGGL(k_gram_mask, grid, dim3(256), 0, h->stream, P, g, gdev, h->cfg.rho,
                           h->at<uint64_t>(h->ws.mask), gram, &sc->near_rho_pairs);
        return launch_status(h->stream);
    }
    if (big) {
        const unsigned wgs = h->big_items < kBigWorkgroups ? (unsigned)h->big_items : (unsigned)kBigWorkgroups;
        hipLaunchKernelGGL(k_gram_tiles256, dim3(wgs), dim3(kBigThreads), kBigLdsBytes, h->stream,
                           h->cfg.x, h->cfg.n, h->at<int32_t>(h->ws.cand), h->L, h->Lpad, items, h->big_items,
                           &sc->gram_next, P);
        return launch_status(h->stream);
    }
    const int load = h->cfg.layout == STRADS_LAYOUT_GENO2 ? kLoadGeno2 : (h->vec4 ? kLoadVec4 : kLoadScalar);
    GenoCols gc;
    gc.mean = h->cfg.col_mean;
    gc.scale = h->cfg.col_scale;
    gc.words = geno_words(h->cfg.n);
    if (dynamic) {
        const int32_t *mcand = h->at<int32_t>(h->ws.mcand);
#define STRADS_GRAM_DYN(LD) hipLaunchKernelGGL(k_gram_tiles_dyn<LD>, dim3(kGramSlots), dim3(256), lds, h->stream, h->cfg.x, h->cfg.n, mcand, gdev, gc, P, &sc->gram_next)
        if (load == kLoadGeno2) STRADS_GRAM_DYN(kLoadGeno2);
        else if (load == kLoadVec4) STRADS_GRAM_DYN(kLoadVec4);
        else STRADS_GRAM_DYN(kLoadScalar);
#undef STRADS_GRAM_DYN
        return launch_status(h->stream);
    }
    CandDots cd = {};
    unsigned extra = 0;
    if (dots_ride_with_gram(h)) {
        cd = cand_dots_args(h);
        extra = cd.wide ? (unsigned)cd.L : (unsigned)((cd.L + 3) / 4);
    }
    if (direct) {
        const int32_t T = h->Lpad / kDirTile, n_tiles = T * (T + 1) / 2;
        float *gram = h->cfg.keep_gram ? h->at<float>(h->ws.gram) : nullptr;
#define STRADS_GRAM_DIRECT(LD) hipLaunchKernelGGL(k_gram_direct<LD>, dim3((unsigned)n_tiles + extra), dim3(256), kDirLdsBytes, h->stream, h->cfg.x, h->cfg.n, h->at<int32_t>(h->ws.cand), h->L, h->Lpad, gc, h->cfg.rho, h->at<uint64_t>(h->ws.mask), gram, &sc->near_rho_pairs, n_tiles, cd)
        if (load == kLoadGeno2) STRADS_GRAM_DIRECT(kLoadGeno2);
        else if (load == kLoadVec4) STRADS_GRAM_DIRECT(kLoadVec4);
        else STRADS_GRAM_DIRECT(kLoadScalar);
#undef STRADS_GRAM_DIRECT
        return launch_status(h->stream);
    }
    const int32_t n_jobs = g.T * (g.T - 1) / 2 * g.split_off + g.T * g.split_diag;
    const dim3 grid((unsigned)n_jobs + extra);
    const int32_t *jobtab = h->jobtab_on ? reinterpret_cast<const int32_t *>(h->base + h->ws.jobtab) : nullptr;
#define STRADS_GRAM(LD) hipLaunchKernelGGL(k_gram_tiles<LD>, grid, dim3(256), lds, h->stream, h->cfg.x, h->cfg.n, h->at<int32_t>(h->ws.cand), g, gc, jobtab, P, n_jobs, cd)
    if (load == kLoadGeno2) STRADS_GRAM(kLoadGeno2);
    else if (load == kLoadVec4) STRADS_GRAM(kLoadVec4);
    else STRADS_GRAM(kLoadScalar);
#undef STRADS_GRAM
    return launch_status(h->stream);
}

hipError_t launch_mask_from_gram_plain(hipStream_t stream, const float *gram, int32_t l, int32_t lpad, float rho,
                                       uint64_t *mask)
{
    hipLaunchKernelGGL(k_mask_from_gram, dim3((lpad + 255) / 256, lpad), dim3(256), 0, stream, gram, l, lpad, rho, mask);
    return launch_status(stream);
}

hipError_t launch_mask_from_gram(strads_lasso *h, const float *gram, int32_t l)
{
    return launch_mask_from_gram_plain(h->stream, gram, l, h->Lpad, h->cfg.rho, h->at<uint64_t>(h->ws.mask));
}

hipError_t gram_prepare()
{
    const int lds = 2 * 2 * kPanel * (int)sizeof(float);
    const void *kernels[] = {reinterpret_cast<const void *>(k_gram_tiles<kLoadScalar>),
                             reinterpret_cast<const void *>(k_gram_tiles<kLoadVec4>),
                             reinterpret_cast<const void *>(k_gram_tiles<kLoadGeno2>),
                             reinterpret_cast<const void *>(k_gram_tiles_dyn<kLoadScalar>),
                             reinterpret_cast<const void *>(k_gram_tiles_dyn<kLoadVec4>),
                             reinterpret_cast<const void *>(k_gram_tiles_dyn<kLoadGeno2>)};
    for (const void *k : kernels) {
        const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_gram_tiles256),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);
}

} // namespace strads
