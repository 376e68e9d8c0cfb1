// Step 2 of SAP for the Lasso, second half (Algorithm 1: "choose a set B_1 of <= P coefficients
// from U such that |x_j^T x_k| < rho for all pairs"): walk the candidates in draw order and keep
// one iff it conflicts with nothing kept so far.
//
// The walk is inherently sequential in the kept set, so one wavefront does it, arranged so that
// the serial chain is short: candidates are taken 64 at a time.  `dead` (one bit per candidate,
// spread over the lanes' registers) marks candidates that conflict with something already kept.
// For a chunk, the 64x64 diagonal block of conflict bits decides the chunk with scalar bit
// operations (one lane-read per KEPT candidate); afterwards the conflict rows of the newly kept
// candidates are OR-ed into `dead` for the later chunks, 64 words per load, all lanes busy.
// Only bits (a, b) with b in a's 128-tile or right of it are read, matching what the Gram
// kernel writes.
#include "strads_internal.h"

namespace strads {

__device__ __forceinline__ uint64_t readlane64(uint64_t v, int l)
{
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}

constexpr int kDeadSlots = STRADS_MAX_L_PRIME / 64 / 64;   // mask words per lane (2)

__global__ __launch_bounds__(64) void k_filter(const uint64_t *__restrict__ mask, int32_t L, int32_t W,
                                               int32_t p_max, const int32_t *__restrict__ cand,
                                               int32_t *__restrict__ kept_pos, int32_t *__restrict__ kept,
                                               RoundScalars *__restrict__ sc, int count_updates)
{
    const int lane = threadIdx.x;
    uint64_t dead[kDeadSlots];
#pragma unroll
    for (int s = 0; s < kDeadSlots; ++s) dead[s] = 0;
    int32_t nk = 0;
    const int32_t cap = p_max > 0 ? p_max : L;
    const int32_t chunks = (L + 63) / 64;
    for (int32_t c = 0; c < chunks && nk < cap; ++c) {
        // word c of `dead` lives in slot c/64 of lane c%64
        uint64_t cur = 0;
#pragma unroll
        for (int s = 0; s < kDeadSlots; ++s)
            if (s == (c >> 6)) cur = readlane64(dead[s], c & 63);
        const int32_t a = c * 64 + lane;
        const uint64_t diag = a < L ? mask[(int64_t)a * W + c] : 0ull;
        const int32_t nvalid = L - c * 64;
        uint64_t alive = ~cur & (nvalid >= 64 ? ~0ull : ((1ull << nvalid) - 1ull));
        uint64_t keptw = 0;
        const int32_t nk0 = nk;
        while (alive != 0 && nk < cap) {            // uniform across the wavefront
            const int l = __ffsll((long long)alive) - 1;
            keptw |= 1ull << l;
            ++nk;
            alive &= ~(1ull << l);
            alive &= ~readlane64(diag, l);
        }
        if ((keptw >> lane) & 1ull) {
            const int32_t idx = nk0 + __popcll(keptw & ((1ull << lane) - 1ull));
            kept_pos[idx] = a;
            kept[idx] = cand[a];
        }
        // rows of the newly kept candidates kill later candidates
        uint64_t m = keptw;
        while (m != 0) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint64_t *row = mask + (int64_t)(c * 64 + l) * W;
#pragma unroll
            for (int s = 0; s < kDeadSlots; ++s) {
                const int32_t w = lane + 64 * s;
                if (w > c && w < W) dead[s] |= row[w];
            }
        }
    }
    if (lane == 0) { sc->n_kept = nk; if (count_updates) sc->updates_total += (unsigned long long)nk; }
}

hipError_t launch_filter(strads_lasso *h, int32_t l, bool count_updates)
{
    hipLaunchKernelGGL(k_filter, dim3(1), dim3(64), 0, h->stream, h->at<uint64_t>(h->ws.mask), l, h->Lpad / 64,
                       h->cfg.p_max, h->at<int32_t>(h->ws.cand), h->at<int32_t>(h->ws.kept_pos),
                       h->at<int32_t>(h->ws.kept), h->at<RoundScalars>(h->ws.scalars), count_updates ? 1 : 0);
    return hipGetLastError();
}

} // namespace strads
