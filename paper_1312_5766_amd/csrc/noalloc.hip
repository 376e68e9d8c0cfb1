// strads_lasso_filter_static: the dependency filter of Step 2 on a caller-supplied Gram, for callers that
// cannot allocate device memory (code under HIP graph capture, serving loops, harnesses that forbid it).
// Same kernels as strads_lasso_stage_filter; what that entry point keeps in the handle's workspace (the
// conflict bitmask, the column-id list the walk reads, the list it writes beside the positions, the
// round scalars) lives here in one file-scope device array.
//
// The array exists once per GPU, at its own address on each; the address is looked up once per device
// (first call on that device, with it current) and only that pointer is ever handed to a kernel.  Every
// call on a GPU uses the same array: calls that overlap on one GPU (two streams, two threads) race.
// Nothing in the array has to start at zero: the mask kernel writes every word of the rows the walk
// reads, the id list is rewritten for the call's length, and the walk writes its outputs before anyone
// reads them.
#include <mutex>

#include "strads_internal.h"

namespace strads {

constexpr int32_t kStaticMaxL = STRADS_FILTER_STATIC_MAX_L;
static_assert(kStaticMaxL % kGramTile == 0 && kStaticMaxL <= STRADS_MAX_L_PRIME, "static filter size");
constexpr size_t kOffMask = 0;                                                        // uint64 [lpad][lpad / 64]
constexpr size_t kOffIds = kOffMask + (size_t)kStaticMaxL * (kStaticMaxL / 64) * 8;   // int32 [l]: 0, 1, 2, ...
constexpr size_t kOffKept = kOffIds + (size_t)kStaticMaxL * 4;                        // int32 [l]: ids of the kept ones
constexpr size_t kOffScalars = kOffKept + (size_t)kStaticMaxL * 4;                    // RoundScalars
constexpr size_t kScratchBytes = kOffScalars + 1024;                                  // 8 MiB + 64 KiB + 1 KiB
static_assert(sizeof(RoundScalars) <= 1024, "scalars block");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static unsigned char *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each GPU, once looked up
static std::mutex g_scratch_mu;

// The array's address on the current device.  `scratch` itself is only a host-side handle of the symbol.
static int scratch_on_current_device(unsigned char **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return STRADS_E_HIP;
    if (dev < 0 || dev >= kMaxDevices) return STRADS_E_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return STRADS_E_HIP;
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *out = g_scratch_ptr[dev];
    return STRADS_OK;
}

__global__ __launch_bounds__(256) void k_iota(int32_t *__restrict__ ids, int32_t l)
{
    const int32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < l) ids[i] = i;
}

} // namespace strads

using namespace strads;

extern "C" int strads_lasso_filter_static(const float *gram, int32_t l, float rho, int32_t p_max, int32_t *kept_pos,
                                          int32_t *n_kept, void *stream)
{
    if (!gram || !kept_pos || !n_kept || l < 1 || p_max < 0 || !(rho > 0.f)) return STRADS_E_INVALID_ARG;
    if (l > kStaticMaxL) return STRADS_E_TOO_LARGE;
    unsigned char *base = nullptr;
    const int rc = scratch_on_current_device(&base);
    if (rc != STRADS_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    const int32_t lpad = (l + kGramTile - 1) / kGramTile * kGramTile;
    uint64_t *mask = reinterpret_cast<uint64_t *>(base + kOffMask);
    int32_t *ids = reinterpret_cast<int32_t *>(base + kOffIds);
    int32_t *kept = reinterpret_cast<int32_t *>(base + kOffKept);
    RoundScalars *sc = reinterpret_cast<RoundScalars *>(base + kOffScalars);
    hipLaunchKernelGGL(k_iota, dim3((l + 255) / 256), dim3(256), 0, s, ids, l);
    if (launch_status(s) != hipSuccess) return STRADS_E_HIP;
    if (launch_mask_from_gram_plain(s, gram, l, lpad, rho, mask) != hipSuccess) return STRADS_E_HIP;
    if (launch_filter_plain(s, mask, l, lpad, p_max, ids, kept_pos, kept, sc, n_kept) != hipSuccess) return STRADS_E_HIP;
    return STRADS_OK;
}
