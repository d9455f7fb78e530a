// topk_refine_static: the second round's final selection (topk_refine of sams.h) for callers that cannot
// allocate device memory -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
// It needs no context: the scratch the selection kernels use (positions among the candidates, radix histogram,
// selection state, per-tile counts and prefixes) lives in a file-scope __device__ array that every GPU the
// library runs on holds until the process ends.  The kernels are the ones topk_refine launches; they receive the
// array's device address as an ordinary argument.
#include <mutex>

#include "sams_ctx.h"

namespace sams {

constexpr int64_t kStaticMaxCand = SAMS_STATIC_MAX_CANDIDATES;
constexpr int64_t kStaticTiles = (kStaticMaxCand + kSelTile - 1) / kSelTile;
constexpr int kStaticMaxDevices = 64;

// layout of the scratch, in bytes from its start (every part 256-byte aligned)
constexpr size_t kOffPos = 0;                                                   // int32 [kStaticMaxCand]
constexpr size_t kOffHist = kOffPos + (size_t)kStaticMaxCand * 4;               // uint32 [kHistBins]
constexpr size_t kOffCnt = kOffHist + (size_t)kHistBins * 4;                    // uint32 [2][kStaticTiles]
constexpr size_t kOffBase = kOffCnt + (size_t)2 * kStaticTiles * 4;             // uint32 [2][kStaticTiles]
constexpr size_t kOffSel = kOffBase + (size_t)2 * kStaticTiles * 4;             // SelState
constexpr size_t kStaticBytes = kOffSel + 256;
static_assert(kOffHist % 256 == 0 && kOffCnt % 256 == 0 && kOffBase % 256 == 0 && kOffSel % 256 == 0, "alignment");
static_assert(sizeof(SelState) <= 256, "selection state");

// In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

static std::mutex g_static_mutex;
static void *g_static_ptr[kStaticMaxDevices];       // device address of `scratch` on each device, once resolved

// Device address of the scratch on the current device (resolved once per device, with that device current).
int static_scratch_ptr(void **out)
{
    int dev = -1;
    SAMS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices) return SAMS_EINVAL;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        SAMS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return SAMS_EHIP;
        g_static_ptr[dev] = p;
    }
    *out = g_static_ptr[dev];
    return SAMS_OK;
}

}  // namespace sams

using namespace sams;

extern "C" {

int64_t topk_refine_static_max_candidates(void) { return kStaticMaxCand; }

int topk_refine_static(const int32_t *idx_in, const float *delta_in, int64_t k_in, int64_t k_out, int32_t *idx_out,
                       float *delta_out, void *hip_stream)
{
    if (!idx_in || !delta_in || !idx_out || !delta_out) return SAMS_EINVAL;
    if (k_in < 1 || k_in > kStaticMaxCand || k_out < 1 || k_out > k_in) return SAMS_EINVAL;
    if (!aligned16(idx_in) || !aligned16(delta_in) || !aligned16(idx_out) || !aligned16(delta_out)) return SAMS_EINVAL;
    void *p = nullptr;
    SAMS_TRY(static_scratch_ptr(&p));
    unsigned char *b = static_cast<unsigned char *>(p);
    const SelScratch sc = {reinterpret_cast<uint32_t *>(b + kOffHist), reinterpret_cast<SelState *>(b + kOffSel),
                           reinterpret_cast<uint32_t *>(b + kOffCnt), reinterpret_cast<uint32_t *>(b + kOffBase),
                           kStaticTiles};
    // Nothing here needs clearing by the host: the selection's first kernel resets the histogram and the state, the
    // counts and prefixes are written for every tile of this call before they are read, and only the first k_out
    // positions are read back.
    return enqueue_refine(nullptr, (hipStream_t)hip_stream, sc, reinterpret_cast<int32_t *>(b + kOffPos), idx_in,
                          delta_in, k_in, k_out, idx_out, delta_out);
}

}  // extern "C"
