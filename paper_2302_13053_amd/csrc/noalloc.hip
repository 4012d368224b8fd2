// retexo_aggregate for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc): the workspace of the
// aggregation — the per-node attention scores el / er that the edge-softmax table kernels
// read — lives in a file-scope device array of fixed size instead of a caller buffer.
//
// In host code the array's name is only a stand-in for the symbol; its device address is
// looked up once per device with hipGetSymbolAddress (each GPU holds its own copy at its
// own address) and that address is what the kernels receive, exactly as they receive the
// caller's workspace in retexo_aggregate.
#include <mutex>

#include "common.hpp"

namespace {

constexpr int64_t kScratchBytes = RETEXO_NOALLOC_SCRATCH_BYTES;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each device; NULL = not looked up yet

// The address of `scratch` on the current device, looked up on the first call there.
int scratch_on_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RETEXO_E_HIP;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RETEXO_E_HIP;
        if (((uintptr_t)p & 255) != 0) return RETEXO_E_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RETEXO_OK;
}

}  // namespace

extern "C" int retexo_aggregate_noalloc(const retexo_plan* plan, int mode, int64_t F, int heads,
                                        const float* d_Z, int64_t ldz,
                                        const float* d_attn_src, const float* d_attn_dst, float negative_slope,
                                        unsigned flags, float* d_out, int64_t ldo, void* stream)
{
    if (!plan) return RETEXO_E_NULL;
    // save mode hands its workspace on to the backward call: it needs a buffer the caller owns
    if (flags & RETEXO_F_SAVE) return RETEXO_E_FLAGS;
    if (F < 0 || F >= (1ll << 30)) return RETEXO_E_SIZE;
    if (mode < RETEXO_MEAN || mode > RETEXO_MAX) return RETEXO_E_MODE;
    if (heads < 1 || heads > kMaxHeads) return RETEXO_E_HEADS;
    const int64_t need = aggregate_workspace_bytes(plan->N, mode, heads, F, false);
    if (need > kScratchBytes) return RETEXO_E_WORKSPACE;
    void* ptr = nullptr;
    if (need > 0) {
        if (int s = scratch_on_current_device(&ptr)) return s;
    }
    // Nothing in the scratch has to start at zero: the score kernel writes every el / er entry
    // (padded heads included) of every node before the aggregation kernels of the same call read them.
    return retexo_aggregate(plan, mode, F, heads, d_Z, ldz, d_attn_src, d_attn_dst, negative_slope, flags,
                            d_out, ldo, ptr, need > 0 ? kScratchBytes : 0, stream);
}
