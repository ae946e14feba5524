// The forward for callers that cannot allocate: the scratch that essa_svdlora_forward takes from the context's growable
// buffer lives here in a fixed array in device memory, one copy per GPU, held until the process ends.
#include <mutex>

#include "essa_internal.h"

// The array's name is a host-side stand-in, not a device address: host code never passes it anywhere.  Its address on
// a GPU comes from hipGetSymbolAddress with that GPU current, once per GPU, and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[ESSA_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices];      // per device, null until first use there

essa_status scratch_for_device(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return essa_fail(ESSA_ERR_UNSUPPORTED, "essa_svdlora_forward_noalloc: device %d beyond %d", device, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        ESSA_HIP(hipSetDevice(device));
        ESSA_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return essa_fail(ESSA_ERR_HIP, "essa_svdlora_forward_noalloc: the scratch array has no address on device %d", device);
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return ESSA_OK;
}
}  // namespace

extern "C" essa_status essa_svdlora_forward_noalloc(essa_ctx* ctx, const essa_proj* proj, const void* X, int x_dtype, int R,
                                                    const int32_t* row2cand, const float* sigmaA, const float* sigmaB,
                                                    int64_t sigma_stride, int K, void* Y, int y_dtype, uint32_t flags) {
    if (!ctx) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_svdlora_forward_noalloc: ctx is NULL");
    ESSA_HIP(hipSetDevice(ctx->device));
    void* ws = nullptr;
    ESSA_TRY(scratch_for_device(ctx->device, &ws));
    essa_fwd_item it{proj, X, row2cand, sigmaA, sigmaB, Y, sigma_stride, R, K};
    return essa_forward_on_scratch(ctx, &it, x_dtype, y_dtype, flags, ws, (size_t)ESSA_NOALLOC_SCRATCH_BYTES, "essa_svdlora_forward_noalloc");
}
