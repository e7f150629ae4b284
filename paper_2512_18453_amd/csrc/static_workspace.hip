// nova_winograd_conv2d_static: the convolution call for callers that cannot allocate or pass a
// workspace (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc).  V and M
// of a slab live in a fixed array in the library's device image instead of a caller buffer; the
// kernels are the ones nova_winograd_conv2d runs and take the array's address as their workspace.
#include <atomic>
#include <mutex>

#include "device_common.hpp"

namespace nova {

constexpr size_t kStaticWorkspaceBytes = (size_t)64 << 20;

// One copy per GPU, at that GPU's own address, held from the first use of the library's device code
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up once per device); a hipError_t as int.
static int static_workspace(void **out)
{
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_acquire);
        if (!p) {
            if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return (int)e;
            if (!p || ((uintptr_t)p & 255) != 0) return (int)hipErrorInvalidSymbol;
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return 0;
}

}  // namespace nova

extern "C" size_t nova_static_workspace_bytes(void) { return nova::kStaticWorkspaceBytes; }

extern "C" int nova_winograd_conv2d_static(const nova_transforms *t, const void *x, const void *U, void *y, int N,
                                           int C, int H, int W, int K, int dtype, int flags, void *stream)
{
    void *ws = nullptr;
    if (int err = nova::static_workspace(&ws)) {
        nova::set_last_hip_error(err);
        return NOVA_EHIP;
    }
    return nova::conv2d_with_workspace(t, x, U, y, N, C, H, W, K, dtype, flags, ws, nova::kStaticWorkspaceBytes,
                                       stream);
}
