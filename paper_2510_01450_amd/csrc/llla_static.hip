// llla_decode_static: the decode call for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid it) and so have no workspace to pass.  The partial-moment records that
// llla_decode keeps in the caller's workspace live here in a file-scope device array of fixed size instead; the
// kernels are the very same ones.
//
// One copy of the array exists on every GPU the library is loaded on, at an address of its own.  In host code the
// array's name is only a handle for the runtime, not a device address: the address is looked up once per device with
// hipGetSymbolAddress, kept, and passed to the kernels exactly as llla_decode passes its workspace pointer.
#include <mutex>

#include "llla_common.hpp"

namespace {

constexpr size_t kScratchBytes = LLLA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each GPU, once looked up

// Device address of this GPU's copy of the array (nullptr if the runtime cannot say).
void *scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> hold(g_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" llla_status llla_decode_static(const void *q, const void *Kc, const void *Vc, void *o, llla_strides sk,
                                          llla_strides sv, const int32_t *seqlens, int B, int H, int L_max, int d,
                                          llla_dtype in, llla_dtype out, float lambda, float scale, void *stream)
{
    // what llla_decode would ask of a workspace for this call (0 for shapes the vector kernels serve, and for bad
    // shapes, which the call below then refuses with their own status)
    const size_t need = llla_decode_workspace_bytes(B, H, L_max, d, in);
    if (need > kScratchBytes) return LLLA_ERR_WORKSPACE;
    void *ptr = nullptr;
    if (need > 0) {
        ptr = scratch_on_current_device();
        if (ptr == nullptr) return LLLA_ERR_LAUNCH;
    }
    // nothing in the records has to start at zero: every record a call reads is written by that call first
    return llla_decode(q, Kc, Vc, o, sk, sv, seqlens, B, H, L_max, d, in, out, lambda, scale, ptr, need ? kScratchBytes : 0,
                       stream);
}
