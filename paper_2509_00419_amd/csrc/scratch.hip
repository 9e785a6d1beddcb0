// The fixed scratch array of lvlm_decode_attn_static, in a translation unit (and so a device code object) of its
// own: the array is loaded onto a GPU only when that entry point is first used there, and tools that copy code
// objects as they are loaded (counter collection) never meet it in runs that do not use it.
#include <mutex>

#include "common.h"

namespace lvlm {

// A fixed device array takes the place of the caller's workspace in lvlm_decode_attn_static.  In host code the
// array's name is only a handle: its device address differs per GPU and is asked for once per device, with that
// device current, and kept; only that address is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[LVLM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char *g_scratch_ptr[kMaxDevices] = {};
}  // namespace

hipError_t attn_static_scratch(int device, char **ptr, size_t *bytes) {
    *ptr = nullptr;
    *bytes = LVLM_STATIC_SCRATCH_BYTES;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));     // the current device's copy
        if (e != hipSuccess) return e;
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<char *>(p);
    }
    *ptr = g_scratch_ptr[device];
    return hipSuccess;
}

}  // namespace lvlm
