// Device check, status strings and version of the gfx950 MX quantization library.
#include <string.h>

#include <atomic>

#include "mx_common.h"

namespace mx {

int check_device() {
    // per-device cache: 0 = unknown, 1 = gfx950, 2 = something else
    static std::atomic<int> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return MX_EUNSUPPORTED; }
    if (dev < 0 || dev >= 64) return MX_EUNSUPPORTED;
    int c = cache[dev].load(std::memory_order_relaxed);
    if (c == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return MX_EUNSUPPORTED; }
        c = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
        cache[dev].store(c, std::memory_order_relaxed);
    }
    return c == 1 ? MX_OK : MX_EUNSUPPORTED;
}

}  // namespace mx

extern "C" const char* mx_status_string(int status) {
    switch (status) {
        case MX_OK: return "ok";
        case MX_EINVAL: return "invalid argument (negative size, K not a multiple of 32, leading dimension too small, or bad enum)";
        case MX_ENULL: return "required pointer is NULL";
        case MX_EALIGN: return "pointer or leading dimension is misaligned";
        case MX_EUNSUPPORTED: return "no HIP device, the current device is not gfx950, or a shape or element format this entry point does not cover";
        case MX_ELAUNCH: return "the HIP runtime rejected the kernel launch";
        default: return "unknown status";
    }
}

extern "C" int mx_version(void) { return 200; }
