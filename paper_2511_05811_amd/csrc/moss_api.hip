// Status strings and cached device properties of libmoss_hip.so.
#include <atomic>

#include "moss_internal.h"

static std::atomic<int> g_cu_count[64];   // per device, 0 = not asked yet; racing first calls store the same value

int moss_internal_cu_count()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int n = g_cu_count[dev].load();
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        g_cu_count[dev].store(n);
    }
    return n;
}

extern "C" int moss_device_cu_count(void) { return moss_internal_cu_count(); }

extern "C" const char *moss_status_string(int status)
{
    switch (status) {
        case MOSS_OK: return "ok";
        case MOSS_ERR_NULL: return "a required pointer is NULL";
        case MOSS_ERR_SHAPE: return "bad shape (non-positive, not a multiple of the group size, or too large)";
        case MOSS_ERR_ALIGN: return "pointer or leading dimension not aligned";
        case MOSS_ERR_WORKSPACE: return "workspace missing or too small";
        case MOSS_ERR_UNSUPPORTED: return "unsupported flag or dtype combination";
        case MOSS_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}
