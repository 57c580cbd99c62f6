// Status strings and cached device properties of libmoss_hip.so.
#include "moss_internal.h"

static int g_cu_count[64];

int moss_internal_cu_count()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (g_cu_count[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        g_cu_count[dev] = n;
    }
    return g_cu_count[dev];
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
