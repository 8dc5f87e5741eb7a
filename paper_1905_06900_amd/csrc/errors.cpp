// Error reporting of the C ABI: a thread-local message behind dcpq_last_error().
#include <stdarg.h>
#include <stdio.h>

#include <map>
#include <mutex>
#include <utility>

#include "common.h"

namespace dcpq {

static thread_local char g_msg[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_msg, sizeof g_msg, fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_msg[0] = '\0'; }

int allow_dynamic_lds(const void *kernel, int bytes, bool no_static_lds)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void *>, int> done;      // (device, kernel) -> bytes allowed so far
    int dev = 0;
    DCPQ_CHECK_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    const auto key = std::make_pair(dev, kernel);
    const auto it = done.find(key);
    if (it != done.end() && it->second >= bytes) return DCPQ_OK;
    if (no_static_lds) {
        hipFuncAttributes fa;
        DCPQ_CHECK_HIP(hipFuncGetAttributes(&fa, kernel));
        if (fa.sharedSizeBytes != 0)
            return fail(DCPQ_EUNSUPPORTED, "kernel has %zu bytes of static LDS, expected none",
                        static_cast<size_t>(fa.sharedSizeBytes));
    }
    DCPQ_CHECK_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    done[key] = bytes;
    return DCPQ_OK;
}

}  // namespace dcpq

extern "C" const char *dcpq_last_error(void) { return dcpq::g_msg; }

extern "C" int dcpq_version(void) { return 2; }
