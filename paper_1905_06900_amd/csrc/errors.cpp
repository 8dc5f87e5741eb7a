// Error reporting of the C ABI: a thread-local message behind dcpq_last_error().
#include <stdarg.h>
#include <stdio.h>

#include "dcpq.h"

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

}  // namespace dcpq

extern "C" const char *dcpq_last_error(void) { return dcpq::g_msg; }

extern "C" int dcpq_version(void) { return 1; }
