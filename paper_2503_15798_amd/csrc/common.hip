// Error string, version and device queries of libmole.
#include <stdarg.h>
#include <stdio.h>

#include "mole_internal.h"

namespace {
thread_local char g_err[512] = "";
}

namespace mole {

mole_status fail(mole_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

void clear_error() { g_err[0] = '\0'; }

int num_cus()
{
    static std::atomic<int> cached{0};
    if (cached.load(std::memory_order_relaxed) > 0)
        return cached.load(std::memory_order_relaxed);
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        return 256;   // MI355X; not cached, so a later call can still learn the real count
    cached.store(n, std::memory_order_relaxed);
    return n;
}

}  // namespace mole

extern "C" const char *mole_last_error(void) { return g_err; }
extern "C" int mole_version(void) { return 1; }
