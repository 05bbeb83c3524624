// Error string, version and device queries of libmole.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

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

namespace {
constexpr int MAX_DEVICES = 64;
std::atomic<int> g_arch_state[MAX_DEVICES];     // 0 = not checked, 1 = gfx950, 2 = another architecture

const char *const KNOB_NAMES[KNOB_COUNT] = {
    "MOLE_FWD_WPB", "MOLE_FWD_WGS_PER_CU", "MOLE_FWD_NTA", "MOLE_FWD_SPLIT", "MOLE_FWD_RUN",
    "MOLE_FWD_TILE", "MOLE_FWD_GENERIC", "MOLE_DEDUP_GENERIC", "MOLE_BUILD_HIDDEN", "MOLE_BUILD_SMALL_TILE",
    "MOLE_FFN_GATHER_LAST"};
std::atomic<int> g_knob[KNOB_COUNT];
std::once_flag g_knob_once;

void read_knobs_from_env()
{
    for (int k = 0; k < KNOB_COUNT; ++k) {
        const char *s = getenv(KNOB_NAMES[k]);
        int v = 0;
        if (s && *s) {
            if (k == KNOB_BUILD_HIDDEN && !strcmp(s, "f16"))
                v = 1;
            else if (k == KNOB_BUILD_HIDDEN && !strcmp(s, "split"))
                v = 2;
            else
                v = atoi(s);
        }
        g_knob[k].store(v > 0 ? v : 0, std::memory_order_relaxed);
    }
}
}  // namespace

mole_status check_arch(const char *who)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return fail(MOLE_EHIP, "%s: no current HIP device", who);
    const int slot = dev >= 0 && dev < MAX_DEVICES ? dev : -1;
    int state = slot >= 0 ? g_arch_state[slot].load(std::memory_order_relaxed) : 0;
    if (state == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return fail(MOLE_EHIP, "%s: hipGetDeviceProperties failed for device %d", who, dev);
        state = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
        if (slot >= 0)
            g_arch_state[slot].store(state, std::memory_order_relaxed);
        if (state == 2)
            return fail(MOLE_EUNSUPPORTED, "%s: device %d is %s; this library holds gfx950 (MI355X) code only", who,
                        dev, prop.gcnArchName);
    }
    if (state == 2)
        return fail(MOLE_EUNSUPPORTED, "%s: device %d is not a gfx950 (MI355X) part", who, dev);
    return MOLE_OK;
}

int knob(Knob k)
{
    std::call_once(g_knob_once, read_knobs_from_env);
    return g_knob[k].load(std::memory_order_relaxed);
}

}  // namespace mole

extern "C" mole_status mole_set_tuning(const char *name, int value)
{
    using namespace mole;
    clear_error();
    if (!name || value < 0)
        return fail(MOLE_EINVAL, "mole_set_tuning: name must not be NULL and value must be >= 0");
    std::call_once(g_knob_once, read_knobs_from_env);
    for (int k = 0; k < KNOB_COUNT; ++k) {
        if (!strcmp(name, KNOB_NAMES[k])) {
            g_knob[k].store(value, std::memory_order_relaxed);
            return MOLE_OK;
        }
    }
    return fail(MOLE_EINVAL, "mole_set_tuning: unknown knob \"%s\"", name);
}

extern "C" const char *mole_last_error(void) { return g_err; }
extern "C" int mole_version(void) { return 2; }
