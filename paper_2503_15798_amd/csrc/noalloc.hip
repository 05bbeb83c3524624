// mole_lookup_forward_noalloc: the planned forward (mole_dedup_ids + mole_lookup_forward with
// MOLE_FLAG_DEDUP) for callers that cannot allocate device memory and therefore have no workspace to hand
// over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The plan, the
// distinct ids, the inverse map and the count live in a fixed array in device memory that belongs to the
// library (one copy per GPU, held until the process ends); the kernels are the ones of the two existing
// entry points and take the array's address as their workspace argument.
#include "mole_internal.h"

namespace {
using namespace mole;

constexpr int NOALLOC_MAX_T = MOLE_NOALLOC_MAX_T;       // largest batch the fixed array serves
constexpr int MAX_DEVICES = 64;

// words: plan of NOALLOC_MAX_T tokens | uniq [NOALLOC_MAX_T] | inv [NOALLOC_MAX_T] | n_uniq (+ padding)
constexpr size_t PLAN_WORDS = (size_t)PLAN_HEADER + 4 * (size_t)NOALLOC_MAX_T + 4 + 4;   // plan_layout, rounded up
constexpr size_t UNIQ_OFF = PLAN_WORDS;
constexpr size_t INV_OFF = UNIQ_OFF + NOALLOC_MAX_T;
constexpr size_t COUNT_OFF = INV_OFF + NOALLOC_MAX_T;
constexpr size_t SCRATCH_WORDS = COUNT_OFF + 4;         // 393 KiB in all

static __device__ __align__(256) int32_t scratch[SCRATCH_WORDS];

// Address of this GPU's copy of `scratch`, looked up once per device.  In host code the array's name is only
// a handle for hipGetSymbolAddress; every use of the memory goes through the pointer kept here.
std::atomic<int32_t *> g_scratch[MAX_DEVICES];

mole_status scratch_of_current_device(int32_t **out)
{
    int dev = 0;
    MOLE_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES)
        return fail(MOLE_EUNSUPPORTED, "mole_lookup_forward_noalloc: device index %d beyond %d", dev, MAX_DEVICES - 1);
    int32_t *p = g_scratch[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        MOLE_HIP_CHECK(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
        if (!sym)
            return fail(MOLE_EHIP, "mole_lookup_forward_noalloc: no device address for the scratch array");
        p = static_cast<int32_t *>(sym);
        g_scratch[dev].store(p, std::memory_order_release);     // every thread finds the same address
    }
    *out = p;
    return MOLE_OK;
}

}  // namespace

extern "C" mole_status mole_lookup_forward_noalloc(const void *table, const int32_t *ids, const void *h,
                                                   const void *W_r, const void *shared_out, const void *residual,
                                                   void *out, int32_t *err_flag, int T, int64_t V, int d, int N,
                                                   mole_dtype dtype, void *hip_stream)
{
    clear_error();
    if (T < 0)
        return fail(MOLE_EINVAL, "mole_lookup_forward_noalloc: T=%d is negative", T);
    if (T > NOALLOC_MAX_T)
        return fail(MOLE_EUNSUPPORTED,
                    "mole_lookup_forward_noalloc: T=%d exceeds the %d tokens the library's fixed scratch array serves "
                    "(use mole_dedup_ids + mole_lookup_forward with a workspace of your own)", T, NOALLOC_MAX_T);
    static_assert(PLAN_WORDS >= (size_t)PLAN_HEADER + 4 * (size_t)NOALLOC_MAX_T + 4 + 3, "plan of the largest batch fits");
    if (T == 0)
        return MOLE_OK;
    if (!table || !ids || !h || !W_r || !out)
        return fail(MOLE_EINVAL, "mole_lookup_forward_noalloc: table, ids, h, W_r and out must not be NULL");
    MOLE_ARCH_CHECK("mole_lookup_forward_noalloc");
    int32_t *base = nullptr;
    const mole_status ss = scratch_of_current_device(&base);
    if (ss != MOLE_OK)
        return ss;
    int32_t *plan = base;
    // Nothing in the array has to start at zero: the dedup kernel writes every word of the plan that the
    // forward reads (header, order, bucket starts) and clears its own counters, whatever the last call left.
    const mole_status ds = mole_dedup_ids(ids, T, V, base + UNIQ_OFF, base + INV_OFF, base + COUNT_OFF, err_flag, plan,
                                          PLAN_WORDS * sizeof(int32_t), hip_stream);
    if (ds != MOLE_OK)
        return ds;
    return mole_lookup_forward(table, ids, nullptr, h, W_r, shared_out, residual, out, nullptr, nullptr, err_flag, T, V,
                               d, N, dtype, MOLE_FLAG_DEDUP, plan, PLAN_WORDS * sizeof(int32_t), hip_stream);
}
