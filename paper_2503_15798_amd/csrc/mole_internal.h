// Internal helpers shared by libmole's translation units (not part of the ABI).
#ifndef MOLE_INTERNAL_H
#define MOLE_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "mole.h"

namespace mole {

// Records a printf-style message for mole_last_error() and returns `st`.
mole_status fail(mole_status st, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_bytes(mole_dtype dt) { return dt == MOLE_F32 ? 4 : (dt == MOLE_U8 ? 1 : 2); }

// Number of compute units of the current device (cached per process; 256 on MI355X).
int num_cus();

// MOLE_OK if the current device is a gfx950 part (the only code object in the library); MOLE_EUNSUPPORTED
// with a message otherwise.  Checked once per process and device, before the first launch of an entry point.
mole_status check_arch(const char *who);

// Tuning knobs (experiments and tests; normal use needs none).  Each is read from the environment variable of
// the same name ONCE, at its first use in the process; mole_set_tuning() overrides it at run time.
// 0 = the library's own choice.
enum Knob {
    KNOB_FWD_WPB,           // MOLE_FWD_WPB          waves per workgroup of the forward kernels: 4 or 8
    KNOB_FWD_WGS_PER_CU,    // MOLE_FWD_WGS_PER_CU   resident workgroups per CU the grid is sized for
    KNOB_FWD_NTA,           // MOLE_FWD_NTA          1 = non-temporal activation loads, 2 = plain
    KNOB_FWD_SPLIT,         // MOLE_FWD_SPLIT        1 = one 512-column chunk per work item, 2 = whole tokens
    KNOB_FWD_RUN,           // MOLE_FWD_RUN          1 / 2 = force / forbid the run kernel for planned calls
    KNOB_FWD_TILE,          // MOLE_FWD_TILE         1 / 2 = force / forbid the tile kernel (N = 32)
    KNOB_FWD_GENERIC,       // MOLE_FWD_GENERIC      1 = the generic forward kernel for every shape
    KNOB_DEDUP_GENERIC,     // MOLE_DEDUP_GENERIC    1 = the generic dedup kernel for every size, 2 = never the split kernel
    KNOB_BUILD_HIDDEN,      // MOLE_BUILD_HIDDEN     1 (or "f16") / 2 (or "split"): hidden activation of the build
    KNOB_BUILD_SMALL_TILE,  // MOLE_BUILD_SMALL_TILE 1 = the 256 x 128 GEMM for every shape
    KNOB_FFN_GATHER_LAST,   // MOLE_FFN_GATHER_LAST  1 = shared-FFN call: every workgroup gathers behind its main loop
    KNOB_COUNT
};
int knob(Knob k);
inline int knob_or(Knob k, int dflt)
{
    const int v = knob(k);
    return v > 0 ? v : dflt;
}

// Raises a kernel's dynamic-LDS limit to `lds` bytes unless a call has already raised it that far.  `seen`
// is the per-kernel cache (a function-local static): callers on several threads may race to set the same
// attribute, which is harmless, but must not tear the cached size.
inline hipError_t ensure_dynamic_lds(std::atomic<size_t> &seen, const void *kernel, size_t lds)
{
    if (lds <= seen.load(std::memory_order_relaxed))
        return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) {
        size_t cur = seen.load(std::memory_order_relaxed);
        while (cur < lds && !seen.compare_exchange_weak(cur, lds, std::memory_order_relaxed)) {
        }
    }
    return e;
}

#define MOLE_ARCH_CHECK(who)                          \
    do {                                              \
        const mole_status st_ = ::mole::check_arch(who); \
        if (st_ != MOLE_OK)                           \
            return st_;                               \
    } while (0)

#define MOLE_HIP_CHECK(expr)                                                             \
    do {                                                                                 \
        hipError_t e_ = (expr);                                                          \
        if (e_ != hipSuccess)                                                            \
            return ::mole::fail(MOLE_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// ---- plan written by mole_dedup_ids and read by the forward kernels ----
// int32 words: header[16] | uniq[T] | order[T] | start[T+2] | counters[T+2]
// header: [0] n_uniq  [1] reserved  [2] T  [3] reserved  [4] V  [5] magic
// order: the token indices sorted by id (out-of-range ids last); bit 31 of an entry is set when
//        the token's id occurs only once in the batch (its rows will not be read again).
// start[u]: position in `order` of the first token of distinct id u (start[U] = out-of-range
//        tokens, start[U+1] = T).
constexpr int PLAN_HEADER = 16;
constexpr int PLAN_MAGIC = 0x4d4f4c45;   // "MOLE"
constexpr uint32_t PLAN_SINGLE = 0x80000000u;
struct PlanLayout {
    int64_t uniq, order, start, counters, words;
};
__host__ __device__ inline PlanLayout plan_layout(int T)
{
    PlanLayout p;
    p.uniq = PLAN_HEADER;
    p.order = p.uniq + T;
    p.start = p.order + T;
    p.counters = p.start + T + 2;
    p.words = p.counters + T + 2;
    p.words = (p.words + 3) & ~int64_t(3);
    return p;
}

// ---- bf16 <-> fp32 on the device ----
__device__ __forceinline__ float bf16lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }
// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return 0x7fc0u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

}  // namespace mole
#endif
