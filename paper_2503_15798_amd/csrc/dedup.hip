// mole_dedup_ids: distinct token ids of a batch (ascending), the inverse map, and a grouping
// plan for the forward kernels.
//
// The paper's lookup (inference listing, the lut(input_ids) line) simply indexes the table once
// per token; repeated ids in a batch therefore re-read the same N rows.  This kernel finds the
// distinct ids so that each row block is read once per group of tokens (and, in offloaded mode,
// crosses the host link once).
//
// One workgroup.  A V-bit presence bitmap sits in LDS (V = 50304 -> 6.3 KB): every id sets its
// bit with an LDS atomic OR; a popcount prefix over the bitmap words then gives each present id
// its rank, which is already the position in ascending order -- no sort.  Tokens are then
// bucketed by rank with a counting pass (LDS counters when they fit), and every bucket is cut
// into groups of at most PLAN_GROUP tokens so that one very frequent id (Zipf head) becomes
// many bounded work items instead of one long one.
#include "mole_internal.h"

namespace {
using namespace mole;

constexpr int DEDUP_THREADS = 1024;
constexpr int64_t DEDUP_MAX_V = 524288;

// exclusive scan of one value per thread over the workgroup; *total gets the sum
__device__ __forceinline__ int block_exclusive_scan(int v, int *wave_sums, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int n = __shfl_up(incl, o);
        if (lane >= o)
            incl += n;
    }
    __syncthreads();   // protects wave_sums against a previous use
    if (lane == 63)
        wave_sums[wave] = incl;
    __syncthreads();
    int base = 0;
    const int nw = blockDim.x >> 6;
    for (int w = 0; w < nw; ++w) {
        const int s = wave_sums[w];
        if (w < wave)
            base += s;
    }
    if (total) {
        int tot = 0;
        for (int w = 0; w < nw; ++w)
            tot += wave_sums[w];
        *total = tot;
    }
    return base + incl - v;
}

// lds_counters != 0: the per-rank counters live in LDS behind bitmap and prefix
__global__ __launch_bounds__(DEDUP_THREADS) void dedup_kernel(const int32_t *__restrict__ ids, int T, int V,
                                                                int32_t *__restrict__ uniq_out,
                                                                int32_t *__restrict__ inv_out,
                                                                int32_t *__restrict__ n_uniq_out,
                                                                int32_t *err_flag, int32_t *plan,
                                                                int lds_counters)
{
    extern __shared__ uint32_t sm[];
    __shared__ int wave_sums[DEDUP_THREADS / 64];
    __shared__ int s_bad;
    const int W = (V + 31) >> 5;
    uint32_t *bitmap = sm;
    int *prefix = reinterpret_cast<int *>(sm + W);
    const PlanLayout pl = plan_layout(T);
    int *counters = lds_counters ? reinterpret_cast<int *>(sm + 2 * W) : plan + pl.counters;
    const int tid = threadIdx.x;

    for (int w = tid; w < W; w += DEDUP_THREADS)
        bitmap[w] = 0u;
    for (int i = tid; i < T + 2; i += DEDUP_THREADS)
        counters[i] = 0;
    if (tid == 0)
        s_bad = 0;
    __syncthreads();

    // 1. presence bits
    int bad = 0;
    for (int t = tid; t < T; t += DEDUP_THREADS) {
        const int id = ids[t];
        if (id < 0 || id >= V)
            bad = 1;
        else
            atomicOr(&bitmap[id >> 5], 1u << (id & 31));
    }
    if (bad)
        s_bad = 1;
    __syncthreads();

    // 2. rank of every word: exclusive popcount prefix; each thread owns a contiguous run of words
    const int per = (W + DEDUP_THREADS - 1) / DEDUP_THREADS;
    const int w0 = min(tid * per, W), w1 = min(w0 + per, W);
    int local = 0;
    for (int w = w0; w < w1; ++w)
        local += __popc(bitmap[w]);
    int U = 0;
    int run = block_exclusive_scan(local, wave_sums, &U);
    for (int w = w0; w < w1; ++w) {
        prefix[w] = run;
        uint32_t bits = bitmap[w];
        while (bits) {                       // 3. emit the distinct ids, ascending
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            const int id = (w << 5) + b;
            uniq_out[run] = id;
            plan[pl.uniq + run] = id;
            ++run;
        }
    }
    __syncthreads();

    // 4. inverse map and bucket sizes; bucket U collects the out-of-range tokens
    for (int t = tid; t < T; t += DEDUP_THREADS) {
        const int id = ids[t];
        int r = -1;
        if (id >= 0 && id < V)
            r = prefix[id >> 5] + __popc(bitmap[id >> 5] & ((1u << (id & 31)) - 1u));
        inv_out[t] = r;
        atomicAdd(&counters[r < 0 ? U : r], 1);
    }
    __syncthreads();

    // 5. bucket offsets and work items: a bucket of c tokens becomes ceil(c / PLAN_GROUP) items
    const int B = U + 1;
    const int perb = (B + DEDUP_THREADS - 1) / DEDUP_THREADS;
    const int b0 = min(tid * perb, B), b1 = min(b0 + perb, B);
    int tok = 0, itm = 0;
    for (int b = b0; b < b1; ++b) {
        const int c = counters[b];
        tok += c;
        itm += (c + PLAN_GROUP - 1) / PLAN_GROUP;
    }
    int n_items = 0;
    int tok_run = block_exclusive_scan(tok, wave_sums, nullptr);
    int itm_run = block_exclusive_scan(itm, wave_sums, &n_items);
    for (int b = b0; b < b1; ++b) {
        const int c = counters[b];
        counters[b] = tok_run;               // becomes the bucket's write cursor
        for (int s = 0; s < c; s += PLAN_GROUP) {
            plan[pl.item_u + itm_run] = b;
            plan[pl.item_begin + itm_run] = tok_run + s;
            plan[pl.item_cnt + itm_run] = min(PLAN_GROUP, c - s);
            ++itm_run;
        }
        tok_run += c;
    }
    __syncthreads();

    // 6. scatter token indices into their buckets (order inside a bucket is irrelevant)
    for (int t = tid; t < T; t += DEDUP_THREADS) {
        const int r = inv_out[t];
        const int pos = atomicAdd(&counters[r < 0 ? U : r], 1);
        plan[pl.order + pos] = t;
    }

    if (tid == 0) {
        plan[0] = n_items;
        plan[1] = U;
        plan[2] = T;
        plan[3] = PLAN_GROUP;
        plan[4] = V;
        plan[5] = PLAN_MAGIC;
        *n_uniq_out = U;
        if (s_bad && err_flag)
            *err_flag = 1;
    }
}

size_t dedup_lds_bytes(int T, int64_t V, int *lds_counters)
{
    const size_t W = (size_t)((V + 31) / 32);
    size_t bytes = 2 * W * 4;
    const size_t with_counters = bytes + (size_t)(T + 2) * 4;
    *lds_counters = with_counters <= 150 * 1024;
    return *lds_counters ? with_counters : bytes;
}

}  // namespace

extern "C" size_t mole_dedup_workspace(int T, int64_t V)
{
    (void)V;
    if (T < 0)
        return 0;
    return (size_t)mole::plan_layout(T).words * 4;
}

extern "C" mole_status mole_dedup_ids(const int32_t *ids, int T, int64_t V, int32_t *uniq, int32_t *inv,
                                      int32_t *n_uniq, int32_t *err_flag, void *workspace,
                                      size_t workspace_bytes, void *hip_stream)
{
    clear_error();
    if (T < 0 || V < 1)
        return fail(MOLE_EINVAL, "mole_dedup_ids: bad size (T=%d, V=%lld)", T, (long long)V);
    if (V > DEDUP_MAX_V)
        return fail(MOLE_EUNSUPPORTED, "mole_dedup_ids: V=%lld exceeds %lld (presence bitmap must fit in LDS)",
                    (long long)V, (long long)DEDUP_MAX_V);
    if (!n_uniq || (T > 0 && (!ids || !uniq || !inv)))
        return fail(MOLE_EINVAL, "mole_dedup_ids: ids, uniq, inv and n_uniq must not be NULL");
    const size_t need = mole_dedup_workspace(T, V);
    if (!workspace || workspace_bytes < need)
        return fail(MOLE_EWORKSPACE, "mole_dedup_ids: workspace of %zu bytes needed, got %zu", need,
                    workspace ? workspace_bytes : (size_t)0);
    if (!aligned16(workspace))
        return fail(MOLE_EINVAL, "mole_dedup_ids: workspace is not 16-byte aligned");
    int lds_counters = 0;
    const size_t lds = dedup_lds_bytes(T, V, &lds_counters);
    static size_t attr_set = 0;
    if (lds > attr_set) {
        MOLE_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&dedup_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = lds;
    }
    hipLaunchKernelGGL(dedup_kernel, dim3(1), dim3(DEDUP_THREADS), lds, static_cast<hipStream_t>(hip_stream),
                       ids, T, (int)V, uniq, inv, n_uniq, err_flag, static_cast<int32_t *>(workspace),
                       lds_counters);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}
