// mole_dedup_ids: distinct token ids of a batch (ascending), the inverse map, and a visiting
// plan (tokens in id order) for the forward kernels.
//
// The paper's lookup (inference listing, the lut(input_ids) line) simply indexes the table once
// per token; repeated ids in a batch therefore re-read the same N rows.  This kernel finds the
// distinct ids so that each row block crosses the memory fabric once (and, in offloaded mode,
// the host link once).
//
// One workgroup (eight, each owning an id range, for batches of more than 4096 tokens: dedup_split.h).
// A V-bit presence bitmap sits in LDS (V = 50304 -> 6.3 KB): every id sets its
// bit with an LDS atomic OR; a popcount prefix over the bitmap words then gives each present id
// its rank, which is already the position in ascending order -- no sort.  Tokens are then
// bucketed by rank with a counting pass (LDS counters when they fit) and scattered, which yields
// the token indices in id order: the forward kernel walks that order so that equal ids are
// processed next to each other (same workgroup, same L2) and marks ids that occur once.
#include "dedup_split.h"

namespace {
using namespace mole;

constexpr int BATCH = 8;   // independent loads per thread and pass

// lds_counters != 0: the per-rank counters live in LDS behind bitmap and prefix
__global__ __launch_bounds__(DEDUP_THREADS) void dedup_kernel(const int32_t *__restrict__ ids, int T, int V,
                                                                int32_t *__restrict__ uniq_out,
                                                                int32_t *__restrict__ inv_out,
                                                                int32_t *__restrict__ n_uniq_out,
                                                                int32_t *err_flag, int32_t *plan,
                                                                int lds_counters, int lds_stage)
{
    extern __shared__ uint32_t sm[];
    __shared__ int wave_sums[2][DEDUP_WAVES];
    __shared__ int s_bad;
    const int W = (V + 31) >> 5;
    uint32_t *bitmap = sm;
    int *prefix = reinterpret_cast<int *>(sm + W);
    const PlanLayout pl = plan_layout(T);
    int *counters = lds_counters ? reinterpret_cast<int *>(sm + 2 * W) : plan + pl.counters;
    // staging area for scattered results (first the distinct ids, then the token order): a single
    // CU issues scattered 4-byte global stores one address at a time, so they are gathered in LDS
    // and written out as full wave-wide stores
    int *stage = lds_stage ? reinterpret_cast<int *>(sm + 2 * W) + (T + 2) : nullptr;
    const int tid = threadIdx.x;

    for (int w = tid; w < W; w += DEDUP_THREADS)
        bitmap[w] = 0u;
    for (int i = tid; i < T + 2; i += DEDUP_THREADS)
        counters[i] = 0;
    if (tid == 0)
        s_bad = 0;
    __syncthreads();

    // Every pass over the tokens reads them in batches of BATCH independent loads per thread, so
    // that a thread pays one memory latency per batch instead of one per token.
    // 1. presence bits
    int bad = 0;
    for (int t0 = tid; t0 < T; t0 += DEDUP_THREADS * BATCH) {
        int idv[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int t = t0 + u * DEDUP_THREADS;
            idv[u] = t < T ? ids[t] : 0;
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int id = idv[u];
            if (t0 + u * DEDUP_THREADS >= T)
                continue;
            if (id < 0 || id >= V)
                bad = 1;
            else if (!(__atomic_load_n(&bitmap[id >> 5], __ATOMIC_RELAXED) & (1u << (id & 31))))
                atomicOr(&bitmap[id >> 5], 1u << (id & 31));   // skipped once the bit is seen set: hot ids
        }
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
    int run = block_exclusive_scan(local, wave_sums[0], &U);
    for (int w = w0; w < w1; ++w) {
        prefix[w] = run;
        uint32_t bits = bitmap[w];
        while (bits) {                       // 3. emit the distinct ids, ascending
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            const int id = (w << 5) + b;
            if (stage) {
                stage[run] = id;
            } else {
                uniq_out[run] = id;
                plan[pl.uniq + run] = id;
            }
            ++run;
        }
    }
    __syncthreads();
    if (stage) {
        for (int i = tid; i < U; i += DEDUP_THREADS) {
            const int id = stage[i];
            uniq_out[i] = id;
            plan[pl.uniq + i] = id;
        }
        // the staging area is reused for the token order; the barrier after pass 4 separates the two
    }

    // 4. inverse map and bucket sizes; bucket U collects the out-of-range tokens
    for (int t0 = tid; t0 < T; t0 += DEDUP_THREADS * BATCH) {
        int idv[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int t = t0 + u * DEDUP_THREADS;
            idv[u] = t < T ? ids[t] : -1;
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int t = t0 + u * DEDUP_THREADS;
            if (t >= T)
                continue;
            const int id = idv[u];
            int r = -1;
            if (id >= 0 && id < V)
                r = prefix[id >> 5] + __popc(bitmap[id >> 5] & ((1u << (id & 31)) - 1u));
            inv_out[t] = r;
            atomicAdd(&counters[r < 0 ? U : r], 1);
        }
    }
    __syncthreads();

    // 5. bucket offsets: exclusive scan of the bucket sizes; counters become write cursors
    const int B = U + 1;
    const int perb = (B + DEDUP_THREADS - 1) / DEDUP_THREADS;
    const int b0 = min(tid * perb, B), b1 = min(b0 + perb, B);
    int tok = 0;
    for (int b = b0; b < b1; ++b)
        tok += counters[b];
    int tok_run = block_exclusive_scan(tok, wave_sums[1], nullptr);
    for (int b = b0; b < b1; ++b) {
        const int c = counters[b];
        counters[b] = tok_run;
        plan[pl.start + b] = tok_run;
        tok_run += c;
    }
    if (tid == 0)
        plan[pl.start + B] = T;
    __syncthreads();

    // 6. scatter token indices into their buckets (order inside a bucket is irrelevant)
    for (int t0 = tid; t0 < T; t0 += DEDUP_THREADS * BATCH) {
        int rv[BATCH], pos[BATCH], cnt[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int t = t0 + u * DEDUP_THREADS;
            rv[u] = t < T ? inv_out[t] : -1;
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int b = rv[u] < 0 ? U : rv[u];
            const bool live = t0 + u * DEDUP_THREADS < T;
            pos[u] = live ? atomicAdd(&counters[b], 1) : 0;
            cnt[u] = live ? plan[pl.start + b + 1] - plan[pl.start + b] : 0;
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int t = t0 + u * DEDUP_THREADS;
            if (t < T) {
                const int val = (int)((uint32_t)t | (rv[u] >= 0 && cnt[u] == 1 ? PLAN_SINGLE : 0u));
                if (stage)
                    stage[pos[u]] = val;
                else
                    plan[pl.order + pos[u]] = val;
            }
        }
    }
    if (stage) {
        __syncthreads();
        for (int i = tid; i < T; i += DEDUP_THREADS)
            plan[pl.order + i] = stage[i];
    }

    if (tid == 0) {
        plan[0] = U;
        plan[1] = 0;
        plan[2] = T;
        plan[3] = 0;
        plan[4] = V;
        plan[5] = PLAN_MAGIC;
        *n_uniq_out = U;
        if (s_bad && err_flag)
            *err_flag = 1;
    }
}

// Batches of at most PER * 1024 tokens: every thread keeps its PER tokens (id, rank, place inside the
// bucket) in registers, so the ids are read from memory once, and the contended counting pass runs once:
// the atomic add that sizes the buckets also hands each token its place inside its bucket.  Counters
// and staging area are always in LDS here.
template <int PER>
__global__ __launch_bounds__(DEDUP_THREADS) void dedup_kernel_regs(const int32_t *__restrict__ ids, int T, int V,
                                                                     int32_t *__restrict__ uniq_out,
                                                                     int32_t *__restrict__ inv_out,
                                                                     int32_t *__restrict__ n_uniq_out,
                                                                     int32_t *err_flag, int32_t *plan)
{
    extern __shared__ uint32_t sm[];
    __shared__ int wave_sums[2][DEDUP_WAVES];
    __shared__ int s_bad;
    const int W = (V + 31) >> 5;
    uint32_t *bitmap = sm;                                   // [W] presence bits
    int *prefix = reinterpret_cast<int *>(sm + W);           // [W] distinct ids below the word
    const PlanLayout pl = plan_layout(T);
    int *counters = reinterpret_cast<int *>(sm + 2 * W);     // [T + 2]: bucket sizes, then bucket starts
    int *stage = counters + (T + 2);                         // [T]
    const int tid = threadIdx.x;

    // the thread's tokens: t = tid + u * 1024 (coalesced), loaded before LDS is cleared
    int idv[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int t = tid + u * DEDUP_THREADS;
        idv[u] = t < T ? ids[t] : 0;
    }
    for (int w = tid; w < W; w += DEDUP_THREADS)
        bitmap[w] = 0u;
    for (int i = tid; i < T + 2; i += DEDUP_THREADS)
        counters[i] = 0;
    if (tid == 0)
        s_bad = 0;
    __syncthreads();

    // 1. presence bits (the atomic is skipped once the bit is seen set: hot ids)
    int bad = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int id = idv[u];
        if (tid + u * DEDUP_THREADS >= T)
            continue;
        if (id < 0 || id >= V)
            bad = 1;
        else if (!(__atomic_load_n(&bitmap[id >> 5], __ATOMIC_RELAXED) & (1u << (id & 31))))
            atomicOr(&bitmap[id >> 5], 1u << (id & 31));
    }
    if (bad)
        s_bad = 1;
    __syncthreads();

    // 2. / 3. rank of every bitmap word, distinct ids in ascending order
    const int per = (W + DEDUP_THREADS - 1) / DEDUP_THREADS;
    const int w0 = min(tid * per, W), w1 = min(w0 + per, W);
    int local = 0;
    for (int w = w0; w < w1; ++w)
        local += __popc(bitmap[w]);
    int U = 0;
    int run = block_exclusive_scan(local, wave_sums[0], &U);
    for (int w = w0; w < w1; ++w) {
        uint32_t bits = bitmap[w];
        prefix[w] = run;
        while (bits) {
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            stage[run++] = (w << 5) + b;
        }
    }
    __syncthreads();
    for (int i = tid; i < U; i += DEDUP_THREADS) {
        const int id = stage[i];
        uniq_out[i] = id;
        plan[pl.uniq + i] = id;
    }

    // 4. inverse map (all ranks first, so that their LDS reads travel together); then the atomic add that sizes
    //    bucket r also gives the token its place in it.  Bucket U collects the out-of-range tokens.
    int bucket[PER], place[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int t = tid + u * DEDUP_THREADS;
        const int id = idv[u];
        int r = -1;
        if (t < T && id >= 0 && id < V)
            r = prefix[id >> 5] + __popc(bitmap[id >> 5] & ((1u << (id & 31)) - 1u));
        bucket[u] = r < 0 ? U : r;
        if (t < T)
            inv_out[t] = r;
    }
#pragma unroll
    for (int u = 0; u < PER; ++u)
        place[u] = tid + u * DEDUP_THREADS < T ? atomicAdd(&counters[bucket[u]], 1) : 0;
    __syncthreads();    // also: `stage` has been copied out and may be reused

    // 5. bucket starts: exclusive scan of the sizes, in place; counters[U + 1] = T
    const int B = U + 1;
    const int perb = (B + DEDUP_THREADS - 1) / DEDUP_THREADS;
    const int b0 = min(tid * perb, B), b1 = min(b0 + perb, B);
    int tok = 0;
    for (int b = b0; b < b1; ++b)
        tok += counters[b];
    int tok_run = block_exclusive_scan(tok, wave_sums[1], nullptr);
    for (int b = b0; b < b1; ++b) {
        const int c = counters[b];
        counters[b] = tok_run;
        tok_run += c;
    }
    if (tid == 0)
        counters[B] = T;
    __syncthreads();
    for (int i = tid; i <= B; i += DEDUP_THREADS)       // the starts leave as full-width stores
        plan[pl.start + i] = counters[i];

    // 6. token indices into their buckets, through LDS so that the order leaves as full-width stores
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int t = tid + u * DEDUP_THREADS;
        if (t < T) {
            const int b = bucket[u];
            const int first = counters[b];
            const bool single = b < U && counters[b + 1] - first == 1;
            stage[first + place[u]] = (int)((uint32_t)t | (single ? PLAN_SINGLE : 0u));
        }
    }
    __syncthreads();
    for (int i = tid; i < T; i += DEDUP_THREADS)
        plan[pl.order + i] = stage[i];

    if (tid == 0) {
        plan[0] = U;
        plan[1] = 0;
        plan[2] = T;
        plan[3] = 0;
        plan[4] = V;
        plan[5] = PLAN_MAGIC;
        *n_uniq_out = U;
        if (s_bad && err_flag)
            *err_flag = 1;
    }
}

template <int PER>
__global__ __launch_bounds__(DEDUP_THREADS) void dedup_kernel_split(const int32_t *__restrict__ ids, int T, int V,
                                                                      int32_t *__restrict__ uniq_out,
                                                                      int32_t *__restrict__ inv_out,
                                                                      int32_t *__restrict__ n_uniq_out,
                                                                      int32_t *err_flag, int32_t *plan)
{
    extern __shared__ uint32_t sm[];
    dedup_split_body<PER>(ids, T, V, uniq_out, inv_out, n_uniq_out, err_flag, plan, blockIdx.x, gridDim.x, sm);
}

template <int PER>
hipError_t launch_split(size_t lds, hipStream_t stream, const int32_t *ids, int T, int V, int32_t *uniq, int32_t *inv,
                        int32_t *n_uniq, int32_t *err_flag, int32_t *plan)
{
    static std::atomic<size_t> lds_seen{0};
    const hipError_t e = ensure_dynamic_lds(lds_seen, reinterpret_cast<const void *>(&dedup_kernel_split<PER>), lds);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(dedup_kernel_split<PER>, dim3(DEDUP_SPLIT_WGS), dim3(DEDUP_THREADS), lds, stream, ids, T, V, uniq,
                       inv, n_uniq, err_flag, plan);
    return hipGetLastError();
}

template <int PER>
hipError_t launch_regs(size_t lds, hipStream_t stream, const int32_t *ids, int T, int V, int32_t *uniq, int32_t *inv,
                       int32_t *n_uniq, int32_t *err_flag, int32_t *plan)
{
    static std::atomic<size_t> lds_seen{0};
    const hipError_t e = ensure_dynamic_lds(lds_seen, reinterpret_cast<const void *>(&dedup_kernel_regs<PER>), lds);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(dedup_kernel_regs<PER>, dim3(1), dim3(DEDUP_THREADS), lds, stream, ids, T, V, uniq, inv, n_uniq,
                       err_flag, plan);
    return hipGetLastError();
}

// LDS plan: bitmap and prefix always; the counters and the staging area when they fit
size_t dedup_lds_bytes(int T, int64_t V, int *lds_counters, int *lds_stage)
{
    const size_t W = (size_t)((V + 31) / 32);
    const size_t limit = DEDUP_LDS_LIMIT;
    const size_t base = 2 * W * 4;
    const size_t with_counters = base + (size_t)(T + 2) * 4;
    const size_t with_stage = with_counters + (size_t)(T + 2) * 4;
    *lds_counters = with_counters <= limit;
    *lds_stage = with_stage <= limit;
    return *lds_stage ? with_stage : (*lds_counters ? with_counters : base);
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
    MOLE_ARCH_CHECK("mole_dedup_ids");
    int lds_counters = 0, lds_stage = 0;
    const size_t lds = dedup_lds_bytes(T, V, &lds_counters, &lds_stage);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int32_t *plan = static_cast<int32_t *>(workspace);
    // up to 16 tokens per thread with everything staged in LDS: the register-resident kernel
    if (lds_stage && T <= 16 * DEDUP_THREADS && knob(KNOB_DEDUP_GENERIC) != 1) {
        const int per = (T + DEDUP_THREADS - 1) / DEDUP_THREADS;
        // from five tokens per thread on the batch is spread over eight workgroups (MOLE_DEDUP_GENERIC = 2: never)
        const bool split = per > 4 && knob(KNOB_DEDUP_GENERIC) != 2;
        hipError_t e;
        if (per <= 1)
            e = launch_regs<1>(lds, stream, ids, T, (int)V, uniq, inv, n_uniq, err_flag, plan);
        else if (per <= 2)
            e = launch_regs<2>(lds, stream, ids, T, (int)V, uniq, inv, n_uniq, err_flag, plan);
        else if (per <= 4)
            e = launch_regs<4>(lds, stream, ids, T, (int)V, uniq, inv, n_uniq, err_flag, plan);
        else if (per <= 8 && split)
            e = launch_split<8>(lds, stream, ids, T, (int)V, uniq, inv, n_uniq, err_flag, plan);
        else if (per <= 8)
            e = launch_regs<8>(lds, stream, ids, T, (int)V, uniq, inv, n_uniq, err_flag, plan);
        else if (split)
            e = launch_split<16>(lds, stream, ids, T, (int)V, uniq, inv, n_uniq, err_flag, plan);
        else
            e = launch_regs<16>(lds, stream, ids, T, (int)V, uniq, inv, n_uniq, err_flag, plan);
        MOLE_HIP_CHECK(e);
        return MOLE_OK;
    }
    static std::atomic<size_t> lds_seen{0};
    MOLE_HIP_CHECK(ensure_dynamic_lds(lds_seen, reinterpret_cast<const void *>(&dedup_kernel), lds));
    hipLaunchKernelGGL(dedup_kernel, dim3(1), dim3(DEDUP_THREADS), lds, stream, ids, T, (int)V, uniq, inv, n_uniq,
                       err_flag, plan, lds_counters, lds_stage);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}
