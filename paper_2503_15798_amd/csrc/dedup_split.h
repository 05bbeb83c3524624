// Device code of mole_dedup_ids that more than one translation unit launches: the workgroup scans and the
// kernel body that spreads a large batch over several workgroups by id range (the lut(input_ids) line of the
// inference listing indexes once per token; this finds the distinct ids).
#ifndef MOLE_DEDUP_SPLIT_H
#define MOLE_DEDUP_SPLIT_H

#include "mole_internal.h"

namespace mole {

constexpr int DEDUP_THREADS = 1024;
constexpr int64_t DEDUP_MAX_V = 524288;

// inclusive scan over the 64 lanes of a wave: DPP row shifts (row_shr:1, 2, 4, 8, zero fill) give the scan inside
// each row of 16 lanes, the three row totals are then added to the rows above them
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
    const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
              t2 = __builtin_amdgcn_readlane(v, 47);
    const int lane = threadIdx.x & 63;
    return v + (lane >= 16 ? t0 : 0) + (lane >= 32 ? t1 : 0) + (lane >= 48 ? t2 : 0);
}

// exclusive scan of one value per thread over the workgroup; *total gets the sum.  One barrier: every use
// in a kernel gets a wave_sums array of its own, so none has to be protected against the one before.
constexpr int DEDUP_WAVES = DEDUP_THREADS / 64;
__device__ __forceinline__ int block_exclusive_scan(int v, int *wave_sums, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int incl = wave_inclusive_scan(v);
    if (lane == 63)
        wave_sums[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < DEDUP_WAVES; ++w) {
        const int s = wave_sums[w];
        base += w < wave ? s : 0;
        tot += s;
    }
    if (total)
        *total = tot;
    return base + incl - v;
}

// The same for the largest batches (8 to 16 tokens per thread), spread over K workgroups by id range:
// workgroup k owns the bitmap words [k W / K, (k + 1) W / K).  There is nothing to exchange between the
// workgroups: each reads all ids and sets all presence bits itself (what it needs from the ranges below its own
// are two counts: their distinct ids and their tokens), and then ranks, sizes and places only the tokens of its
// own range, which is the part that is bound by random LDS accesses (two thirds of the one-workgroup kernel's
// time).  Its distinct ids, bucket starts and token order are contiguous pieces of the outputs.  Out-of-range
// tokens form the last bucket of the last workgroup.
// k, K: this workgroup's index and the number of workgroups that share the batch; sm: the workgroup's LDS area of
// dedup_split_lds_bytes(T, V) bytes.  A device function, so that a launch can hold other work beside it.
template <int PER>
__device__ __forceinline__ void dedup_split_body(const int32_t *__restrict__ ids, int T, int V,
                                                 int32_t *__restrict__ uniq_out, int32_t *__restrict__ inv_out,
                                                 int32_t *__restrict__ n_uniq_out, int32_t *err_flag, int32_t *plan,
                                                 int k, int K, uint32_t *sm)
{
    __shared__ int wave_sums[3][DEDUP_WAVES];
    __shared__ int s_bad;
    const int W = (V + 31) >> 5;
    uint32_t *bitmap = sm;                                   // [W] presence bits
    int *prefix = reinterpret_cast<int *>(sm + W);           // [W] distinct ids below the word
    const PlanLayout pl = plan_layout(T);
    int *counters = reinterpret_cast<int *>(sm + 2 * W);     // [T + 2]: bucket sizes, then bucket starts (own range)
    int *stage = counters + (T + 2);                         // [T]
    const int tid = threadIdx.x;
    const bool last_wg = k == K - 1;
    const int my_w0 = (int)((int64_t)W * k / K), my_w1 = (int)((int64_t)W * (k + 1) / K);

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

    // 1. presence bits of all tokens; tokens of the ranges below this one are counted
    int bad = 0, below = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int id = idv[u];
        if (tid + u * DEDUP_THREADS >= T)
            continue;
        if (id < 0 || id >= V) {
            bad = 1;
        } else {
            below += (id >> 5) < my_w0;
            if (!(__atomic_load_n(&bitmap[id >> 5], __ATOMIC_RELAXED) & (1u << (id & 31))))
                atomicOr(&bitmap[id >> 5], 1u << (id & 31));
        }
    }
    if (bad)
        s_bad = 1;
    int T_before = 0;
    block_exclusive_scan(below, wave_sums[2], &T_before);    // its barrier also ends pass 1

    // 2. rank of every bitmap word (all words: the ranks are global)
    const int per = (W + DEDUP_THREADS - 1) / DEDUP_THREADS;
    const int w0 = min(tid * per, W), w1 = min(w0 + per, W);
    int local = 0;
    for (int w = w0; w < w1; ++w)
        local += __popc(bitmap[w]);
    int U = 0;
    int run = block_exclusive_scan(local, wave_sums[0], &U);
    for (int w = w0; w < w1; ++w) {
        prefix[w] = run;
        run += __popc(bitmap[w]);
    }
    __syncthreads();
    const int U_before = my_w0 < W ? prefix[my_w0] : U;
    const int U_mine = (my_w1 < W ? prefix[my_w1] : U) - U_before;

    // 3. the distinct ids of this range, ascending
    for (int w = my_w0 + tid; w < my_w1; w += DEDUP_THREADS) {
        uint32_t bits = bitmap[w];
        int at = prefix[w] - U_before;
        while (bits) {
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            stage[at++] = (w << 5) + b;
        }
    }
    __syncthreads();
    for (int i = tid; i < U_mine; i += DEDUP_THREADS) {
        const int id = stage[i];
        uniq_out[U_before + i] = id;
        plan[pl.uniq + U_before + i] = id;
    }

    // 4. inverse map, bucket sizes and places of this range's tokens (bucket index relative to the range; the
    //    last workgroup's bucket U_mine collects the out-of-range tokens)
    int bucket[PER], place[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int t = tid + u * DEDUP_THREADS;
        const int id = idv[u];
        bucket[u] = -1;
        if (t < T) {
            if (id >= 0 && id < V) {
                const int w = id >> 5;
                if (w >= my_w0 && w < my_w1) {
                    const int r = prefix[w] + __popc(bitmap[w] & ((1u << (id & 31)) - 1u));
                    bucket[u] = r - U_before;
                    inv_out[t] = r;
                }
            } else if (last_wg) {
                bucket[u] = U_mine;
                inv_out[t] = -1;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < PER; ++u)
        place[u] = bucket[u] >= 0 ? atomicAdd(&counters[bucket[u]], 1) : 0;
    __syncthreads();    // also: `stage` has been copied out and may be reused

    // 5. bucket starts of this range: exclusive scan of the sizes, in place; counters[B] = tokens of the range
    const int B = U_mine + (last_wg ? 1 : 0);
    const int perb = (B + DEDUP_THREADS - 1) / DEDUP_THREADS;
    const int b0 = min(tid * perb, B), b1 = min(b0 + perb, B);
    int tok = 0;
    for (int b = b0; b < b1; ++b)
        tok += counters[b];
    int T_mine = 0;
    int tok_run = block_exclusive_scan(tok, wave_sums[1], &T_mine);
    for (int b = b0; b < b1; ++b) {
        const int c = counters[b];
        counters[b] = tok_run;
        tok_run += c;
    }
    if (tid == 0)
        counters[B] = T_mine;
    __syncthreads();
    // starts of this range's buckets (the next range writes the end of the last one as its own first start;
    // the last workgroup writes the two closing entries)
    for (int i = tid; i < B + (last_wg ? 1 : 0); i += DEDUP_THREADS)
        plan[pl.start + U_before + i] = T_before + counters[i];

    // 6. token indices into their buckets, through LDS so that the order leaves as full-width stores
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int t = tid + u * DEDUP_THREADS;
        const int b = bucket[u];
        if (b >= 0) {
            const int first = counters[b];
            const bool single = b < U_mine && counters[b + 1] - first == 1;
            stage[first + place[u]] = (int)((uint32_t)t | (single ? PLAN_SINGLE : 0u));
        }
    }
    __syncthreads();
    for (int i = tid; i < T_mine; i += DEDUP_THREADS)
        plan[pl.order + T_before + i] = stage[i];

    if (tid == 0 && k == 0) {
        plan[0] = U;
        plan[1] = 0;
        plan[2] = T;
        plan[3] = 0;
        plan[4] = V;
        plan[5] = PLAN_MAGIC;
        *n_uniq_out = U;
    }
    if (tid == 0 && last_wg && s_bad && err_flag)
        *err_flag = 1;
}

// LDS bytes of dedup_split_body: bitmap, prefix, counters [T + 2], staging area [T + 2]
__host__ __device__ constexpr size_t dedup_split_lds_bytes(int T, int64_t V)
{
    return (size_t)((V + 31) / 32) * 8 + (size_t)(T + 2) * 8;
}
constexpr int DEDUP_SPLIT_WGS = 8;
constexpr size_t DEDUP_LDS_LIMIT = 156 * 1024;

}  // namespace mole
#endif
