// mole_dedup_forward: the dedup of a batch's ids and the layer forward in its id order, as one call.
//
// Paper: the lut(input_ids) line of the inference listing (one table read per token; the dedup finds the
// distinct ids), Sec. 3.2 (router equation) and Sec. 3.3 (inference-layer equation).
//
// The forward in id order needs the plan before its first row is read, so as two calls the dedup (12 us for
// 16384 tokens: a few workgroups, bound by LDS latency) sits in front of the forward with the rest of the chip
// idle.  The router does not need the plan: gates depend on a token's own h only.  Here the first launch holds
// both: workgroups 0 .. K-1 run the dedup (dedup_split_body), all others compute the gates of all tokens on
// the matrix pipe (router_tile), tiles of 32 tokens in token order; the second launch gathers and combines in
// the plan's order with the gates given (one wave per token, handed out by the hardware dispatcher).  The
// dedup's time disappears behind the router's.
// Large batches at N = 32 (the prefill shape); every other shape runs the two calls one after the other.
#include "dedup_split.h"
#include "tile_router.h"

namespace {
using namespace mole;

struct DedupArgs {
    const int32_t *ids;
    int32_t *uniq, *inv, *n_uniq, *err_flag, *plan;
    int T, V;
};
struct RouteArgs {
    const uint16_t *h, *W_r, *ln_w;     // ln_w: NORM only
    float ln_eps;
    float *gates;                       // [T, N] fp32
    int d;
};

constexpr int ROUTE_N = 32;
constexpr int ROUTE_WPB = 8;            // waves per tile: the split of d must be the tile kernel's, so that the gates
                                        // (and with them the output) are the two-call path's bit for bit
constexpr int ROUTE_GROUPS = DEDUP_THREADS / (ROUTE_WPB * 64);      // tiles a workgroup works on at a time
constexpr size_t ROUTE_GROUP_FLOATS = router_part_floats(ROUTE_N, ROUTE_WPB) + router_ssq_floats(ROUTE_WPB);
constexpr size_t ROUTE_LDS_BYTES = ROUTE_GROUPS * ROUTE_GROUP_FLOATS * sizeof(float);

// WT: the router weight is transposed into LDS once per workgroup (behind the two groups' areas)
template <int PER, bool NORM, bool WT>
__global__ __launch_bounds__(DEDUP_THREADS) void dedup_route_kernel(DedupArgs dd, RouteArgs ra, int K)
{
    extern __shared__ uint32_t sm[];
    if ((int)blockIdx.x < K) {
        dedup_split_body<PER>(dd.ids, dd.T, dd.V, dd.uniq, dd.inv, dd.n_uniq, dd.err_flag, dd.plan, (int)blockIdx.x, K, sm);
        return;
    }
    // router: the workgroup's 16 waves are two groups of eight, each with a tile of its own; both go round the loop
    // the same number of times (a group without a tile computes on token 0 and stores nothing), so the barriers match
    const int T = dd.T;
    const int group = __builtin_amdgcn_readfirstlane(threadIdx.x >> 9);
    const int wave = __builtin_amdgcn_readfirstlane((threadIdx.x >> 6) & (ROUTE_WPB - 1));
    const int lane = threadIdx.x & 63;
    float *part = reinterpret_cast<float *>(sm) + group * ROUTE_GROUP_FLOATS;
    float *ssq = part + router_part_floats(ROUTE_N, ROUTE_WPB);
    const int G = gridDim.x - K, g = blockIdx.x - K;
    const int tiles = (T + ROUTER_TILE - 1) / ROUTER_TILE;
    const uint16_t *wt = nullptr;
    if constexpr (WT) {
        uint16_t *w = reinterpret_cast<uint16_t *>(reinterpret_cast<float *>(sm) + ROUTE_GROUPS * ROUTE_GROUP_FLOATS);
        router_fill_wt<ROUTE_N>(w, ra.W_r, ra.d, DEDUP_THREADS);
        wt = w;
        __syncthreads();
    }
    for (int pair = g; pair * ROUTE_GROUPS < tiles; pair += G) {
        const int tok0 = (pair * ROUTE_GROUPS + group) * ROUTER_TILE;
        router_tile<ROUTE_N, ROUTE_WPB, NORM, WT>(
            part, ssq, ra.h, ra.W_r, ra.ln_w, ra.ln_eps, ra.d, wave, lane,
            [&](int c) { return tok0 + c < T ? tok0 + c : -1; },
            [&](int, int tok, int j, float gj) {
                if (tok >= 0)
                    ra.gates[(int64_t)tok * ROUTE_N + j] = gj;
            },
            wt);
        __syncthreads();    // the next tile's partial products overwrite what step 2 read
    }
}

template <int PER, bool NORM, bool WT>
mole_status launch_dedup_route_wt(const DedupArgs &dd, const RouteArgs &ra, hipStream_t stream)
{
    size_t lds = dedup_split_lds_bytes(dd.T, dd.V);
    const size_t route_lds = ROUTE_LDS_BYTES + (WT ? router_wt_bytes(ROUTE_N, ra.d) : 0);
    if (lds < route_lds)
        lds = route_lds;
    static std::atomic<size_t> lds_seen{0};
    MOLE_HIP_CHECK(ensure_dynamic_lds(lds_seen, reinterpret_cast<const void *>(&dedup_route_kernel<PER, NORM, WT>), lds));
    const int K = DEDUP_SPLIT_WGS;
    const int tiles = (dd.T + ROUTER_TILE - 1) / ROUTER_TILE;
    int router_wgs = (tiles + ROUTE_GROUPS - 1) / ROUTE_GROUPS;
    const int room = num_cus() - K;     // one workgroup per CU (the dedup's LDS area sizes the launch)
    if (router_wgs > room)
        router_wgs = room > 0 ? room : 1;
    hipLaunchKernelGGL((dedup_route_kernel<PER, NORM, WT>), dim3(K + router_wgs), dim3(DEDUP_THREADS), lds, stream, dd, ra, K);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

template <int PER, bool NORM>
mole_status launch_dedup_route(const DedupArgs &dd, const RouteArgs &ra, hipStream_t stream)
{
    // the transposed weight in LDS when it fits behind the partial products (d = 1024: 66 of 156 KB)
    if (ROUTE_LDS_BYTES + router_wt_bytes(ROUTE_N, ra.d) <= DEDUP_LDS_LIMIT)
        return launch_dedup_route_wt<PER, NORM, true>(dd, ra, stream);
    return launch_dedup_route_wt<PER, NORM, false>(dd, ra, stream);
}

size_t align16_up(size_t n) { return (n + 15) & ~size_t(15); }

}  // namespace

extern "C" size_t mole_dedup_forward_workspace(int T, int64_t V, int N, int L)
{
    if (T < 0 || N < 1 || L < 1)
        return 0;
    return align16_up(mole_dedup_workspace(T, V)) + (size_t)L * T * N * sizeof(float);
}

extern "C" mole_status mole_dedup_forward(const void *table, int64_t table_stride, const int32_t *ids, const void *h,
                                          const void *ln_w, float ln_eps, const void *W_r, const void *shared_out,
                                          const void *residual, void *out, int64_t act_stride, int32_t *uniq,
                                          int32_t *inv, int32_t *n_uniq, int32_t *err_flag, int L, int T, int64_t V,
                                          int d, int N, mole_dtype dtype, void *workspace, size_t workspace_bytes,
                                          void *hip_stream)
{
    clear_error();
    if (T < 0 || L < 1 || V < 1 || d < 1 || N < 1)
        return fail(MOLE_EINVAL, "mole_dedup_forward: bad size (T=%d, L=%d, V=%lld, d=%d, N=%d)", T, L, (long long)V, d, N);
    if (ln_w && residual)
        return fail(MOLE_EINVAL, "mole_dedup_forward: with ln_w the state itself is the residual; residual must be NULL");
    const size_t need = mole_dedup_forward_workspace(T, V, N, L);
    if (!workspace || workspace_bytes < need)
        return fail(MOLE_EWORKSPACE, "mole_dedup_forward: workspace of %zu bytes needed, got %zu", need,
                    workspace ? workspace_bytes : (size_t)0);
    if (!aligned16(workspace))
        return fail(MOLE_EINVAL, "mole_dedup_forward: workspace is not 16-byte aligned");
    const size_t plan_bytes = mole_dedup_workspace(T, V);

    const bool fused = dtype == MOLE_BF16 && N == ROUTE_N && L == 1 && d % 8 == 0 && T > 4 * DEDUP_THREADS &&
                       T <= 16 * DEDUP_THREADS && V <= DEDUP_MAX_V && dedup_split_lds_bytes(T, V) <= DEDUP_LDS_LIMIT &&
                       knob(KNOB_DEDUP_GENERIC) == 0 && knob(KNOB_FWD_TILE) != 2 && knob(KNOB_FWD_GENERIC) != 1 &&
                       knob(KNOB_FWD_RUN) != 1;
    if (!fused) {
        // every other shape: the two calls, one after the other
        mole_status st = mole_dedup_ids(ids, T, V, uniq, inv, n_uniq, err_flag, workspace, plan_bytes, hip_stream);
        if (st != MOLE_OK)
            return st;
        if (ln_w)
            return mole_layer_forward(table, table_stride, ids, nullptr, h, ln_w, ln_eps, W_r, shared_out, out, act_stride,
                                      nullptr, nullptr, err_flag, L, T, V, d, N, dtype, MOLE_FLAG_DEDUP, workspace,
                                      plan_bytes, hip_stream);
        return mole_lookup_forward_layers(table, table_stride, ids, nullptr, h, W_r, shared_out, residual, out, act_stride,
                                          nullptr, nullptr, err_flag, L, T, V, d, N, dtype, MOLE_FLAG_DEDUP, workspace,
                                          plan_bytes, hip_stream);
    }

    if (!table || !ids || !h || !W_r || !out || !uniq || !inv || !n_uniq)
        return fail(MOLE_EINVAL, "mole_dedup_forward: table, ids, h, W_r, out, uniq, inv and n_uniq must not be NULL");
    if (ln_w && !(ln_eps >= 0.f))
        return fail(MOLE_EINVAL, "mole_dedup_forward: ln_eps = %g must be >= 0", (double)ln_eps);
    const void *ptrs[] = {table, h, W_r, shared_out, residual, out, ln_w};
    for (const void *p : ptrs)
        if (p && !aligned16(p))
            return fail(MOLE_EINVAL, "mole_dedup_forward: tensor pointer %p is not 16-byte aligned", p);
    MOLE_ARCH_CHECK("mole_dedup_forward");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int32_t *plan = static_cast<int32_t *>(workspace);
    float *gates = reinterpret_cast<float *>(static_cast<char *>(workspace) + align16_up(plan_bytes));

    const DedupArgs dd{ids, uniq, inv, n_uniq, err_flag, plan, T, (int)V};
    const RouteArgs ra{static_cast<const uint16_t *>(h), static_cast<const uint16_t *>(W_r),
                       static_cast<const uint16_t *>(ln_w), ln_eps, gates, d};
    const int per = (T + DEDUP_THREADS - 1) / DEDUP_THREADS;
    mole_status st;
    if (per <= 8)
        st = ln_w ? launch_dedup_route<8, true>(dd, ra, stream) : launch_dedup_route<8, false>(dd, ra, stream);
    else
        st = ln_w ? launch_dedup_route<16, true>(dd, ra, stream) : launch_dedup_route<16, false>(dd, ra, stream);
    if (st != MOLE_OK)
        return st;
    const TileArgs ta{table, ids, h, W_r, shared_out, residual, out, nullptr, nullptr, err_flag, plan, ln_w, ln_eps,
                      table_stride, act_stride, V, T, d};
    return launch_tile_gather(ta, gates, N, 1, stream);
}
