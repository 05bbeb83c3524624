// mole_shared_ffn_forward: the MoLE layer with its shared expert evaluated inside the call,
//     out = residual + FFN_shared(h) + sum_j g_j * LUT[id, j, :],   g = softmax(h . W_r)
// (Sec. 3.3, inference-layer equation; the "Shared Expert" and "Routed Expert" lines of the inference
// listing).  FFN_shared is read like a routed expert (Sec. 3.4: 4 d D_s flops): two matrices, GELU between.
//
// Three launches:
//   1. router_gates_kernel   gates [T, N] fp32 (router weight in LDS, one wave per token: the router of the
//                            forward kernels)
//   2. GEMM 1 on the matrix cores: hidden = GELU(h . W1^T + b1).  A plain bf16 hidden activation (2^-9) would
//      show in the result at the tolerance the layer is held to, so it is carried as in the LUT build: in fp16
//      (2^-12), with GEMM 2 on the fp16 matrix instruction and W2 converted to fp16 (exact), whenever a bound
//      computed on the device (max |h_t|_2 * max |W1 row|_2 + max |b1|, and max |W2|) rules out fp16 overflow;
//      else as a bf16 hi + lo pair (2^-17) with GEMM 2 over both planes.  Both variants are launched, the one
//      not chosen returns at once (no host synchronisation).
//   3. GEMM 2: hidden . W2^T + b2, whose EPILOGUE adds the residual and the gate-weighted sum of the token's
//      table rows to each output tile before the single rounding: FFN_shared(h) never exists in memory.
// The weights come as a linear layer stores them ([out, in]), which is the K-contiguous form the GEMM
// kernels read, so nothing is transposed per call.
#include "gemm_nt.h"

namespace {
using namespace mole;

constexpr size_t LDS_BYTES_PER_CU = 160 * 1024;

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// gates[t, :] = softmax(h[t, :] . W_r), fp32.  N in {2, 4, 8, 16, 32, 64}.
template <int N>
__global__ __launch_bounds__(256) void router_gates_kernel(const uint16_t *__restrict__ h, const uint16_t *__restrict__ W_r,
                                                            float *__restrict__ gates, float *__restrict__ gates_dbg,
                                                            int T, int d)
{
    extern __shared__ uint4 smem[];
    constexpr int NR = N < 4 ? 4 : N;
    constexpr int LPJ = 64 / NR;
    const int kgroups = d >> 3;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    fill_router_lds<NR, N>(smem, W_r, kgroups, 256);
    __syncthreads();
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        const uint16_t *hrow = h + (int64_t)t * d;
        uint4 h0, h1;
        load_h2<false>(h0, h1, hrow, d, lane);
        const float g = router_gate<NR, false, false, N>(smem, kgroups, hrow, d, lane, h0, h1);
        if ((lane & (LPJ - 1)) == 0 && lane / LPJ < N) {
            gates[(int64_t)t * N + lane / LPJ] = g;
            if (gates_dbg)
                gates_dbg[(int64_t)t * N + lane / LPJ] = g;
        }
    }
}

template <int N>
mole_status launch_router(const uint16_t *h, const uint16_t *W_r, float *gates, float *gates_dbg, int T, int d,
                          hipStream_t st)
{
    const size_t lds = router_lds_bytes(d, N < 4 ? 4 : N);
    static std::atomic<size_t> lds_seen{0};
    MOLE_HIP_CHECK(ensure_dynamic_lds(lds_seen, reinterpret_cast<const void *>(&router_gates_kernel<N>), lds));
    // a workgroup stages the whole router weight: at least 16 tokens each, at most two workgroups per CU
    int64_t blocks = ((int64_t)T + 15) / 16;
    const int64_t cap = (int64_t)num_cus() * 2;
    if (blocks > cap)
        blocks = cap;
    hipLaunchKernelGGL(router_gates_kernel<N>, dim3((unsigned)blocks), dim3(256), lds, st, h, W_r, gates, gates_dbg, T, d);
    return MOLE_OK;
}

struct FfnWs {
    size_t hid, gates, w2f16, ctl, total;
    int64_t ldh;
};

inline FfnWs ffn_ws(int T, int d, int D_s, int N)
{
    FfnWs w;
    w.ldh = D_s + 64;        // rows padded by 128 bytes: tile rows must not all start in one L2 channel
    size_t off = 0;
    w.hid = off;   off += align256((size_t)2 * T * w.ldh * 2);      // bf16 hi and lo planes, or one fp16 plane
    w.gates = off; off += align256((size_t)T * N * 4);
    w.w2f16 = off; off += align256((size_t)d * w.ldh * 2);          // W2 as fp16, rows padded like the hidden planes
    w.ctl = off;   off += 256;                                      // bounds [8] and the chosen mode
    w.total = off;
    return w;
}

mole_status check_args(int T, int64_t rows, int d, int D_s, int N, mole_dtype dtype)
{
    if (dtype != MOLE_BF16)
        return fail(dtype == MOLE_F32 ? MOLE_EUNSUPPORTED : MOLE_EINVAL,
                    "mole_shared_ffn_forward: dtype %d; the call is built for bf16 storage", (int)dtype);
    if (T < 0 || rows < 1 || d < 1 || D_s < 1)
        return fail(MOLE_EINVAL, "mole_shared_ffn_forward: bad size (T=%d, rows=%lld, d=%d, D_s=%d)", T, (long long)rows, d,
                    D_s);
    if (d % BN || D_s % BN)
        return fail(MOLE_EUNSUPPORTED, "mole_shared_ffn_forward: d=%d and D_s=%d must be multiples of %d (matrix-core tiles)",
                    d, D_s, BN);
    if (N != 2 && N != 4 && N != 8 && N != 16 && N != 32 && N != 64)
        return fail(MOLE_EUNSUPPORTED, "mole_shared_ffn_forward: N=%d, built for 2, 4, 8, 16, 32, 64", N);
    if (router_lds_bytes(d, N < 4 ? 4 : N) > LDS_BYTES_PER_CU)
        return fail(MOLE_EUNSUPPORTED, "mole_shared_ffn_forward: router weight of %d x %d does not fit in LDS", d, N);
    return MOLE_OK;
}

}  // namespace

extern "C" size_t mole_shared_ffn_workspace(int T, int d, int D_s, int N)
{
    if (check_args(T, 1, d, D_s, N, MOLE_BF16) != MOLE_OK)
        return 0;
    return ffn_ws(T, d, D_s, N).total;
}

extern "C" mole_status mole_shared_ffn_forward(const void *table, const int32_t *ids, const int32_t *slot, const void *h,
                                               const void *W_r, const void *W1, const void *b1, const void *W2,
                                               const void *b2, const void *residual, void *out, float *gates_dbg,
                                               int32_t *err_flag, int T, int64_t rows, int d, int D_s, int N,
                                               mole_dtype dtype, mole_act act, void *workspace, size_t workspace_bytes,
                                               void *hip_stream)
{
    clear_error();
    const mole_status cs = check_args(T, rows, d, D_s, N, dtype);
    if (cs != MOLE_OK)
        return cs;
    if (act != MOLE_GELU_ERF && act != MOLE_GELU_TANH)
        return fail(MOLE_EINVAL, "mole_shared_ffn_forward: unknown activation %d", (int)act);
    if (T == 0)
        return MOLE_OK;
    if (!table || !ids || !h || !W_r || !W1 || !W2 || !out)
        return fail(MOLE_EINVAL, "mole_shared_ffn_forward: table, ids, h, W_r, W1, W2 and out must not be NULL");
    const void *ptrs[] = {table, h, W_r, W1, b1, W2, b2, residual, out, workspace};
    for (const void *p : ptrs)
        if (p && !aligned16(p))
            return fail(MOLE_EINVAL, "mole_shared_ffn_forward: pointer %p is not 16-byte aligned", p);
    const FfnWs lay = ffn_ws(T, d, D_s, N);
    if (!workspace || workspace_bytes < lay.total)
        return fail(MOLE_EWORKSPACE, "mole_shared_ffn_forward: workspace of %zu bytes needed, got %zu", lay.total,
                    workspace ? workspace_bytes : (size_t)0);
    MOLE_ARCH_CHECK("mole_shared_ffn_forward");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    uint16_t *hid = reinterpret_cast<uint16_t *>(ws + lay.hid);
    float *gates = reinterpret_cast<float *>(ws + lay.gates);
    const uint16_t *hp = static_cast<const uint16_t *>(h), *wr = static_cast<const uint16_t *>(W_r);

    mole_status rs = MOLE_OK;
    // large batches at N = 32: the router as a product on the matrix pipe (steps 1 and 2 of the tile kernel:
    // 16384 tokens 8 us against 31 us)
    const bool tile_router = N == 32 && T >= 4096;
    if (tile_router) {
        rs = launch_tile_router(h, W_r, nullptr, 0.f, gates, T, d, N, 1, 0, st);
        if (rs == MOLE_OK && gates_dbg)
            MOLE_HIP_CHECK(hipMemcpyAsync(gates_dbg, gates, (size_t)T * N * sizeof(float), hipMemcpyDeviceToDevice, st));
    } else
    switch (N) {
    case 2: rs = launch_router<2>(hp, wr, gates, gates_dbg, T, d, st); break;
    case 4: rs = launch_router<4>(hp, wr, gates, gates_dbg, T, d, st); break;
    case 8: rs = launch_router<8>(hp, wr, gates, gates_dbg, T, d, st); break;
    case 16: rs = launch_router<16>(hp, wr, gates, gates_dbg, T, d, st); break;
    case 32: rs = launch_router<32>(hp, wr, gates, gates_dbg, T, d, st); break;
    default: rs = launch_router<64>(hp, wr, gates, gates_dbg, T, d, st); break;
    }
    if (rs != MOLE_OK)
        return rs;

    // format of the hidden activation, chosen on the device: fp16 if it provably cannot overflow, else bf16 hi + lo
    unsigned *bound = reinterpret_cast<unsigned *>(ws + lay.ctl);
    int *mode = reinterpret_cast<int *>(ws + lay.ctl) + 8;
    uint16_t *w2f16 = reinterpret_cast<uint16_t *>(ws + lay.w2f16);
    const uint16_t *w1 = static_cast<const uint16_t *>(W1), *w2 = static_cast<const uint16_t *>(W2);
    const unsigned cap = (unsigned)num_cus() * 8;
    auto blocks16 = [&](int64_t rows_) { return (unsigned)((rows_ + 15) / 16 < cap ? (rows_ + 15) / 16 : cap); };
    hipLaunchKernelGGL(bound_clear_kernel, dim3(1), dim3(64), 0, st, bound);
    hipLaunchKernelGGL(row_sumsq_max_kernel, dim3(blocks16(T)), dim3(256), 0, st, hp, (int64_t)T, d, d, bound + 0);
    hipLaunchKernelGGL(row_sumsq_max_kernel, dim3(blocks16(D_s)), dim3(256), 0, st, w1, (int64_t)D_s, d, d, bound + 1);
    if (b1)
        hipLaunchKernelGGL(abs_max_kernel, dim3(16), dim3(256), 0, st, static_cast<const uint16_t *>(b1), (int64_t)D_s,
                           bound + 2);
    // eight 16-byte pieces per thread: every workgroup ends with a look at one word of memory, and two thousand of
    // those in a row cost more than the 8 MB read
    const int64_t w2_blocks = ((int64_t)d * D_s / 8 + 2047) / 2048;
    hipLaunchKernelGGL(abs_max_kernel, dim3((unsigned)(w2_blocks < cap ? w2_blocks : cap)), dim3(256), 0, st, w2,
                       (int64_t)d * D_s, bound + 3);
    const int forced = knob(KNOB_BUILD_HIDDEN) == 1 ? MODE_F16 : (knob(KNOB_BUILD_HIDDEN) == 2 ? MODE_SPLIT : 0);
    hipLaunchKernelGGL(choose_mode_kernel, dim3(1), dim3(64), 0, st, bound, mode, forced);
    hipLaunchKernelGGL(bf16_to_f16_rows_kernel, dim3(cap), dim3(256), 0, st, w2, w2f16, (int64_t)d, D_s, (int)lay.ldh);

    // GEMM 1: hidden = GELU(h . W1^T + b1); GEMM 2's epilogue finishes the layer.  fp16 variant, then hi + lo variant.
    GemmArgs g1{};
    g1.A = hp; g1.lda = d; g1.a_planes = 1;
    g1.Bt = w1; g1.ldb = d;
    g1.bias = static_cast<const uint16_t *>(b1);
    g1.C = hid; g1.ldc = lay.ldh;
    g1.M = T; g1.Nn = D_s; g1.K = d; g1.act = (int)act; g1.mode = mode;
    GemmArgs g2{};
    g2.A = hid; g2.lda = lay.ldh;
    g2.bias = static_cast<const uint16_t *>(b2);
    g2.C = static_cast<uint16_t *>(out); g2.ldc = d;
    g2.M = T; g2.Nn = d; g2.K = D_s; g2.epilogue = EPI_LOOKUP; g2.act = (int)act; g2.mode = mode;
    g2.table = static_cast<const uint16_t *>(table); g2.rowsrc = slot ? slot : ids; g2.gates = gates;
    g2.residual = static_cast<const uint16_t *>(residual); g2.table_rows = rows; g2.n_experts = N; g2.err_flag = err_flag;
    g2.lookup_first = knob(KNOB_FFN_GATHER_LAST) != 1;

    g1.epilogue = EPI_GELU_F16; g1.run_mode = MODE_F16; g1.c_plane_stride = 0;
    if (mole_status e = launch_gemm<EPI_GELU_F16, false>(g1, 1, st))
        return e;
    g2.run_mode = MODE_F16; g2.a_planes = 1; g2.a_plane_stride = 0; g2.Bt = w2f16; g2.ldb = lay.ldh;
    if (mole_status e = launch_gemm<EPI_LOOKUP, true>(g2, 1, st))
        return e;

    g1.epilogue = EPI_GELU_SPLIT; g1.run_mode = MODE_SPLIT; g1.c_plane_stride = (int64_t)T * lay.ldh;
    if (mole_status e = launch_gemm<EPI_GELU_SPLIT, false>(g1, 1, st))
        return e;
    g2.run_mode = MODE_SPLIT; g2.a_planes = 2; g2.a_plane_stride = (int64_t)T * lay.ldh; g2.Bt = w2; g2.ldb = D_s;
    if (mole_status e = launch_gemm<EPI_LOOKUP, false>(g2, 1, st))
        return e;
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}
