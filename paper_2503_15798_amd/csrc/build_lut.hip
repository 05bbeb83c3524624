// mole_build_lut: the re-parameterization LUT[v, j, :] = FFN_j(Embedding(v)).
//
// Paper: Sec. 3.3, LUT entry equation (the experts are run once over every row of the embedding
// matrix), with the expert taken as a two-matrix FFN (Sec. 3.4: 4dD flops, 2dD parameters) and
// GELU; optionally the RMSNorm the training listing applies to the embedding states first.
//
// This is the one dense contraction of the library (4*V*d*D*N flop, 1.35e13 for one 410M
// layer), so it runs on the matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//   GEMM 1:  A = E[v, :]           B = W1_j     epilogue: + b1, GELU, stored as one fp16 plane
//                                                (or a bf16 high and a bf16 low plane, see below)
//   GEMM 2:  A = hidden of GEMM 1   B = W2_j     epilogue: + b2, round to bf16, stored
//                                                straight into LUT[v, j, :] (row stride N*d)
// A bf16 hidden activation would carry a rounding error of 2^-9, which shows in the result (the
// table's own final rounding is the only one the tolerance budgets for).  Two ways around it:
//   * fp16 hidden activation (2^-12) and GEMM 2 on the fp16 MFMA with W2 converted to fp16 (exact:
//     fp16 has the wider significand).  Used whenever it provably cannot overflow: a bound kernel
//     computes max_v |x_v|_2 * max_col |W1 col|_2 + max |b1| >= every pre-activation (Cauchy-Schwarz),
//     and |GELU(a)| <= |a|; the bound and max |W2| must stay below 60000.
//   * otherwise the activation is carried as a bf16 high part plus a bf16 low part (2^-17) and GEMM 2
//     runs over both planes: 1.5 x the MFMA work, no range limit.
// The choice is taken on the device (no host synchronisation): both variants of each GEMM are
// launched and the one whose mode is not selected returns at once.
// Both weight matrices are first transposed into K-contiguous form so that A and B tiles are
// fetched the same way (16-byte pieces along K) and match the MFMA operand layout directly.
//
// Two GEMM kernels.  Column counts that are multiples of 256 take the 256 x 256 kernel fed by direct
// global -> LDS loads (described at gemm_nt_direct_kernel).  Other shapes take the 256 x 128 kernel below:
// workgroup of 4 waves (2 x 2), each wave 128 x 64 = 4 x 2 MFMA tiles, K step 64 through LDS with 16
// bytes of row padding (conflict-free 16-byte reads), next K tile prefetched into registers while the
// current one is multiplied.
#include "gemm_nt.h"

#include <stdlib.h>
#include <string.h>

namespace {
using namespace mole;

// dst[b][c][r] = src[b][r][c]   (bf16, 32 x 32 tiles through LDS).  dst16 (nullable) receives the same
// transposed matrix converted to fp16 (exact for |x| in [2^-14, 65504]; smaller values become fp16
// subnormals, absolute error below 3e-8).
__global__ __launch_bounds__(256) void transpose_kernel(const uint16_t *__restrict__ src,
                                                         uint16_t *__restrict__ dst,
                                                         uint16_t *__restrict__ dst16, int R, int Cn, int dst_ld)
{
    __shared__ uint16_t tile[32][33];
    const int64_t base = (int64_t)blockIdx.z * R * Cn;
    const int64_t dbase = (int64_t)blockIdx.z * Cn * dst_ld;     // dst rows (Cn of them) are dst_ld apart
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < R && c0 + tx < Cn)
            tile[i][tx] = src[base + (int64_t)(r0 + i) * Cn + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < Cn && r0 + tx < R) {
            const uint16_t x = tile[tx][i];
            dst[dbase + (int64_t)(c0 + i) * dst_ld + r0 + tx] = x;
            if (dst16)
                dst16[dbase + (int64_t)(c0 + i) * dst_ld + r0 + tx] = __builtin_bit_cast(uint16_t, (_Float16)bf16_to_f32(x));
        }
}

// The same for R and Cn multiples of 64: 64 x 64 tiles, 16-byte accesses on both sides (128 contiguous
// bytes per row segment), the transposition itself in 2-byte LDS reads.
__global__ __launch_bounds__(256) void transpose64_kernel(const uint16_t *__restrict__ src,
                                                           uint16_t *__restrict__ dst,
                                                           uint16_t *__restrict__ dst16, int R, int Cn, int dst_ld)
{
    __shared__ __attribute__((aligned(16))) uint16_t tile[64][72];      // rows of 144 bytes: 16-byte aligned
    const int64_t base = (int64_t)blockIdx.z * R * Cn;
    const int64_t dbase = (int64_t)blockIdx.z * Cn * dst_ld;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int p = threadIdx.x + u * 256;            // piece: row p / 8, columns 8 * (p % 8) ..+7
        const int r = p >> 3, cp = (p & 7) * 8;
        *reinterpret_cast<uint4 *>(&tile[r][cp]) =
            *reinterpret_cast<const uint4 *>(src + base + (int64_t)(r0 + r) * Cn + c0 + cp);
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int p = threadIdx.x + u * 256;            // output piece: row c = p / 8, rows-of-src 8 * (p % 8) ..+7
        const int c = p >> 3, rp = (p & 7) * 8;
        uint16_t x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            x[e] = tile[rp + e][c];
        const int64_t o = dbase + (int64_t)(c0 + c) * dst_ld + r0 + rp;
        *reinterpret_cast<uint4 *>(dst + o) =
            make_uint4(x[0] | (uint32_t)x[1] << 16, x[2] | (uint32_t)x[3] << 16, x[4] | (uint32_t)x[5] << 16,
                       x[6] | (uint32_t)x[7] << 16);
        if (dst16) {
            uint16_t hx[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                hx[e] = __builtin_bit_cast(uint16_t, (_Float16)bf16_to_f32(x[e]));
            *reinterpret_cast<uint4 *>(dst16 + o) =
                make_uint4(hx[0] | (uint32_t)hx[1] << 16, hx[2] | (uint32_t)hx[3] << 16, hx[4] | (uint32_t)hx[5] << 16,
                           hx[6] | (uint32_t)hx[7] << 16);
        }
    }
}

// dst[b][c][r] = src[b][r][c] for N matrices of R x Cn: the 64 x 64 kernel when shapes and row stride allow
void launch_transpose(const uint16_t *src, uint16_t *dst, uint16_t *dst16, int R, int Cn, int dst_ld, int N, hipStream_t st)
{
    if (R % 64 == 0 && Cn % 64 == 0 && dst_ld % 8 == 0)
        hipLaunchKernelGGL(transpose64_kernel, dim3(Cn / 64, R / 64, N), dim3(256), 0, st, src, dst, dst16, R, Cn, dst_ld);
    else
        hipLaunchKernelGGL(transpose_kernel, dim3(Cn / 32, R / 32, N), dim3(256), 0, st, src, dst, dst16, R, Cn, dst_ld);
}

// RMSNorm of the embedding rows, written as a bf16 hi plane and a bf16 lo plane.  One wave per row.
__global__ __launch_bounds__(256) void rmsnorm_split_kernel(const uint16_t *__restrict__ E,
                                                             const uint16_t *__restrict__ w, float eps,
                                                             uint16_t *__restrict__ hi, uint16_t *__restrict__ lo,
                                                             int64_t V, int d)
{
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (v >= V)
        return;
    float ss = 0.f;
    for (int k = lane; k < d; k += 64) {
        const float x = bf16_to_f32(E[v * d + k]);
        ss = fmaf(x, x, ss);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1)
        ss += __shfl_xor(ss, o);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int k = lane; k < d; k += 64) {
        const float y = bf16_to_f32(E[v * d + k]) * inv * bf16_to_f32(w[k]);
        const uint32_t h = f32_to_bf16_bits(y);
        hi[v * d + k] = (uint16_t)h;
        lo[v * d + k] = (uint16_t)f32_to_bf16_bits(y - __uint_as_float(h << 16));
    }
}

// ------------------------------------------------------------------------------------------
// Plain path (fp32 storage, or bf16 shapes the MFMA tiles do not cover): fp32 arithmetic,
// one thread per output element, hidden activations kept in fp32.
// ------------------------------------------------------------------------------------------
template <typename E> __device__ __forceinline__ float ldv(const E *p);
template <> __device__ __forceinline__ float ldv<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ldv<uint16_t>(const uint16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void stv(float *p, float v) { *p = v; }
__device__ __forceinline__ void stv(uint16_t *p, float v) { *p = (uint16_t)f32_to_bf16_bits(v); }

template <typename E>
__global__ __launch_bounds__(256) void plain_norm_kernel(const E *__restrict__ Em, const E *__restrict__ w, float eps,
                                                          float *__restrict__ X, int64_t V, int d)
{
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (v >= V)
        return;
    float ss = 0.f;
    for (int k = lane; k < d; k += 64) {
        const float x = ldv(Em + v * d + k);
        ss = fmaf(x, x, ss);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1)
        ss += __shfl_xor(ss, o);
    const float inv = w ? 1.0f / sqrtf(ss / (float)d + eps) : 1.0f;
    for (int k = lane; k < d; k += 64)
        X[v * d + k] = ldv(Em + v * d + k) * inv * (w ? ldv(w + k) : 1.0f);
}

// H[v - v0, j, m] = GELU(sum_k X[v,k] W1[j,k,m] + b1[j,m]) for v in [v0, v0 + nv)
template <typename E>
__global__ __launch_bounds__(256) void plain_hidden_kernel(const float *__restrict__ X, const E *__restrict__ W1,
                                                            const E *__restrict__ b1, float *__restrict__ H,
                                                            int64_t v0, int nv, int d, int D, int N, int act)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)nv * N * D;
    if (idx >= total)
        return;
    const int m = (int)(idx % D);
    const int j = (int)((idx / D) % N);
    const int64_t v = v0 + idx / ((int64_t)D * N);
    float s = 0.f;
    for (int k = 0; k < d; ++k)
        s = fmaf(X[v * d + k], ldv(W1 + ((int64_t)j * d + k) * D + m), s);
    if (b1)
        s += ldv(b1 + (int64_t)j * D + m);
    H[idx] = gelu_f(s, act);
}

template <typename E>
__global__ __launch_bounds__(256) void plain_out_kernel(const float *__restrict__ H, const E *__restrict__ W2,
                                                         const E *__restrict__ b2, E *__restrict__ LUT,
                                                         int64_t v0, int nv, int d, int D, int N)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)nv * N * d;
    if (idx >= total)
        return;
    const int c = (int)(idx % d);
    const int j = (int)((idx / d) % N);
    const int64_t vl = idx / ((int64_t)d * N);
    const float *h = H + (vl * N + j) * D;
    float s = 0.f;
    for (int m = 0; m < D; ++m)
        s = fmaf(h[m], ldv(W2 + ((int64_t)j * D + m) * d + c), s);
    if (b2)
        s += ldv(b2 + (int64_t)j * d + c);
    stv(LUT + ((v0 + vl) * N + j) * d + c, s);
}

// ---- workspace layout --------------------------------------------------------------------
constexpr int64_t SLAB_ROWS = 16384;   // vocabulary rows whose hidden activations are resident at once

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline bool mfma_shape(int64_t V, int d, int D, mole_dtype dt)
{
    (void)V;
    return dt == MOLE_BF16 && d % BN == 0 && D % BN == 0 && d % BK == 0 && D % BK == 0;
}

// Rows of the K-contiguous operands the library lays out itself are padded by 128 bytes: with a
// power-of-two row stride every row of a tile starts in the same L2 channel, and because all workgroups
// walk K in step the whole chip would queue on one or two channels at a time.
constexpr int LD_PAD = 64;   // elements

struct BuildWs {
    size_t w1t, w2t, w2t16, xn, hid, ctl, total;
    int64_t slab;
};

inline BuildWs build_ws(int64_t V, int d, int D, int N, mole_dtype dt)
{
    BuildWs w;
    w.slab = V < SLAB_ROWS ? V : SLAB_ROWS;
    size_t off = 0;
    if (mfma_shape(V, d, D, dt)) {
        w.w1t = off; off += align256((size_t)N * D * (d + LD_PAD) * 2);
        w.w2t = off; off += align256((size_t)N * d * (D + LD_PAD) * 2);
        w.w2t16 = off; off += align256((size_t)N * d * (D + LD_PAD) * 2);          // W2^T as fp16
        w.xn = off;  off += align256((size_t)2 * V * d * 2);                       // hi + lo planes (norm only)
        w.hid = off; off += align256((size_t)N * 2 * w.slab * (D + LD_PAD) * 2);   // hi + lo planes per expert, or one fp16 plane
        w.ctl = off; off += 256;                                         // bounds [8] and the chosen mode
    } else {
        w.w1t = w.w2t = w.w2t16 = w.ctl = 0;
        w.xn = off;  off += align256((size_t)V * d * 4);
        w.hid = off; off += align256((size_t)w.slab * N * D * 4);
    }
    w.total = off;
    return w;
}

// the knob MOLE_BUILD_HIDDEN (1 = f16, 2 = split) forces the format of the hidden activation (tests, experiments)
inline int forced_mode()
{
    const int v = knob(KNOB_BUILD_HIDDEN);
    return v == 1 ? MODE_F16 : (v == 2 ? MODE_SPLIT : 0);
}

template <typename E>
mole_status build_plain(const void *Em, const void *W1, const void *b1, const void *W2, const void *b2,
                        const void *norm_w, float eps, void *LUT, int64_t V, int d, int D, int N, int act,
                        char *ws, const BuildWs &lay, hipStream_t st)
{
    float *X = reinterpret_cast<float *>(ws + lay.xn);
    float *H = reinterpret_cast<float *>(ws + lay.hid);
    hipLaunchKernelGGL(plain_norm_kernel<E>, dim3((unsigned)((V + 3) / 4)), dim3(256), 0, st,
                       static_cast<const E *>(Em), static_cast<const E *>(norm_w), eps, X, V, d);
    for (int64_t v0 = 0; v0 < V; v0 += lay.slab) {
        const int nv = (int)((V - v0) < lay.slab ? (V - v0) : lay.slab);
        const int64_t th = (int64_t)nv * N * D, to = (int64_t)nv * N * d;
        hipLaunchKernelGGL(plain_hidden_kernel<E>, dim3((unsigned)((th + 255) / 256)), dim3(256), 0, st, X,
                           static_cast<const E *>(W1), static_cast<const E *>(b1), H, v0, nv, d, D, N, act);
        hipLaunchKernelGGL(plain_out_kernel<E>, dim3((unsigned)((to + 255) / 256)), dim3(256), 0, st, H,
                           static_cast<const E *>(W2), static_cast<const E *>(b2), static_cast<E *>(LUT), v0, nv,
                           d, D, N);
    }
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

mole_status build_mfma(const void *Em, const void *W1, const void *b1, const void *W2, const void *b2,
                       const void *norm_w, float eps, void *LUT, int64_t V, int d, int D, int N, int act,
                       char *ws, const BuildWs &lay, hipStream_t st)
{
    uint16_t *w1t = reinterpret_cast<uint16_t *>(ws + lay.w1t);       // [N, D, d]
    uint16_t *w2t = reinterpret_cast<uint16_t *>(ws + lay.w2t);       // [N, d, D]
    uint16_t *w2t16 = reinterpret_cast<uint16_t *>(ws + lay.w2t16);   // [N, d, D] fp16
    uint16_t *xn = reinterpret_cast<uint16_t *>(ws + lay.xn);
    uint16_t *hid = reinterpret_cast<uint16_t *>(ws + lay.hid);       // [N][2][slab, D] bf16 or [N][slab, D] fp16
    unsigned *bound = reinterpret_cast<unsigned *>(ws + lay.ctl);
    int *mode = reinterpret_cast<int *>(ws + lay.ctl) + 8;
    const int ldw1 = d + LD_PAD, ldh = D + LD_PAD;      // row strides of W1^T, and of W2^T and the hidden planes
    launch_transpose(static_cast<const uint16_t *>(W1), w1t, nullptr, d, D, ldw1, N, st);
    launch_transpose(static_cast<const uint16_t *>(W2), w2t, w2t16, D, d, ldh, N, st);
    const uint16_t *X = static_cast<const uint16_t *>(Em);
    int x_planes = 1;
    if (norm_w) {
        hipLaunchKernelGGL(rmsnorm_split_kernel, dim3((unsigned)((V + 3) / 4)), dim3(256), 0, st, X,
                           static_cast<const uint16_t *>(norm_w), eps, xn, xn + V * d, V, d);
        X = xn;
        x_planes = 2;
    }
    // format of the hidden activation: fp16 if it provably cannot overflow, else bf16 hi + lo
    const unsigned cap = (unsigned)num_cus() * 8;
    hipLaunchKernelGGL(bound_clear_kernel, dim3(1), dim3(64), 0, st, bound);
    // (a workgroup takes 16 rows per round: 4 waves x 4 rows)
    hipLaunchKernelGGL(row_sumsq_max_kernel, dim3((unsigned)((V + 15) / 16 < cap ? (V + 15) / 16 : cap)), dim3(256), 0, st,
                       X, V, d, d, bound + 0);
    const int64_t w1rows = (int64_t)N * D;
    hipLaunchKernelGGL(row_sumsq_max_kernel, dim3((unsigned)((w1rows + 15) / 16 < cap ? (w1rows + 15) / 16 : cap)),
                       dim3(256), 0, st, w1t, w1rows, d, ldw1, bound + 1);
    if (b1)
        hipLaunchKernelGGL(abs_max_kernel, dim3(64), dim3(256), 0, st, static_cast<const uint16_t *>(b1),
                           (int64_t)N * D, bound + 2);
    hipLaunchKernelGGL(abs_max_kernel, dim3(cap), dim3(256), 0, st, static_cast<const uint16_t *>(W2),
                       (int64_t)N * d * D, bound + 3);
    hipLaunchKernelGGL(choose_mode_kernel, dim3(1), dim3(64), 0, st, bound, mode, forced_mode());
    for (int64_t v0 = 0; v0 < V; v0 += lay.slab) {
        const int nv = (int)((V - v0) < lay.slab ? (V - v0) : lay.slab);
        GemmArgs g1{};
        g1.A = X + v0 * d; g1.lda = d; g1.a_plane_stride = V * (int64_t)d; g1.a_batch_stride = 0;
        g1.a_planes = x_planes;
        g1.Bt = w1t; g1.ldb = ldw1; g1.b_batch_stride = (int64_t)D * ldw1;
        g1.bias = static_cast<const uint16_t *>(b1); g1.bias_batch_stride = D;
        g1.C = hid; g1.ldc = ldh; g1.M = nv; g1.Nn = D; g1.K = d; g1.act = act; g1.mode = mode;
        GemmArgs g2{};
        g2.lda = ldh; g2.ldb = ldh; g2.b_batch_stride = (int64_t)d * ldh;
        g2.A = hid;
        g2.bias = static_cast<const uint16_t *>(b2); g2.bias_batch_stride = d;
        g2.C = static_cast<uint16_t *>(LUT) + v0 * N * d; g2.ldc = (int64_t)N * d; g2.c_plane_stride = 0;
        g2.c_batch_stride = d;
        g2.M = nv; g2.Nn = d; g2.K = D; g2.epilogue = EPI_STORE; g2.act = act; g2.mode = mode;

        // fp16 mode: one plane, GEMM 2 on the fp16 MFMA
        g1.epilogue = EPI_GELU_F16; g1.run_mode = MODE_F16;
        g1.c_plane_stride = 0; g1.c_batch_stride = lay.slab * ldh;
        if (mole_status e = launch_gemm<EPI_GELU_F16, false>(g1, N, st))
            return e;
        g2.run_mode = MODE_F16; g2.Bt = w2t16; g2.a_planes = 1;
        g2.a_plane_stride = 0; g2.a_batch_stride = lay.slab * ldh;
        if (mole_status e = launch_gemm<EPI_STORE, true>(g2, N, st))
            return e;

        // split mode: bf16 hi and lo planes, GEMM 2 over both
        g1.epilogue = EPI_GELU_SPLIT; g1.run_mode = MODE_SPLIT;
        g1.c_plane_stride = lay.slab * ldh; g1.c_batch_stride = 2 * lay.slab * ldh;
        if (mole_status e = launch_gemm<EPI_GELU_SPLIT, false>(g1, N, st))
            return e;
        g2.run_mode = MODE_SPLIT; g2.Bt = w2t; g2.a_planes = 2;
        g2.a_plane_stride = lay.slab * ldh; g2.a_batch_stride = 2 * lay.slab * ldh;
        if (mole_status e = launch_gemm<EPI_STORE, false>(g2, N, st))
            return e;
    }
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

mole_status check_build_args(int64_t V, int d, int D, int N, mole_dtype dtype)
{
    if (dtype != MOLE_F32 && dtype != MOLE_BF16)
        return fail(MOLE_EINVAL, "mole_build_lut: unknown dtype %d", (int)dtype);
    if (V < 1 || d < 1 || D < 1)
        return fail(MOLE_EINVAL, "mole_build_lut: bad size (V=%lld, d=%d, D=%d)", (long long)V, d, D);
    if (N < 1 || N > 64)
        return fail(MOLE_EUNSUPPORTED, "mole_build_lut: N=%d outside 1..64", N);
    if (d % 16 || D % 16)
        return fail(MOLE_EUNSUPPORTED, "mole_build_lut: d=%d and D=%d must be multiples of 16", d, D);
    return MOLE_OK;
}

}  // namespace

extern "C" size_t mole_build_lut_workspace(int64_t V, int d, int D, int N, mole_dtype dtype)
{
    if (check_build_args(V, d, D, N, dtype) != MOLE_OK)
        return 0;
    return build_ws(V, d, D, N, dtype).total;
}

extern "C" mole_status mole_build_lut(const void *E, const void *W1, const void *b1, const void *W2,
                                      const void *b2, const void *norm_w, float norm_eps, void *LUT, int64_t V,
                                      int d, int D, int N, mole_dtype dtype, mole_act act, void *workspace,
                                      size_t workspace_bytes, void *hip_stream)
{
    clear_error();
    const mole_status st = check_build_args(V, d, D, N, dtype);
    if (st != MOLE_OK)
        return st;
    if (act != MOLE_GELU_ERF && act != MOLE_GELU_TANH)
        return fail(MOLE_EINVAL, "mole_build_lut: unknown activation %d", (int)act);
    if (!E || !W1 || !W2 || !LUT)
        return fail(MOLE_EINVAL, "mole_build_lut: E, W1, W2 and LUT must not be NULL");
    const void *ptrs[] = {E, W1, b1, W2, b2, norm_w, LUT, workspace};
    for (const void *p : ptrs)
        if (p && !aligned16(p))
            return fail(MOLE_EINVAL, "mole_build_lut: pointer %p is not 16-byte aligned", p);
    const BuildWs lay = build_ws(V, d, D, N, dtype);
    if (!workspace || workspace_bytes < lay.total)
        return fail(MOLE_EWORKSPACE, "mole_build_lut: workspace of %zu bytes needed, got %zu", lay.total,
                    workspace ? workspace_bytes : (size_t)0);
    MOLE_ARCH_CHECK("mole_build_lut");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    if (mfma_shape(V, d, D, dtype))
        return build_mfma(E, W1, b1, W2, b2, norm_w, norm_eps, LUT, V, d, D, N, (int)act, ws, lay, stream);
    if (dtype == MOLE_F32)
        return build_plain<float>(E, W1, b1, W2, b2, norm_w, norm_eps, LUT, V, d, D, N, (int)act, ws, lay, stream);
    return build_plain<uint16_t>(E, W1, b1, W2, b2, norm_w, norm_eps, LUT, V, d, D, N, (int)act, ws, lay, stream);
}
