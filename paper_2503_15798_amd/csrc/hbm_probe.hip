// hbm_probe: what this GPU delivers for the forward kernel's traffic pattern, without its arithmetic.
//
// A stand-alone measurement program (not part of libmole.so).  It reads N rows of d bf16 per token from
// random row blocks of an 8 GiB buffer exactly as the forward kernel does (one wave per token, 16-byte
// loads, two 512-column chunks), optionally together with the kernel's activation traffic (h, shared
// read; out written), and prints TB/s for each mix.  The numbers bound what the fused kernel can reach:
// they are quoted in profiles/hbm_ceilings.md.
//
//   hipcc --offload-arch=gfx950 -O3 -o hbm_probe hbm_probe.hip && ./hbm_probe
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);    \
            exit(1);                                                                 \
        }                                                                            \
    } while (0)

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
__device__ inline uint4 ld(const uint4 *p, bool nt)
{
    if (!nt)
        return *p;
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ inline void st(uint4 *p, uint4 o, bool nt)
{
    if (!nt) {
        *p = o;
        return;
    }
    const u32x4 v = {o.x, o.y, o.z, o.w};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
}

enum { LOAD_H = 1, LOAD_SHARED = 2, STORE_OUT = 4, NT_STORE = 8, NT_ACT = 16, NT_ROWS = 32 };

// d = 1024 bf16 = 128 uint4 per row; a token reads N rows from row block rows[t]
template <int N, int MIX>
__global__ __launch_bounds__(256) void pattern(const uint4 *__restrict__ tab, const int *__restrict__ rows, int T,
                                               const uint4 *__restrict__ h, const uint4 *__restrict__ sh,
                                               uint4 *__restrict__ out, uint32_t *sink)
{
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nw = gridDim.x * 4;
    uint32_t acc = 0;
    for (int t = wave; t < T; t += nw) {
        const uint4 *q = tab + (size_t)rows[t] * (N * 128);
        uint4 hv0 = make_uint4(0, 0, 0, 0), hv1 = hv0;
        if (MIX & LOAD_H) {
            hv0 = ld(h + (size_t)t * 128 + lane, MIX & NT_ACT);
            hv1 = ld(h + (size_t)t * 128 + 64 + lane, MIX & NT_ACT);
        }
        for (int c = 0; c < 2; ++c) {
            uint4 v[N];
            uint4 s0 = make_uint4(0, 0, 0, 0);
            if (MIX & LOAD_SHARED)
                s0 = ld(sh + (size_t)t * 128 + c * 64 + lane, MIX & NT_ACT);
#pragma unroll
            for (int j = 0; j < N; ++j)
                v[j] = ld(q + j * 128 + c * 64 + lane, MIX & NT_ROWS);
#pragma unroll
            for (int j = 0; j < N; ++j)
                acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
            uint4 o = s0;
            o.x ^= acc ^ hv0.x ^ hv1.y;
            if (MIX & STORE_OUT)
                st(out + (size_t)t * 128 + c * 64 + lane, o, MIX & NT_STORE);
            else
                acc += s0.y ^ hv0.z ^ hv1.w;   // keep every load alive without cancelling acc
        }
    }
    if (acc == 0x12345678u)
        *sink = acc;
}

// The same row traffic through direct global -> LDS loads (global_load_lds_dwordx4): a wave-wide load
// drops 1 KiB (one 512-column chunk of one row) into the wave's LDS buffer; the N rows of a chunk are then
// read back from LDS.  BUFS = 2: the next chunk travels while the current one is read.
template <int N, int WPB, int BUFS, int MIX>
__global__ __launch_bounds__(WPB * 64) void pattern_dma(const uint4 *__restrict__ tab, const int *__restrict__ rows,
                                                        int T, const uint4 *__restrict__ h,
                                                        const uint4 *__restrict__ sh, uint4 *__restrict__ out,
                                                        uint32_t *sink)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int wib = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wave = blockIdx.x * WPB + wib;
    const int nw = gridDim.x * WPB;
    unsigned char *buf = lds + (size_t)wib * BUFS * N * 1024;
    auto issue = [&](int t, int c, int b) {
        const uint4 *q = tab + (size_t)rows[t] * (N * 128) + c * 64 + lane;
#pragma unroll
        for (int j = 0; j < N; ++j)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(q + j * 128),
                                             (__attribute__((address_space(3))) void *)(buf + (b * N + j) * 1024),
                                             16, 0, 0);
    };
    uint32_t acc = 0;
    int item = 0;                       // chunks processed by this wave (selects the buffer)
    if (BUFS == 2 && wave < T)
        issue(wave, 0, 0);
    for (int t = wave; t < T; t += nw) {
        uint4 hv0 = make_uint4(0, 0, 0, 0), hv1 = hv0;
        if (MIX & LOAD_H) {
            hv0 = ld(h + (size_t)t * 128 + lane, MIX & NT_ACT);
            hv1 = ld(h + (size_t)t * 128 + 64 + lane, MIX & NT_ACT);
        }
        for (int c = 0; c < 2; ++c, ++item) {
            const int b = BUFS == 2 ? (item & 1) : 0;
            uint4 s0 = make_uint4(0, 0, 0, 0);
            if (MIX & LOAD_SHARED)
                s0 = ld(sh + (size_t)t * 128 + c * 64 + lane, MIX & NT_ACT);
            if (BUFS == 2) {
                // next chunk (or the next token's first chunk) into the other buffer
                const int tn = c == 0 ? t : t + nw, cn = c == 0 ? 1 : 0;
                if (tn < T)
                    issue(tn, cn, b ^ 1);
                // the loads issued before those N (and the activation loads) have landed
                if (tn < T)
                    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
                else
                    __builtin_amdgcn_s_waitcnt(0x0F70);
            } else {
                issue(t, c, 0);
                __builtin_amdgcn_s_waitcnt(0x0F70);
            }
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const uint4 v = *reinterpret_cast<const uint4 *>(buf + (b * N + j) * 1024 + lane * 16);
                acc ^= v.x ^ v.y ^ v.z ^ v.w;
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);      // LDS reads done before the buffer is refilled
            uint4 o = s0;
            o.x ^= acc ^ hv0.x ^ hv1.y;
            if (MIX & STORE_OUT)
                st(out + (size_t)t * 128 + c * 64 + lane, o, MIX & NT_STORE);
            else
                acc += s0.y ^ hv0.z ^ hv1.w;
        }
    }
    if (acc == 0x12345678u)
        *sink = acc;
}

__global__ void stream_read(const uint4 *__restrict__ p, size_t n16, uint32_t *sink)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = p[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u)
        *sink = acc;
}
__global__ void stream_copy(const uint4 *__restrict__ p, uint4 *__restrict__ q, size_t n16)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride)
        q[i] = p[i];
}
__global__ void stream_write(uint4 *o, size_t n16)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    const uint4 v = make_uint4(1, 2, 3, 4);
    for (; i < n16; i += stride)
        o[i] = v;
}

template <typename F>
float time_us(F f, int iters)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    for (int i = 0; i < 3; ++i)
        f();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    for (int i = 0; i < iters; ++i)
        f();
    CK(hipEventRecord(b));
    CK(hipEventSynchronize(b));
    float ms;
    CK(hipEventElapsedTime(&ms, a, b));
    return ms / iters * 1e3f;
}

template <int N>
void run(const uint4 *tab, size_t bytes, uint32_t *sink)
{
    const int T = 16384 * (32 / N);
    const size_t row_block = (size_t)N * 2048;
    const int nrows = (int)(bytes / row_block);
    std::vector<int> rows(T);
    srand(1);
    for (auto &r : rows)
        r = (int)(((size_t)rand() * 65536 + rand()) % nrows);
    int *drows;
    CK(hipMalloc(&drows, T * 4));
    CK(hipMemcpy(drows, rows.data(), T * 4, hipMemcpyHostToDevice));
    uint4 *h, *sh, *out;
    CK(hipMalloc(&h, (size_t)T * 2048));
    CK(hipMalloc(&sh, (size_t)T * 2048));
    CK(hipMalloc(&out, (size_t)T * 2048));
    CK(hipMemset(h, 1, (size_t)T * 2048));
    CK(hipMemset(sh, 1, (size_t)T * 2048));
    const double rb = (double)T * row_block, a1 = (double)T * 2048;
    const int g = 1024;
    printf("N=%d, T=%d tokens, %d workgroups of 4 waves\n", N, T, g);
#define RUN(MIX, BYTES, NAME)                                                                       \
    {                                                                                               \
        const float us = time_us([&] { pattern<N, MIX><<<g, 256>>>(tab, drows, T, h, sh, out, sink); }, 10); \
        printf("  %-44s %8.1f us  %5.2f TB/s\n", NAME, us, (BYTES) / us / 1e6);                     \
    }
    RUN(0, rb, "rows only")
    RUN(NT_ROWS, rb, "rows only, non-temporal loads")
    RUN(LOAD_H | LOAD_SHARED, rb + 2 * a1, "rows + h + shared")
    RUN(STORE_OUT, rb + a1, "rows + out store")
    RUN(STORE_OUT | NT_STORE, rb + a1, "rows + non-temporal out store")
    RUN(LOAD_H | LOAD_SHARED | STORE_OUT, rb + 3 * a1, "full mix")
    RUN(LOAD_H | LOAD_SHARED | STORE_OUT | NT_STORE, rb + 3 * a1, "full mix, non-temporal store")
    RUN(LOAD_H | LOAD_SHARED | STORE_OUT | NT_STORE | NT_ACT, rb + 3 * a1, "full mix, non-temporal store and act loads")
    RUN(LOAD_H | LOAD_SHARED | STORE_OUT | NT_STORE | NT_ACT | NT_ROWS, rb + 3 * a1, "full mix, everything non-temporal")
#undef RUN
#define RUND(WPB, BUFS, MIX, BYTES, NAME)                                                          \
    {                                                                                               \
        const size_t lds = (size_t)WPB * BUFS * N * 1024;                                           \
        CK(hipFuncSetAttribute(reinterpret_cast<const void *>(&pattern_dma<N, WPB, BUFS, MIX>),      \
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));              \
        const int gd = 256 * (int)(160 * 1024 / lds);                                               \
        const float us = time_us([&] { pattern_dma<N, WPB, BUFS, MIX><<<gd, WPB * 64, lds>>>(tab, drows, T, h, sh, out, sink); }, 10); \
        printf("  %-44s %8.1f us  %5.2f TB/s\n", NAME, us, (BYTES) / us / 1e6);                     \
    }
    constexpr int W1 = 128 / N, W2 = 64 / N;    // waves per workgroup so that the buffers take 128 KiB
    RUND(W1, 1, 0, rb, "to LDS, one buffer per wave: rows only")
    RUND(W2, 2, 0, rb, "to LDS, two buffers per wave: rows only")
    RUND(W1, 1, LOAD_H | LOAD_SHARED | STORE_OUT | NT_STORE | NT_ACT, rb + 3 * a1, "to LDS, one buffer: full mix, NT store + act")
    RUND(W2, 2, LOAD_H | LOAD_SHARED | STORE_OUT | NT_STORE | NT_ACT, rb + 3 * a1, "to LDS, two buffers: full mix, NT store + act")
#undef RUND
    CK(hipFree(drows));
    CK(hipFree(h));
    CK(hipFree(sh));
    CK(hipFree(out));
}

int main()
{
    const size_t bytes = (size_t)8 << 30, n16 = bytes / 16;
    uint4 *p, *q;
    uint32_t *sink;
    CK(hipMalloc(&p, bytes));
    CK(hipMalloc(&q, bytes));
    CK(hipMalloc(&sink, 4));
    CK(hipMemset(p, 1, bytes));
    CK(hipMemset(q, 2, bytes));
    float us = time_us([&] { stream_read<<<16384, 256>>>(p, n16, sink); }, 5);
    printf("grid-stride read of 8 GiB                       %8.1f us  %5.2f TB/s\n", us, bytes / us / 1e6);
    us = time_us([&] { stream_copy<<<65536, 256>>>(p, q, n16); }, 5);
    printf("grid-stride copy of 8 GiB (read + write bytes)  %8.1f us  %5.2f TB/s\n", us, 2.0 * bytes / us / 1e6);
    us = time_us([&] { stream_write<<<4096, 256>>>(q, (size_t)1 << 26); }, 5);
    printf("write of 1 GiB                                  %8.1f us  %5.2f TB/s\n", us, (double)(1 << 30) / us / 1e6);
    CK(hipFree(q));
    run<16>(p, bytes, sink);
    run<32>(p, bytes, sink);
    return 0;
}
