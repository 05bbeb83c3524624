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
#include "mole_internal.h"

#include <stdlib.h>
#include <string.h>

namespace {
using namespace mole;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // native vector: stays in registers

constexpr int BM = 256, BN = 128, BK = 64;
constexpr int LDS_ROW = BK * 2 + 16;   // bytes per tile row in LDS
constexpr int GEMM_THREADS = 256;

enum { EPI_STORE = 0, EPI_GELU_SPLIT = 1, EPI_GELU_F16 = 2 };
enum { MODE_F16 = 1, MODE_SPLIT = 2 };   // how the hidden activation is carried (chosen on the device)
constexpr float F16_SAFE = 60000.0f;

struct GemmArgs {
    const uint16_t *A;       // [planes][M, K] row-major, K contiguous
    int64_t lda, a_plane_stride, a_batch_stride;
    int a_planes;
    const uint16_t *Bt;      // [Nn, K] row-major (the transposed weight)
    int64_t ldb, b_batch_stride;
    const uint16_t *bias;    // [Nn] nullable
    int64_t bias_batch_stride;
    uint16_t *C;             // EPI_STORE: [M, ldc]; EPI_GELU_SPLIT: planes hi, lo
    int64_t ldc, c_plane_stride, c_batch_stride;
    int M, Nn, K;
    int epilogue, act;
    const int *mode;         // nullable: run only if *mode == run_mode
    int run_mode;
};

__device__ __forceinline__ float gelu_f(float x, int act)
{
    if (act == MOLE_GELU_TANH) {
        const float k = 0.7978845608028654f;
        return 0.5f * x * (1.0f + tanhf(k * (x + 0.044715f * x * x * x)));
    }
    return 0.5f * x * (1.0f + erff(x * 0.7071067811865476f));
}

struct BStage {
    u32x4 b0, b1, b2, b3;
};

__device__ __forceinline__ void gemm_fetch(u32x4 (&ra)[8], BStage &rb, const GemmArgs &g, const uint16_t *A,
                                           const uint16_t *Bt, int kt, int ktiles_per_plane, int m0, int n0,
                                           int prow, int pk)
{
    const int plane = kt / ktiles_per_plane;
    const int kk = (kt - plane * ktiles_per_plane) * BK + pk * 8;
    const uint16_t *Ap = A + plane * g.a_plane_stride;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = m0 + prow + i * 32;
        ra[i] = row < g.M ? *reinterpret_cast<const u32x4 *>(Ap + (int64_t)row * g.lda + kk) : u32x4{0, 0, 0, 0};
    }
    const uint16_t *Bp = Bt + (int64_t)(n0 + prow) * g.ldb + kk;
    rb.b0 = *reinterpret_cast<const u32x4 *>(Bp);
    rb.b1 = *reinterpret_cast<const u32x4 *>(Bp + 32 * g.ldb);
    rb.b2 = *reinterpret_cast<const u32x4 *>(Bp + 64 * g.ldb);
    rb.b3 = *reinterpret_cast<const u32x4 *>(Bp + 96 * g.ldb);
}

__device__ __forceinline__ void gemm_stash(const u32x4 (&ra)[8], const BStage &rb, unsigned char *As,
                                           unsigned char *Bs, int prow, int pk)
{
#pragma unroll
    for (int i = 0; i < 8; ++i)
        *reinterpret_cast<u32x4 *>(As + (prow + i * 32) * LDS_ROW + pk * 16) = ra[i];
    unsigned char *bp = Bs + prow * LDS_ROW + pk * 16;
    *reinterpret_cast<u32x4 *>(bp) = rb.b0;
    *reinterpret_cast<u32x4 *>(bp + 32 * LDS_ROW) = rb.b1;
    *reinterpret_cast<u32x4 *>(bp + 64 * LDS_ROW) = rb.b2;
    *reinterpret_cast<u32x4 *>(bp + 96 * LDS_ROW) = rb.b3;
}

// GELU for the MFMA epilogue.  The epilogue of the first GEMM handles V*D*N values with only K = d
// multiply-adds behind each, so it has to be cheap: erf by the five-term rational/exponential
// approximation (absolute error 1.5e-7, far below the 2^-17 of the hi/lo split), tanh through one
// fast exponential.
__device__ __forceinline__ float gelu_fast(float x, int act)
{
    if (act == MOLE_GELU_TANH) {
        const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
        const float th = 1.0f - 2.0f * __builtin_amdgcn_rcpf(__expf(2.0f * u) + 1.0f);
        return 0.5f * x * (1.0f + th);
    }
    // x Phi(x) with Phi(-|x|) = erfc(|x| / sqrt 2) / 2 =: c: the result is max(x, 0) - |x| c for either sign.
    // c = q(t) e with t = 1 / (1 + p |x| / sqrt 2), q the five-term polynomial (coefficients halved),
    // e = exp(-x^2 / 2) = 2^(-x^2 log2(e) / 2); the constants of z = |x| / sqrt 2 are folded in.
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.7071067811865476f, ax, 1.0f));
    float q = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
    q = fmaf(q, t, 0.5f * 1.421413741f);
    q = fmaf(q, t, 0.5f * -0.284496736f);
    q = fmaf(q, t, 0.5f * 0.254829592f);
    const float e = __builtin_amdgcn_exp2f(x * x * -0.7213475204444817f);
    return fmaxf(x, 0.0f) - ax * (q * t * e);
}

// round-to-nearest-even without the NaN branch (inputs are finite here), two values into one dword
__device__ __forceinline__ uint32_t rne_pair(float a, float b)
{
    const uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    const uint32_t ra = (ua + 0x7fffu + ((ua >> 16) & 1u)) >> 16;
    const uint32_t rb = (ub + 0x7fffu + ((ub >> 16) & 1u)) & 0xffff0000u;
    return ra | rb;
}

// F16: both operands hold fp16 (GEMM 2 of the fp16 mode), else bf16.
template <int EPI, bool F16>
__global__ __launch_bounds__(GEMM_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_nt_kernel(GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) unsigned char As[BM * LDS_ROW];
    __shared__ __attribute__((aligned(16))) unsigned char Bs[BN * LDS_ROW];
    if (g.mode && *g.mode != g.run_mode)
        return;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int batch = blockIdx.z;
    const uint16_t *A = g.A + batch * g.a_batch_stride;
    const uint16_t *Bt = g.Bt + batch * g.b_batch_stride;

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[i][j][e] = 0.f;

    // staging registers: A tile = 256 rows x 8 pieces -> 8 per thread; B tile = 128 x 8 -> 4
    u32x4 ra[8];
    BStage rb;
    const int prow = tid >> 3, pk = tid & 7;   // piece (row, 16-byte column) for i = 0; +32 rows per i
    const int ktiles_per_plane = g.K / BK;
    const int ktiles = ktiles_per_plane * g.a_planes;

    gemm_fetch(ra, rb, g, A, Bt, 0, ktiles_per_plane, m0, n0, prow, pk);
    const int frow = lane & 31, fk = (lane >> 5) * 16;   // fragment row and byte offset of its K run
    for (int kt = 0; kt < ktiles; ++kt) {
        gemm_stash(ra, rb, As, Bs, prow, pk);
        __syncthreads();
        if (kt + 1 < ktiles)
            gemm_fetch(ra, rb, g, A, Bt, kt + 1, ktiles_per_plane, m0, n0, prow, pk);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            u32x4 af[4], bfr[2];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                af[i] = *reinterpret_cast<const u32x4 *>(As + (wm * 128 + i * 32 + frow) * LDS_ROW + ks * 32 + fk);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                bfr[j] = *reinterpret_cast<const u32x4 *>(Bs + (wn * 64 + j * 32 + frow) * LDS_ROW + ks * 32 + fk);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if constexpr (F16)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, bfr[j]),
                                                                           __builtin_bit_cast(f16x8, af[i]),
                                                                           acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfr[j]),
                                                                            __builtin_bit_cast(bf16x8, af[i]),
                                                                            acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    // Epilogue.  The weight fragment is the MFMA's first operand, so the accumulator holds the tile
    // transposed: lane l has output row m = l % 32 and, in elements 4q..4q+3, the four consecutive
    // output columns n = 8q + 4*(l/32) + 0..3.  Results go through LDS (the operand tiles are dead by
    // now) so that global memory sees full 16-byte, row-contiguous stores: four passes of 64 rows
    // (32 from each wave row), hi plane at Cs, lo plane behind it.
    const uint16_t *bias = g.bias ? g.bias + batch * g.bias_batch_stride : nullptr;
    uint16_t *C = g.C + batch * g.c_batch_stride;
    constexpr int CROW = BN * 2 + 8;                 // bytes per staged row (padded: conflict-free 8-byte writes)
    constexpr int CPLANE = 64 * CROW;
    static_assert(2 * CPLANE <= BM * LDS_ROW, "epilogue staging must fit in the A tile");
    unsigned char *Cs = As;
    float bv[2][4][4];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = n0 + wn * 64 + j * 32 + 8 * q + 4 * (lane >> 5);
            uint2 b4 = make_uint2(0, 0);
            if (bias)
                b4 = *reinterpret_cast<const uint2 *>(bias + col);
            bv[j][q][0] = bf16lo(b4.x); bv[j][q][1] = bf16hi(b4.x);
            bv[j][q][2] = bf16lo(b4.y); bv[j][q][3] = bf16hi(b4.y);
        }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // stage this pass: row wm*32 + l%32 of the 64-row slab
        unsigned char *srow = Cs + (wm * 32 + (lane & 31)) * CROW;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cl = wn * 64 + j * 32 + 8 * q + 4 * (lane >> 5);   // column inside the tile
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    v[e] = acc[i][j][4 * q + e] + bv[j][q][e];
                if constexpr (EPI == EPI_GELU_SPLIT) {
                    float lo[4];
                    uint32_t hbits[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = gelu_fast(v[e], g.act);
                        const uint32_t u = __float_as_uint(v[e]);
                        hbits[e] = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
                        lo[e] = v[e] - __uint_as_float(hbits[e]);
                    }
                    uint2 hi2, lo2;
                    hi2.x = (hbits[0] >> 16) | hbits[1];
                    hi2.y = (hbits[2] >> 16) | hbits[3];
                    lo2.x = rne_pair(lo[0], lo[1]);
                    lo2.y = rne_pair(lo[2], lo[3]);
                    *reinterpret_cast<uint2 *>(srow + cl * 2) = hi2;
                    *reinterpret_cast<uint2 *>(srow + CPLANE + cl * 2) = lo2;
                } else if constexpr (EPI == EPI_GELU_F16) {
                    uint16_t hb[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // the mode was only selected if no value can reach the fp16 range limit; the
                        // clamp keeps a violated assumption finite
                        const float a = fminf(fmaxf(gelu_fast(v[e], g.act), -65504.0f), 65504.0f);
                        hb[e] = __builtin_bit_cast(uint16_t, (_Float16)a);      // round to nearest even
                    }
                    uint2 o;
                    o.x = (uint32_t)hb[0] | ((uint32_t)hb[1] << 16);
                    o.y = (uint32_t)hb[2] | ((uint32_t)hb[3] << 16);
                    *reinterpret_cast<uint2 *>(srow + cl * 2) = o;
                } else {
                    uint2 o;
                    o.x = pack_bf16(v[0], v[1]);
                    o.y = pack_bf16(v[2], v[3]);
                    *reinterpret_cast<uint2 *>(srow + cl * 2) = o;
                }
            }
        }
        __syncthreads();
        // write out: 64 rows x 256 bytes per plane = 1024 16-byte pieces, 4 per thread and plane
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int piece = tid + u * GEMM_THREADS;
            const int sr = piece >> 4, sc = piece & 15;                 // staged row, 16-byte column
            const int row = m0 + (sr >> 5) * 128 + i * 32 + (sr & 31);
            if (row < g.M) {
                uint16_t *cp = C + (int64_t)row * g.ldc + n0 + sc * 8;
                *reinterpret_cast<u32x4 *>(cp) = *reinterpret_cast<const u32x4 *>(Cs + sr * CROW + sc * 16);
                if constexpr (EPI == EPI_GELU_SPLIT)
                    *reinterpret_cast<u32x4 *>(cp + g.c_plane_stride) =
                        *reinterpret_cast<const u32x4 *>(Cs + CPLANE + sr * CROW + sc * 16);
            }
        }
        __syncthreads();
    }
}

constexpr int DBM = 256, DBN = 256, D_THREADS = 512;

// ------------------------------------------------------------------------------------------
// 256 x 256 tile fed by direct global -> LDS loads (global_load_lds_dwordx4, gfx950): no staging
// registers, no ds_write.  A wave-wide load drops lane l's 16 bytes at LDS base + 16*l, i.e. 1 KiB
// contiguous = 8 tile rows of 128 bytes (K step 64: every row segment is a whole 128-byte line; with
// 64-byte segments the same L2 delivers a third less).  Rows are therefore unpadded, and bank
// conflicts are avoided by a swizzle applied on the global side: slot s of row r holds K piece
// s ^ ((r >> 1) & 7), so the 16 rows a fragment read touches per pass cover all 64 banks.
// Two stages of 64 KiB: step kt + 1 travels while step kt is multiplied.  8 waves (2 x 4), each
// 128 x 64 outputs, two per SIMD.
// ------------------------------------------------------------------------------------------
constexpr int D_ROW_BYTES = BK * 2;                        // bytes per tile row (128)
constexpr int D_STAGE_BYTES = (DBM + DBN) * D_ROW_BYTES;          // 64 KiB
constexpr int D_STAGES = 2;
constexpr size_t D_LDS_BYTES = (size_t)D_STAGES * D_STAGE_BYTES;

#define MOLE_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

template <int EPI, bool F16>
__global__ __launch_bounds__(D_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_nt_direct_kernel(GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char dsmem[];
    if (g.mode && *g.mode != g.run_mode)
        return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int m0 = blockIdx.x * DBM, n0 = blockIdx.y * DBN;
    const int batch = blockIdx.z;
    const uint16_t *A = g.A + batch * g.a_batch_stride;
    const uint16_t *Bt = g.Bt + batch * g.b_batch_stride;

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[i][j][e] = 0.f;

    // feed: per K step the tile pair is 64 chunks of 8 rows (A: 0..31, B: 32..63); wave w moves
    // A chunks w, w + 8, w + 16, w + 24 and the same B chunks.  Lane l of a chunk load: row l >> 3,
    // slot l & 7.
    const int rr = lane >> 3, slot = lane & 7;
    const uint16_t *gp[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int chunk = wave + 8 * (i & 3);
        const int row = chunk * 8 + rr;                        // row inside the tile
        const int piece = slot ^ ((row >> 1) & 7);             // K piece this lane fetches
        if (i < 4)   // rows past M are clamped: their products are never stored
            gp[i] = A + (int64_t)min(m0 + row, g.M - 1) * g.lda + piece * 8;
        else
            gp[i] = Bt + (int64_t)(n0 + row) * g.ldb + piece * 8;
    }
    const int ktiles_per_plane = g.K / BK;
    const int ktiles = ktiles_per_plane * g.a_planes;
    // load i (0..7) of K step kt; the eight loads of a step are issued one at a time between groups of
    // MFMAs: a burst of them right after the barrier keeps every wave of the workgroup waiting in the
    // memory pipeline's queue, and nothing feeds the matrix pipe meanwhile (measured: the step then
    // takes compute time plus load-issue time)
    int64_t cur_aoff = 0, cur_kk = 0;
    unsigned char *cur_stage = dsmem;
    auto begin_issue = [&](int kt) {
        const int plane = kt / ktiles_per_plane;
        cur_kk = (kt - plane * ktiles_per_plane) * BK;
        cur_aoff = plane * g.a_plane_stride + cur_kk;
        cur_stage = dsmem + (kt & (D_STAGES - 1)) * D_STAGE_BYTES + wave * 1024;
    };
    auto issue_one = [&](int i) {
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void *)(gp[i] + (i < 4 ? cur_aoff : cur_kk)),
            (__attribute__((address_space(3))) void *)(cur_stage + (i < 4 ? 0 : DBM * D_ROW_BYTES) + (i & 3) * 8192), 16, 0, 0);
    };

    // fragment addressing: row frow of a 32-row block, K piece 2*ks + (lane >> 5), swizzled
    const int frow = lane & 31, swz = (frow >> 1) & 7, hi = lane >> 5;
    const int a_base = (wm * 128 + frow) * D_ROW_BYTES, b_base = (DBM + wn * 64 + frow) * D_ROW_BYTES;
    struct Frag {
        u32x4 a[4], b[2];
    };
    auto load_frag = [&](Frag &f, const unsigned char *stage, int ks) {
        const int koff = ((2 * ks + hi) ^ swz) * 16;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            f.a[i] = *reinterpret_cast<const u32x4 *>(stage + a_base + i * 32 * D_ROW_BYTES + koff);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            f.b[j] = *reinterpret_cast<const u32x4 *>(stage + b_base + j * 32 * D_ROW_BYTES + koff);
    };
    // four MFMAs: A blocks i0, i0 + 1 against both B blocks
    auto multiply2 = [&](const Frag &f, int i0) {
#pragma unroll
        for (int i = i0; i < i0 + 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if constexpr (F16)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, f.b[j]),
                                                                       __builtin_bit_cast(f16x8, f.a[i]),
                                                                       acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.b[j]),
                                                                        __builtin_bit_cast(bf16x8, f.a[i]),
                                                                        acc[i][j], 0, 0, 0);
            }
    };

    begin_issue(0);
#pragma unroll
    for (int i = 0; i < 8; ++i)
        issue_one(i);
    for (int kt = 0; kt < ktiles; ++kt) {
        // Step kt has landed for this thread once nothing is outstanding (the next step is issued
        // below); the barrier extends that to every thread's loads and also says that nobody reads
        // the other stage any more.  A bare barrier: __syncthreads() adds fences the explicit waits
        // make unnecessary.
        MOLE_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        const bool more = kt + 1 < ktiles;
        if (more)
            begin_issue(kt + 1);
        const unsigned char *stage = dsmem + (kt & (D_STAGES - 1)) * D_STAGE_BYTES;
        // Order of the step (kept by the scheduling barriers; left alone the compiler re-sorts the
        // region to save registers): fragments of slice ks + 1 are requested before slice ks is
        // multiplied, and one load of the next step goes out per group of four MFMAs.
#define MOLE_STEP(LOADI, FRAG, I0)             \
        if (more)                              \
            issue_one(LOADI);                  \
        __builtin_amdgcn_sched_barrier(0);     \
        multiply2(FRAG, I0);                   \
        __builtin_amdgcn_sched_barrier(0);
        Frag f0, f1;
        load_frag(f0, stage, 0);
        load_frag(f1, stage, 1);
        __builtin_amdgcn_sched_barrier(0);
        MOLE_STEP(0, f0, 0)
        MOLE_STEP(1, f0, 2)
        load_frag(f0, stage, 2);
        __builtin_amdgcn_sched_barrier(0);
        MOLE_STEP(2, f1, 0)
        MOLE_STEP(3, f1, 2)
        load_frag(f1, stage, 3);
        __builtin_amdgcn_sched_barrier(0);
        MOLE_STEP(4, f0, 0)
        MOLE_STEP(5, f0, 2)
        MOLE_STEP(6, f1, 0)
        MOLE_STEP(7, f1, 2)
#undef MOLE_STEP
        __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0): this wave's LDS reads of the stage are complete
    }
    __syncthreads();

    // Epilogue: as in the 256 x 128 kernel (accumulator layout, staging through LDS, 16-byte stores),
    // four passes of 64 rows (32 from each wave row) by 256 columns.
    const uint16_t *bias = g.bias ? g.bias + batch * g.bias_batch_stride : nullptr;
    uint16_t *C = g.C + batch * g.c_batch_stride;
    constexpr int CROW = DBN * 2 + 8;
    constexpr int CPLANE = 64 * CROW;
    static_assert(2 * CPLANE <= (int)D_LDS_BYTES, "epilogue staging must fit in the operand stages");
    unsigned char *Cs = dsmem;
    float bv[2][4][4];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = n0 + wn * 64 + j * 32 + 8 * q + 4 * (lane >> 5);
            uint2 b4 = make_uint2(0, 0);
            if (bias)
                b4 = *reinterpret_cast<const uint2 *>(bias + col);
            bv[j][q][0] = bf16lo(b4.x); bv[j][q][1] = bf16hi(b4.x);
            bv[j][q][2] = bf16lo(b4.y); bv[j][q][3] = bf16hi(b4.y);
        }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        unsigned char *srow = Cs + (wm * 32 + (lane & 31)) * CROW;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cl = wn * 64 + j * 32 + 8 * q + 4 * (lane >> 5);
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    v[e] = acc[i][j][4 * q + e] + bv[j][q][e];
                if constexpr (EPI == EPI_GELU_SPLIT) {
                    float lo[4];
                    uint32_t hbits[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = gelu_fast(v[e], g.act);
                        const uint32_t u = __float_as_uint(v[e]);
                        hbits[e] = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
                        lo[e] = v[e] - __uint_as_float(hbits[e]);
                    }
                    uint2 hi2, lo2;
                    hi2.x = (hbits[0] >> 16) | hbits[1];
                    hi2.y = (hbits[2] >> 16) | hbits[3];
                    lo2.x = rne_pair(lo[0], lo[1]);
                    lo2.y = rne_pair(lo[2], lo[3]);
                    *reinterpret_cast<uint2 *>(srow + cl * 2) = hi2;
                    *reinterpret_cast<uint2 *>(srow + CPLANE + cl * 2) = lo2;
                } else if constexpr (EPI == EPI_GELU_F16) {
                    uint16_t hb[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float a = fminf(fmaxf(gelu_fast(v[e], g.act), -65504.0f), 65504.0f);
                        hb[e] = __builtin_bit_cast(uint16_t, (_Float16)a);
                    }
                    uint2 o;
                    o.x = (uint32_t)hb[0] | ((uint32_t)hb[1] << 16);
                    o.y = (uint32_t)hb[2] | ((uint32_t)hb[3] << 16);
                    *reinterpret_cast<uint2 *>(srow + cl * 2) = o;
                } else {
                    uint2 o;
                    o.x = pack_bf16(v[0], v[1]);
                    o.y = pack_bf16(v[2], v[3]);
                    *reinterpret_cast<uint2 *>(srow + cl * 2) = o;
                }
            }
        }
        __syncthreads();
        // write out: 64 rows x 512 bytes per plane = 2048 16-byte pieces, 4 per thread and plane
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int piece = tid + u * D_THREADS;
            const int sr = piece >> 5, sc = piece & 31;
            const int row = m0 + (sr >> 5) * 128 + i * 32 + (sr & 31);
            if (row < g.M) {
                uint16_t *cp = C + (int64_t)row * g.ldc + n0 + sc * 8;
                *reinterpret_cast<u32x4 *>(cp) = *reinterpret_cast<const u32x4 *>(Cs + sr * CROW + sc * 16);
                if constexpr (EPI == EPI_GELU_SPLIT)
                    *reinterpret_cast<u32x4 *>(cp + g.c_plane_stride) =
                        *reinterpret_cast<const u32x4 *>(Cs + CPLANE + sr * CROW + sc * 16);
            }
        }
        __syncthreads();
    }
}

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

// ---- choice of the hidden-activation format -----------------------------------------------
// bound[0] = max over rows of sum of squares (rows of X), bound[1] = the same for the rows of W1^T
// (= columns of W1), bound[2] = max |b1|, bound[3] = max |W2|.  Non-negative floats order like their
// bit patterns, so the maxima are taken with integer atomics.
__global__ __launch_bounds__(64) void bound_clear_kernel(unsigned *bound)
{
    if (threadIdx.x < 8)
        bound[threadIdx.x] = 0u;
}

// sum of the squares of the 8 bf16 values of a 16-byte piece
__device__ __forceinline__ float piece_sumsq(const uint4 &v, float ss)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        ss = fmaf(bf16lo(w[e]), bf16lo(w[e]), ss);
        ss = fmaf(bf16hi(w[e]), bf16hi(w[e]), ss);
    }
    return ss;
}

// One atomicMax per workgroup, and none when the stored bound already covers the group's value: thousands
// of atomics on one address are served one after the other and would cost more than the reduction's reads.
__device__ __forceinline__ void group_max_to(unsigned *out, float wave_best)
{
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0)
        part[threadIdx.x >> 6] = wave_best;
    __syncthreads();
    if (threadIdx.x == 0) {
        float b = part[0];
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w)
            b = (part[w] == part[w]) ? fmaxf(b, part[w]) : INFINITY;
        const unsigned bits = __float_as_uint(b);        // b >= 0 and not NaN: the bit patterns order like the values
        if (bits > __hip_atomic_load(out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(out, bits);
    }
}

// A wavefront takes RB rows at a time so that RB loads per lane are in flight (one row of 1024 values
// is only two 16-byte pieces per lane: a row at a time is bound by latency).
__global__ __launch_bounds__(256) void row_sumsq_max_kernel(const uint16_t *__restrict__ M, int64_t rows, int cols,
                                                             int ld, unsigned *out)
{
    constexpr int RB = 4;
    const int lane = threadIdx.x & 63;
    float best = 0.f;
    for (int64_t r0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RB; r0 < rows; r0 += (int64_t)gridDim.x * 4 * RB) {
        float ss[RB];
#pragma unroll
        for (int u = 0; u < RB; ++u)
            ss[u] = 0.f;
        for (int k = lane * 8; k < cols; k += 512) {          // cols is a multiple of 16
            uint4 v[RB];
#pragma unroll
            for (int u = 0; u < RB; ++u)
                v[u] = r0 + u < rows ? *reinterpret_cast<const uint4 *>(M + (r0 + u) * ld + k) : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < RB; ++u)
                ss[u] = piece_sumsq(v[u], ss[u]);
        }
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            float s1 = ss[u];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1)
                s1 += __shfl_xor(s1, o);
            best = fmaxf(best, s1);                           // a NaN row leaves best unchanged or NaN
            if (!(s1 == s1))
                best = INFINITY;
        }
    }
    group_max_to(out, best);
}

// max |x| over n bf16 values (x 16-byte aligned): 16-byte pieces, the last n % 8 values one by one
__global__ __launch_bounds__(256) void abs_max_kernel(const uint16_t *__restrict__ x, int64_t n, unsigned *out)
{
    float best = 0.f;
    auto take = [&](float v) {
        v = fabsf(v);
        best = v == v ? fmaxf(best, v) : INFINITY;
    };
    const int64_t n8 = n >> 3;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        const uint4 v = reinterpret_cast<const uint4 *>(x)[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            take(bf16lo(w[e]));
            take(bf16hi(w[e]));
        }
    }
    if (blockIdx.x == 0)
        for (int64_t i = (n8 << 3) + threadIdx.x; i < n; i += 256)
            take(bf16_to_f32(x[i]));
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1)
        best = fmaxf(best, __shfl_xor(best, o));
    group_max_to(out, best);
}

__global__ __launch_bounds__(64) void choose_mode_kernel(const unsigned *bound, int *mode, int forced)
{
    if (threadIdx.x != 0)
        return;
    const float pre = sqrtf(__uint_as_float(bound[0])) * sqrtf(__uint_as_float(bound[1])) * 1.01f +
                      __uint_as_float(bound[2]);
    const bool safe = pre <= F16_SAFE && __uint_as_float(bound[3]) <= F16_SAFE;   // false for NaN / inf
    *mode = forced ? forced : (safe ? MODE_F16 : MODE_SPLIT);
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

// launch one GEMM: the 256 x 256 direct-to-LDS kernel when the column count allows, else the 256 x 128 one
template <int EPI, bool F16>
mole_status launch_gemm(const GemmArgs &g, int batches, hipStream_t st)
{
    const bool big = g.Nn % DBN == 0 && knob(KNOB_BUILD_SMALL_TILE) != 1;
    if (big) {
        static std::atomic<size_t> lds_seen{0};
        MOLE_HIP_CHECK(ensure_dynamic_lds(lds_seen, reinterpret_cast<const void *>(&gemm_nt_direct_kernel<EPI, F16>),
                                          D_LDS_BYTES));
        hipLaunchKernelGGL((gemm_nt_direct_kernel<EPI, F16>), dim3((g.M + DBM - 1) / DBM, g.Nn / DBN, batches),
                           dim3(D_THREADS), D_LDS_BYTES, st, g);
    } else {
        hipLaunchKernelGGL((gemm_nt_kernel<EPI, F16>), dim3((g.M + BM - 1) / BM, g.Nn / BN, batches),
                           dim3(GEMM_THREADS), 0, st, g);
    }
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
        GemmArgs g1;
        g1.A = X + v0 * d; g1.lda = d; g1.a_plane_stride = V * (int64_t)d; g1.a_batch_stride = 0;
        g1.a_planes = x_planes;
        g1.Bt = w1t; g1.ldb = ldw1; g1.b_batch_stride = (int64_t)D * ldw1;
        g1.bias = static_cast<const uint16_t *>(b1); g1.bias_batch_stride = D;
        g1.C = hid; g1.ldc = ldh; g1.M = nv; g1.Nn = D; g1.K = d; g1.act = act; g1.mode = mode;
        GemmArgs g2;
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
