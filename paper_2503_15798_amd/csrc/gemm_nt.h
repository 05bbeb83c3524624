// The two bf16 / fp16 MFMA GEMM kernels of the library (C = A . B^T with both operands K-contiguous), shared by
// the LUT build (Sec. 3.3, LUT entry equation) and the layer call that evaluates the shared expert itself
// (inference-layer equation).  v_mfma_f32_32x32x16_{bf16,f16}, fp32 accumulation.
//   gemm_nt_direct_kernel  256 x 256 tile, operands fed by direct global -> LDS loads (column counts that are
//                          multiples of 256)
//   gemm_nt_kernel         256 x 128 tile, register-staged (other multiples of 128)
// Epilogues: plain store; GELU with the result stored as a bf16 hi + lo pair or as fp16 (hidden activations);
// and the lookup epilogue, which adds the residual and the gate-weighted sum of the token's table rows to the
// output tile before its single rounding.
#ifndef MOLE_GEMM_NT_H
#define MOLE_GEMM_NT_H

#include "fwd_common.h"

namespace {
using namespace mole;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // native vector: stays in registers

constexpr int BM = 256, BN = 128, BK = 64;
constexpr int LDS_ROW = BK * 2 + 16;   // bytes per tile row in LDS
constexpr int GEMM_THREADS = 256;

enum { EPI_STORE = 0, EPI_GELU_SPLIT = 1, EPI_GELU_F16 = 2, EPI_LOOKUP = 3 };
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
    // EPI_LOOKUP (the GEMM's rows are tokens, its Nn columns the hidden size): out = product + bias + residual
    // + sum_j gates[t, j] * table[row(t), j, :], rounded once
    const uint16_t *table;   // [rows, n_experts, Nn]
    const int32_t *rowsrc;   // [M]: row(t)
    const float *gates;      // [M, n_experts] fp32
    const uint16_t *residual;   // [M, ldc] nullable
    int64_t table_rows;
    int n_experts;
    int32_t *err_flag;       // nullable
    int lookup_first;        // 1: every other workgroup (checkerboard over the tile grid) gathers BEFORE its main loop
};

// acc[0..7] += sum_j gates[t, j] * table[row(t), j, col .. col + 7] (B row pieces in flight at a time); a token whose
// id is outside the table adds nothing and is flagged by the reporter
template <int B = 8>
__device__ __forceinline__ void lookup_rows8(float (&acc)[8], const GemmArgs &g, int t, int col, bool reporter)
{
    const int64_t row = g.rowsrc[t];
    if (row >= 0 && row < g.table_rows) {
        const int N = g.n_experts;
        const uint16_t *tp = g.table + (row * N) * (int64_t)g.Nn + col;
        const float *gp = g.gates + (int64_t)t * N;
        for (int j0 = 0; j0 < N; j0 += B) {
            uint4 piece[B];
            float gj[B];
#pragma unroll
            for (int u = 0; u < B; ++u) {
                const int j = j0 + u < N ? j0 + u : N - 1;
                piece[u] = *reinterpret_cast<const uint4 *>(tp + (int64_t)j * g.Nn);
                gj[u] = j0 + u < N ? gp[j] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < B; ++u)
                fma8(acc, gj[u], piece[u]);
        }
    } else if (reporter && g.err_flag) {
        atomicOr(g.err_flag, 1);
    }
}

// Lookup epilogue for one 16-byte piece of the output (8 columns starting at `col` of token `t`): sp holds the
// tile's fp32 values (product + bias) for these columns.  Adds the residual and the gate-weighted sum of the
// token's N table rows, rounds once and stores.
// with_rows = false: the gate-weighted rows are already part of sp (they were the accumulators' start values)
__device__ __forceinline__ uint4 lookup_value(const GemmArgs &g, const float *sp, int t, int col, bool reporter,
                                              bool with_rows = true)
{
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
        acc[e] = sp[e];
    if (g.residual)
        add8(acc, *reinterpret_cast<const uint4 *>(g.residual + (int64_t)t * g.ldc + col));
    if (with_rows)
        lookup_rows8(acc, g, t, col, reporter);
    return pack8(acc);
}

__device__ __forceinline__ void lookup_piece(const GemmArgs &g, uint16_t *C, const float *sp, int t, int col, bool reporter)
{
    *reinterpret_cast<uint4 *>(C + (int64_t)t * g.ldc + col) = lookup_value(g, sp, t, col, reporter);
}

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
    // bytes per staged row (padded); the lookup epilogue stages fp32 values: it rounds after its own additions
    constexpr int CROW = EPI == EPI_LOOKUP ? BN * 4 + 16 : BN * 2 + 8;
    constexpr int CPLANE = 64 * CROW;
    static_assert((EPI == EPI_LOOKUP ? 1 : 2) * CPLANE <= BM * LDS_ROW, "epilogue staging must fit in the A tile");
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
                } else if constexpr (EPI == EPI_LOOKUP) {
                    *reinterpret_cast<float4 *>(srow + cl * 4) = make_float4(v[0], v[1], v[2], v[3]);
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
            if constexpr (EPI == EPI_LOOKUP) {
                if (row < g.M)
                    lookup_piece(g, C, reinterpret_cast<const float *>(Cs + sr * CROW) + sc * 8, row, n0 + sc * 8,
                                 sc == 0);
            } else if (row < g.M) {
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

    // EPI_LOOKUP, g.lookup_first: the workgroups of one colour of a checkerboard over the tile grid gather their
    // gate-weighted table rows BEFORE the main loop and start the accumulators from them; the others gather behind it.
    // A tile's rows are 4 MB of memory traffic and its main loop runs on operands from L2: when every workgroup of a
    // one-round grid gathers at the end, the memory system idles during the main loops and the matrix pipe during the
    // gathers.  Staging as in the epilogue, the other way round: pieces in row order -> LDS (fp32) -> accumulator layout.
    bool rows_in_acc = false;
    if constexpr (EPI == EPI_LOOKUP) {
        rows_in_acc = g.lookup_first && ((blockIdx.x + blockIdx.y) & 1);
        if (rows_in_acc) {
            constexpr int CROW0 = DBN * 4 + 16;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int piece = tid + u * D_THREADS;
                    const int sr = piece >> 5, sc = piece & 31;
                    const int row = m0 + (sr >> 5) * 128 + i * 32 + (sr & 31);
                    float s8[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        s8[e] = 0.f;
                    if (row < g.M)
                        lookup_rows8<16>(s8, g, row, n0 + sc * 8, sc == 0);
                    float *dst = reinterpret_cast<float *>(dsmem + sr * CROW0) + sc * 8;
                    *reinterpret_cast<float4 *>(dst) = make_float4(s8[0], s8[1], s8[2], s8[3]);
                    *reinterpret_cast<float4 *>(dst + 4) = make_float4(s8[4], s8[5], s8[6], s8[7]);
                }
                __syncthreads();
                const unsigned char *srow = dsmem + (wm * 32 + (lane & 31)) * CROW0;
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int cl = wn * 64 + j * 32 + 8 * q + 4 * (lane >> 5);
                        const float4 v = *reinterpret_cast<const float4 *>(srow + cl * 4);
                        acc[i][j][4 * q + 0] = v.x;
                        acc[i][j][4 * q + 1] = v.y;
                        acc[i][j][4 * q + 2] = v.z;
                        acc[i][j][4 * q + 3] = v.w;
                    }
                __syncthreads();
            }
        }
    }

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
    constexpr int CROW = EPI == EPI_LOOKUP ? DBN * 4 + 16 : DBN * 2 + 8;
    constexpr int CPLANE = 64 * CROW;
    static_assert((EPI == EPI_LOOKUP ? 1 : 2) * CPLANE <= (int)D_LDS_BYTES, "epilogue staging must fit in the operand stages");
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
                } else if constexpr (EPI == EPI_LOOKUP) {
                    *reinterpret_cast<float4 *>(srow + cl * 4) = make_float4(v[0], v[1], v[2], v[3]);
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
        if constexpr (EPI == EPI_LOOKUP) {
            // values first, stores behind them: a store between two pieces' loads would keep the compiler from
            // requesting the second piece's rows while the first piece's travel
            uint4 o[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int piece = tid + u * D_THREADS;
                const int sr = piece >> 5, sc = piece & 31;
                const int row = m0 + (sr >> 5) * 128 + i * 32 + (sr & 31);
                o[u] = lookup_value(g, reinterpret_cast<const float *>(Cs + sr * CROW) + sc * 8, min(row, g.M - 1), n0 + sc * 8,
                                    sc == 0, !rows_in_acc);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int piece = tid + u * D_THREADS;
                const int sr = piece >> 5, sc = piece & 31;
                const int row = m0 + (sr >> 5) * 128 + i * 32 + (sr & 31);
                if (row < g.M)
                    *reinterpret_cast<uint4 *>(C + (int64_t)row * g.ldc + n0 + sc * 8) = o[u];
            }
        } else {
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
        }
        __syncthreads();
    }
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

// dst[r, 0..cols) = fp16(src[r, 0..cols)) for bf16 src with row stride cols and dst row stride dst_ld (exact for
// |x| in [2^-14, 65504]; smaller values become fp16 subnormals, absolute error below 3e-8).  cols % 8 == 0.
__global__ __launch_bounds__(256) void bf16_to_f16_rows_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                                int64_t rows, int cols, int dst_ld)
{
    const int per_row = cols >> 3;
    const int64_t total = rows * per_row;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / per_row;
        const int c = (int)(i - r * per_row) * 8;
        const uint4 v = *reinterpret_cast<const uint4 *>(src + r * cols + c);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)bf16lo(w[e])) |
                   ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)bf16hi(w[e])) << 16);
        *reinterpret_cast<uint4 *>(dst + r * dst_ld + c) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

}  // namespace
#endif
