// Router of a tile of 32 tokens on the matrix pipe (Sec. 3.2 router equation: softmax over all N experts of
// h . r_j), as a device function shared by the tile kernel of the forward and the kernels that compute gates only.
//   1. v_mfma_f32_32x32x16_bf16 with the router weight as its first operand (row = expert) and the tokens' h as
//      its second (row = token); wave w of the WPB waves contracts the w-th part of d.  Lane l supplies 8
//      consecutive k of token l % 32 (one 16-byte load) and the same 8 k of expert l % 32 (eight 2-byte loads from
//      the [d, N] weight, which stays in L1 / L2).  The WPB partial 32 x 32 products meet in LDS.
//   2. wave w sums the partials of ITS 32 / WPB tokens, lane = expert, takes the softmax over the 32 lanes of a
//      half-wave (two tokens per pass) and writes the gates to memory.
// With NORM the state times the norm weight enters step 1 exactly, as a bf16 hi + lo pair (two matrix
// instructions), and 1 / rms scales the logits in step 2 (inference listing: the router reads the normed state).
#ifndef MOLE_TILE_ROUTER_H
#define MOLE_TILE_ROUTER_H

#include "fwd_common.h"

namespace mole {

constexpr int ROUTER_TILE = 32;                 // tokens per tile = rows of the matrix instruction's second operand
constexpr int ROUTER_PROW = ROUTER_TILE + 1;    // padded row of the partial-product array

// LDS floats of one router_tile call: partial logits [WPB][N][33] and (NORM) sums of squares [WPB][64]
__host__ __device__ constexpr size_t router_part_floats(int N, int WPB) { return (size_t)WPB * N * ROUTER_PROW; }
__host__ __device__ constexpr size_t router_ssq_floats(int WPB) { return (size_t)WPB * 64; }

// Gates of one tile.  tok_of(c) is the token in column c of the tile (0 .. 31), or -1 for an empty column;
// sink(c, tok, j, g) receives the gate of expert j of column c (tok = tok_of(c) >= 0), called by the wave that
// owns the column (wave c / (32 / WPB)), lane = expert within a block of 32.  All WPB waves of the group call it
// together, `wave` being the index inside the group; it holds one workgroup barrier, and the caller puts another
// between two calls that use the same LDS area.  hbase / Wr / lnw: the layer's activations [T, d], router weight
// [d, N] and norm weight [d].  part: WPB * N * 33 floats of LDS; ssq: WPB * 64 floats (NORM only).
// WT: the weight's operand pieces come from a transposed copy in LDS (wt: [N][router_wt_row(d)] bf16, filled by
// router_fill_wt) instead of eight 2-byte loads each: for a kernel that does nothing but route, those loads keep
// the CU's address unit busy for longer than anything else in the tile.
__host__ __device__ constexpr int router_wt_row(int d) { return d + 8; }     // padded: rows 16 bytes apart in the banks
__host__ __device__ constexpr size_t router_wt_bytes(int N, int d) { return (size_t)N * router_wt_row(d) * 2; }

template <int N>
__device__ __forceinline__ void router_fill_wt(uint16_t *wt, const uint16_t *Wr, int d, int nthreads)
{
    const int pieces = d * (N / 8);     // 16-byte pieces of the [d, N] weight: piece i = W[i / (N/8)][8 (i % (N/8)) ..]
    const int row = router_wt_row(d);
    for (int i = threadIdx.x; i < pieces; i += nthreads) {
        const uint4 v = reinterpret_cast<const uint4 *>(Wr)[i];
        const int k = i / (N / 8), j0 = (i % (N / 8)) * 8;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            wt[(j0 + 2 * e) * row + k] = (uint16_t)(w[e] & 0xffffu);
            wt[(j0 + 2 * e + 1) * row + k] = (uint16_t)(w[e] >> 16);
        }
    }
}

template <int N, int WPB, bool NORM, bool WT = false, class TokOf, class Sink>
__device__ __forceinline__ void router_tile(float *part_lds, float *ssq_lds, const uint16_t *hbase, const uint16_t *Wr,
                                            const uint16_t *lnw, float ln_eps, int d, int wave, int lane, TokOf tok_of,
                                            Sink sink, const uint16_t *wt = nullptr)
{
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    static_assert(N % 32 == 0 && ROUTER_TILE % WPB == 0 && (ROUTER_TILE / WPB) % 2 == 0, "");
    constexpr int PB = 4;               // router steps whose loads are issued together
    constexpr int MB = N / 32;          // blocks of 32 experts
    constexpr int TPW = ROUTER_TILE / WPB;
    constexpr int PROW = ROUTER_PROW;
    float(*part)[N][PROW] = reinterpret_cast<float(*)[N][PROW]>(part_lds);
    float(*ssq)[64] = reinterpret_cast<float(*)[64]>(ssq_lds);
    const int n = lane & 31, half = lane >> 5;
    const int npieces = d >> 3;                 // 16-byte pieces per row of h
    const int steps = (npieces + 1) >> 1;       // matrix instructions over the whole of d (two pieces each)
    const int spw = (steps + WPB - 1) / WPB;    // per wave
    const int s_begin = wave * spw, s_end = min(steps, s_begin + spw);

    // ---- 1. partial products of this wave's part of d, all 32 tokens x N experts
    {
        const int tok = tok_of(n);
        const uint16_t *hrow = hbase + (int64_t)max(tok, 0) * d;
        f32x16 acc[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[mb][e] = 0.f;
        float ss = 0.f;
        // the loads of PB steps are issued together (all addresses clamped into the row, what lies past the end
        // of d is masked to zero afterwards), then the steps' matrix instructions follow
        for (int s0 = s_begin; s0 < s_end; s0 += PB) {
            uint4 hv[PB];
            uint16_t wraw[WT ? 1 : PB][MB][8];
            uint4 wlds[WT ? PB : 1][MB];
            uint4 lw[NORM ? PB : 1];
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                const int piece = min(2 * (s0 + u) + half, npieces - 1);
                const int kp = piece * 8;
                hv[u] = *reinterpret_cast<const uint4 *>(hrow + kp);
                if constexpr (NORM)
                    lw[u] = *reinterpret_cast<const uint4 *>(lnw + kp);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    if constexpr (WT) {
                        wlds[u][mb] = *reinterpret_cast<const uint4 *>(wt + (mb * 32 + n) * router_wt_row(d) + kp);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            wraw[u][mb][e] = Wr[(int64_t)(kp + e) * N + mb * 32 + n];
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                const bool on = s0 + u < s_end && 2 * (s0 + u) + half < npieces;
                const uint32_t mask = on ? 0xffffffffu : 0u;
                hv[u].x &= mask; hv[u].y &= mask; hv[u].z &= mask; hv[u].w &= mask;
                uint4 wv[MB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    if constexpr (WT) {
                        wv[mb] = make_uint4(wlds[u][mb].x & mask, wlds[u][mb].y & mask, wlds[u][mb].z & mask,
                                            wlds[u][mb].w & mask);
                    } else {
                        wv[mb].x = ((uint32_t)wraw[u][mb][0] | ((uint32_t)wraw[u][mb][1] << 16)) & mask;
                        wv[mb].y = ((uint32_t)wraw[u][mb][2] | ((uint32_t)wraw[u][mb][3] << 16)) & mask;
                        wv[mb].z = ((uint32_t)wraw[u][mb][4] | ((uint32_t)wraw[u][mb][5] << 16)) & mask;
                        wv[mb].w = ((uint32_t)wraw[u][mb][6] | ((uint32_t)wraw[u][mb][7] << 16)) & mask;
                    }
                }
                if constexpr (NORM) {
                    // x_k * ln_w_k exactly, as a bf16 hi + lo pair (two matrix instructions per block)
                    ss += sumsq8(hv[u]);
                    const uint32_t xp[4] = {hv[u].x, hv[u].y, hv[u].z, hv[u].w};
                    const uint32_t lp[4] = {lw[u].x, lw[u].y, lw[u].z, lw[u].w};
                    uint32_t ph[4], pl[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float a0 = bf16lo(xp[q]) * bf16lo(lp[q]), a1 = bf16hi(xp[q]) * bf16hi(lp[q]);
                        ph[q] = cvt_pk_bf16(a0, a1);
                        pl[q] = cvt_pk_bf16(a0 - bf16lo(ph[q]), a1 - bf16hi(ph[q]));
                    }
                    const uint4 vh = make_uint4(ph[0], ph[1], ph[2], ph[3]), vl = make_uint4(pl[0], pl[1], pl[2], pl[3]);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wv[mb]),
                                                                          __builtin_bit_cast(bf16x8, vh), acc[mb], 0, 0, 0);
                        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wv[mb]),
                                                                          __builtin_bit_cast(bf16x8, vl), acc[mb], 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wv[mb]),
                                                                          __builtin_bit_cast(bf16x8, hv[u]), acc[mb], 0, 0, 0);
                }
            }
        }
        // lane l holds token l % 32 and, in elements 4q..4q+3, experts 8q + 4*(l/32) + 0..3 of the block
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    part[wave][mb * 32 + 8 * q + 4 * half + e][n] = acc[mb][4 * q + e];
        if constexpr (NORM)
            ssq[wave][lane] = ss;
    }
    __syncthreads();

    // ---- 2. gates of this wave's own tokens: lane = expert, two tokens (half-waves) per pass
#pragma unroll
    for (int p = 0; p < TPW / 2; ++p) {
        const int pos = wave * TPW + 2 * p + half;
        float z[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            z[mb] = 0.f;
#pragma unroll
            for (int w = 0; w < WPB; ++w)
                z[mb] += part[w][mb * 32 + n][pos];
        }
        if constexpr (NORM) {
            float s2 = 0.f;
#pragma unroll
            for (int w = 0; w < WPB; ++w)
                s2 += ssq[w][pos] + ssq[w][32 + pos];
            const float rs = __builtin_amdgcn_rsqf(s2 / (float)d + ln_eps);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                z[mb] *= rs;
        }
        float m = z[0];
#pragma unroll
        for (int mb = 1; mb < MB; ++mb)
            m = fmaxf(m, z[mb]);
        m = span_reduce<16, 1, OpMax>(m);
        float e[MB], s = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            e[mb] = __expf(z[mb] - m);
            s += e[mb];
        }
        s = span_reduce<16, 1, OpAdd>(s);
        const int tok = tok_of(pos);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            sink(pos, tok, mb * 32 + n, e[mb] / s);
    }
}

}  // namespace mole
#endif
