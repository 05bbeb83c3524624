// Device helpers shared by the forward kernels (bf16 tables and NF-quantised tables): visiting
// order, the LDS-resident router (Sec. 3.2 router equation), streaming loads and stores, epilogue.
#ifndef MOLE_FWD_COMMON_H
#define MOLE_FWD_COMMON_H

#include "mole_internal.h"

namespace mole {

// Visiting order.  Without a plan token i is item i.  With the plan of mole_dedup_ids the tokens
// are visited in id order, so equal ids are adjacent in time and place (same workgroup, same
// XCD): the repeats of a row block are then served by that L2 instead of crossing the fabric
// again.  `single` is true when the plan says the id occurs once in the batch.
struct Visit {
    int t;
    bool single;
};

// p[i] for a wave-uniform i, read through the scalar cache.  Ids and plan entries are inputs that no kernel of the
// launch writes, and a wave asks for them one at a time: as vector loads they share the counter of the row loads,
// memory returns a wave's loads in order, and the wait for the NEXT token's id became a wait for every row piece
// in flight (the router of a token started only when its rows were there).  Scalar loads are counted apart.
__device__ __forceinline__ int32_t ld_scalar(const int32_t *p, int i)
{
    typedef const __attribute__((address_space(4))) int32_t *const_as_ptr;
    return reinterpret_cast<const_as_ptr>(reinterpret_cast<uintptr_t>(p))[__builtin_amdgcn_readfirstlane(i)];
}

__device__ __forceinline__ Visit visit(const int32_t *order, int item)
{
    Visit v;
    if (order) {
        const uint32_t o = (uint32_t)ld_scalar(order, item);
        v.t = (int)(o & ~PLAN_SINGLE);
        v.single = (o & PLAN_SINGLE) != 0;
    } else {
        v.t = item;
        v.single = false;
    }
    return v;
}

// false (and bit 1 of *err_flag set) if `plan` was not written by mole_dedup_ids for T tokens; the kernels then visit
// the tokens in their own order, so the output is still the defined one
template <typename Args>
__device__ __forceinline__ bool plan_ok(const Args &a)
{
    if (a.plan[5] == PLAN_MAGIC && a.plan[2] == a.T)
        return true;
    if (threadIdx.x == 0 && a.err_flag)
        atomicOr(a.err_flag, 2);
    return false;
}

// acc += h[k]*w[k] + h[k+1]*w[k+1] for one packed pair of bf16 operands, fp32 accumulation
__device__ __forceinline__ float mac2(float acc, uint32_t hp, uint32_t wp)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, hp), __builtin_bit_cast(bf16x2, wp), acc, false);
}

// Cross-lane exchange without the LDS crossbar.  gfx950 has v_permlane32_swap / v_permlane16_swap
// (swap the upper 32 lanes of one register with the lower 32 of another; swap the odd 16-lane rows
// of one with the even rows of the other) and DPP modifiers that reach lane ^ 8 (row_ror:8 inside a
// 16-lane row), ^ 2 and ^ 1 (quad_perm).  Only ^ 4 still goes through ds_bpermute.
typedef __attribute__((ext_vector_type(2))) unsigned int swap_pair;

// (a, b) -> (a with its upper 32 lanes replaced by b's lower 32, b with its lower 32 lanes replaced by
// a's upper 32) for ROW = 32; the same with odd / even 16-lane rows for ROW = 16.  The two results
// pass through an empty asm as integers: read directly as floats, hipcc (ROCm 7.2) uses the first
// result for both.
template <int ROW>
__device__ __forceinline__ void lane_swap(float &a, float &b)
{
    static_assert(ROW == 32 || ROW == 16, "");
    const unsigned ua = __builtin_bit_cast(unsigned, a), ub = __builtin_bit_cast(unsigned, b);
    const swap_pair r = ROW == 32 ? __builtin_amdgcn_permlane32_swap(ua, ub, false, false)
                                  : __builtin_amdgcn_permlane16_swap(ua, ub, false, false);
    unsigned rx = r.x, ry = r.y;
    asm("" : "+v"(rx), "+v"(ry));
    a = __builtin_bit_cast(float, rx);
    b = __builtin_bit_cast(float, ry);
}

struct OpAdd {
    static __device__ __forceinline__ float run(float a, float b) { return a + b; }
};
struct OpMax {
    static __device__ __forceinline__ float run(float a, float b) { return fmaxf(a, b); }
};

// value of lane (l ^ W) for W in {1, 2, 4, 8}
template <int W>
__device__ __forceinline__ float lane_xor(float v)
{
    static_assert(W == 1 || W == 2 || W == 4 || W == 8, "other distances use the swap instructions");
    const int iv = __builtin_bit_cast(int, v);
    if constexpr (W == 8)
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, iv, 0x128 /* row_ror:8 */, 0xf, 0xf, false));
    else if constexpr (W == 2)
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, iv, 0x4E /* quad_perm:[2,3,0,1] */, 0xf, 0xf, false));
    else if constexpr (W == 1)
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, iv, 0xB1 /* quad_perm:[1,0,3,2] */, 0xf, 0xf, false));
    else
        return __shfl_xor(v, 4);
}

// op(v[l], v[l ^ W]) in every lane, W in {1, ..., 32}
template <int W, class Op>
__device__ __forceinline__ float pair_reduce(float v)
{
    if constexpr (W == 32 || W == 16) {
        // swapping a value with itself leaves (own half, own half) and (other half, other half)
        float a = v, b = v;
        lane_swap<W>(a, b);
        return Op::run(a, b);
    } else {
        return Op::run(v, lane_xor<W>(v));
    }
}

// op over the lanes that differ from l in the bits FROM, FROM/2, ..., TO (powers of two)
template <int FROM, int TO, class Op>
__device__ __forceinline__ float span_reduce(float v)
{
    if constexpr (FROM < TO) {
        return v;
    } else {
        v = pair_reduce<FROM, Op>(v);
        if constexpr (FROM > TO)
            return span_reduce<FROM / 2, TO, Op>(v);
        else
            return v;
    }
}

// Fold N per-lane partial sums over the 64 lanes.  Each step halves the number of values a
// lane carries by trading one half with the lane `W` away: lanes with bit W clear keep value i and
// take the partner's value i, lanes with it set keep value i + N/2 and take the partner's.  For
// W = 32 and 16 that trade is exactly one swap instruction on the pair (z[i], z[i + N/2]) followed by
// an add.  Returns, in every lane, the full sum of value j = lane >> log2(64/N).
template <int N, int W>
struct Fold {
    static __device__ __forceinline__ float run(float *z, int lane)
    {
        if constexpr (N == 1) {
            return span_reduce<W, 1, OpAdd>(z[0]);
        } else if constexpr (W == 32 || W == 16) {
#pragma unroll
            for (int i = 0; i < N / 2; ++i) {
                float a = z[i], b = z[i + N / 2];
                lane_swap<W>(a, b);
                z[i] = a + b;
            }
            return Fold<N / 2, W / 2>::run(z, lane);
        } else {
            const bool up = (lane & W) != 0;
#pragma unroll
            for (int i = 0; i < N / 2; ++i) {
                const float send = up ? z[i] : z[i + N / 2];
                const float keep = up ? z[i + N / 2] : z[i];
                z[i] = keep + lane_xor<W>(send);
            }
            return Fold<N / 2, W / 2>::run(z, lane);
        }
    }
};

// Activations are read once and written once per call.  Stores are always non-temporal; loads are
// non-temporal (NTA) in the large-batch regime, where keeping them out of L2 / Infinity Cache leaves
// more room for table rows (which ARE reused across tokens with equal ids).  For small batches the
// plain load is used: it returns sooner, and latency is what bounds those launches.
template <bool NTA>
__device__ __forceinline__ uint4 ld16_stream(const uint16_t *p)
{
    if constexpr (NTA) {
        typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    } else {
        return *reinterpret_cast<const uint4 *>(p);
    }
}
__device__ __forceinline__ void st16_stream(uint16_t *p, const uint4 &o)
{
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
    const u32x4 v = {o.x, o.y, o.z, o.w};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
}

template <bool NT>
__device__ __forceinline__ uint4 ld16_row(const uint16_t *p)
{
    return ld16_stream<NT>(p);
}

// Router weight [d, N] -> LDS as (W[k,j], W[k+1,j]) bf16 pairs.  The 16-byte piece holding experts
// 4*jq..4*jq+3 of k-pair q (k = 8*kg + 2*q, +1) of k-group kg sits at index kg * (N + 1) + q*N/4 + jq: the N
// pieces of a k-group lie together, so a lane (one k-group per piece of h) forms one address and reaches its N
// pieces through the instruction's constant offset (with the pieces of a plane together instead, every read took a
// vector add for its address: the plane stride depends on d).  The one piece of padding per k-group makes the
// lanes' stride 4 dwords modulo the 64 banks: any 16 consecutive lanes' 16-byte reads cover all banks once.
// The fill reads W_r with consecutive threads on consecutive 8-byte pieces (row pairs are 2*N*2 bytes
// of contiguous memory) and issues a batch of loads before it touches any of them.
__host__ __device__ constexpr size_t router_lds_bytes(int d, int N) { return (size_t)(d >> 3) * (N + 1) * 16; }

// NREAL < N (= 4): the weight has only NREAL (= 2) columns; the missing experts get zero weights here and
// are removed from the softmax in router_gate.
template <int N, int NREAL = N>
__device__ __forceinline__ void fill_router_lds(uint4 *smem, const uint16_t *Wr, int kgroups, int nthreads)
{
    static_assert(NREAL == N || (N == 4 && NREAL == 2), "padding is only provided from 2 to 4 experts");
    constexpr int NQ = N / 4;
    constexpr int B = 8;            // pieces per thread whose loads are issued before any is used
    const int n_w4 = kgroups * N;   // = (d/2 k-pairs) * NQ pieces
    for (int i0 = threadIdx.x; i0 < n_w4; i0 += nthreads * B) {
        uint2 w0[B], w1[B];
#pragma unroll
        for (int u = 0; u < B; ++u) {
            const int i = min(i0 + u * nthreads, n_w4 - 1);
            const int jq = i % NQ, kp = i / NQ;
            if constexpr (NREAL == N) {
                w0[u] = *reinterpret_cast<const uint2 *>(Wr + (int64_t)(2 * kp) * N + jq * 4);
                w1[u] = *reinterpret_cast<const uint2 *>(Wr + (int64_t)(2 * kp + 1) * N + jq * 4);
            } else {
                w0[u] = make_uint2(*reinterpret_cast<const uint32_t *>(Wr + (int64_t)(2 * kp) * NREAL), 0u);
                w1[u] = make_uint2(*reinterpret_cast<const uint32_t *>(Wr + (int64_t)(2 * kp + 1) * NREAL), 0u);
            }
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
            const int i = i0 + u * nthreads;
            if (i < n_w4) {
                const int jq = i % NQ, kp = i / NQ;
                uint4 v;
                v.x = (w0[u].x & 0xffffu) | (w1[u].x << 16);
                v.y = (w0[u].x >> 16) | (w1[u].x & 0xffff0000u);
                v.z = (w0[u].y & 0xffffu) | (w1[u].y << 16);
                v.w = (w0[u].y >> 16) | (w1[u].y & 0xffff0000u);
                smem[(kp >> 2) * (N + 1) + (kp & 3) * NQ + jq] = v;
            }
        }
    }
}

// z[j] += sum over the lane's 8 k of h[k] * W_r[k, j], for one 16-byte piece of h (k-group kg)
template <int N>
__device__ __forceinline__ void router_piece(float (&z)[N], const uint4 *smem, int kgroups, const uint4 &hv, int kg)
{
    constexpr int NQ = N / 4;
    const uint32_t hp[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int jq = 0; jq < NQ; ++jq) {
            const uint4 w = smem[kg * (N + 1) + q * NQ + jq];
            z[4 * jq + 0] = mac2(z[4 * jq + 0], hp[q], w.x);
            z[4 * jq + 1] = mac2(z[4 * jq + 1], hp[q], w.y);
            z[4 * jq + 2] = mac2(z[4 * jq + 2], hp[q], w.z);
            z[4 * jq + 3] = mac2(z[4 * jq + 3], hp[q], w.w);
        }
    }
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

// two fp32 values to a packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(float2_t{lo, hi}, bf16x2_t));
}

// The same for a piece of the state x that the router reads through an RMSNorm with weight w:
// z[j] += sum_k (x[k] * w[k]) * W_r[k, j].  A product x[k] * w[k] of two bf16 values has at most 16 significant
// bits: it enters the dot products EXACTLY as hi + lo, hi = the product rounded to bf16, lo = the rest (at
// most 8 significant bits, so a bf16 value itself).  Each router weight is read from LDS once and multiplied
// with both.  One k-pair at a time, so that only one (hi, lo) pair is live.
template <int N>
__device__ __forceinline__ void router_piece_scaled(float (&z)[N], const uint4 *smem, int kgroups, const uint4 &xv,
                                                    const uint32_t *wv, int kg)
{
    constexpr int NQ = N / 4;
    const uint32_t xp[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t wq = wv[q];
        const float a0 = bf16lo(xp[q]) * bf16lo(wq), a1 = bf16hi(xp[q]) * bf16hi(wq);
        const uint32_t hi = cvt_pk_bf16(a0, a1);
        const uint32_t lo = cvt_pk_bf16(a0 - bf16lo(hi), a1 - bf16hi(hi));
#pragma unroll
        for (int jq = 0; jq < NQ; ++jq) {
            const uint4 w = smem[kg * (N + 1) + q * NQ + jq];
            z[4 * jq + 0] = mac2(mac2(z[4 * jq + 0], hi, w.x), lo, w.x);
            z[4 * jq + 1] = mac2(mac2(z[4 * jq + 1], hi, w.y), lo, w.y);
            z[4 * jq + 2] = mac2(mac2(z[4 * jq + 2], hi, w.z), lo, w.z);
            z[4 * jq + 3] = mac2(mac2(z[4 * jq + 3], hi, w.w), lo, w.w);
        }
    }
}

// The norm weight [d] sits in LDS behind the router weight when the kernel applies the RMSNorm itself
// (one 16-byte piece per k-group, read by the lane that owns the k-group).
__host__ __device__ constexpr size_t norm_lds_bytes(int d) { return (size_t)d * 2; }
__device__ __forceinline__ void fill_norm_lds(uint4 *lnw_lds, const uint16_t *ln_w, int kgroups, int nthreads)
{
    for (int i = threadIdx.x; i < kgroups; i += nthreads)
        lnw_lds[i] = *reinterpret_cast<const uint4 *>(ln_w + 8 * i);
}

// Router equation for one token on one wavefront: returns, in lane l, the gate of expert
// l / (64/N) (softmax over all N experts of h . r_j).  h0 / h1 are the lane's pieces of the first
// two 512-column chunks, already loaded by the caller; further chunks are loaded here.
// sum of the squares of the 8 bf16 values of one 16-byte piece
__device__ __forceinline__ float sumsq8(const uint4 &v)
{
    float s = bf16lo(v.x) * bf16lo(v.x);
    s = fmaf(bf16hi(v.x), bf16hi(v.x), s);
    s = fmaf(bf16lo(v.y), bf16lo(v.y), s);
    s = fmaf(bf16hi(v.y), bf16hi(v.y), s);
    s = fmaf(bf16lo(v.z), bf16lo(v.z), s);
    s = fmaf(bf16hi(v.z), bf16hi(v.z), s);
    s = fmaf(bf16lo(v.w), bf16lo(v.w), s);
    s = fmaf(bf16hi(v.w), bf16hi(v.w), s);
    return s;
}

// NORM: hrow is the state x BEFORE the RMSNorm in front of the router (inference listing: the router reads the
// post-attention-normed state).  With hn = x / rms(x) * ln_w the logits are
//     hn . r_j = (1 / rms(x)) * sum_k (x_k ln_w_k) W_r[k, j],
// and x_k ln_w_k enters the dot products exactly, as a pair of bf16 values (router_piece_scaled), so the only
// roundings are those of the fp32 accumulation and of 1 / rms.  lnw: the norm weight in LDS.
template <int N, bool NTA, bool NORM = false, int NREAL = N>
__device__ __forceinline__ float router_gate(const uint4 *smem, int kgroups, const uint16_t *hrow, int d, int lane,
                                             const uint4 &h0, const uint4 &h1, float eps = 0.f,
                                             const uint4 *lnw = nullptr)
{
    constexpr int LPJ = 64 / N;
    const int col0 = lane * 8;
    float rs = 1.f;
    if constexpr (NORM) {
        // 1 / rms first, while few registers are live (pieces past the end of the row were loaded as zeros)
        float ss = sumsq8(h0) + sumsq8(h1);
        for (int c0 = 1024; c0 < d; c0 += 512)
            if (c0 + col0 < d)
                ss += sumsq8(ld16_stream<NTA>(hrow + c0 + col0));
        ss = span_reduce<32, 1, OpAdd>(ss);
        rs = __builtin_amdgcn_rsqf(ss / (float)d + eps);
    }
    float z[N];
#pragma unroll
    for (int j = 0; j < N; ++j)
        z[j] = 0.f;
    if constexpr (NORM) {
        if (col0 < d)
            router_piece_scaled<N>(z, smem, kgroups, h0, reinterpret_cast<const uint32_t *>(lnw + (col0 >> 3)), col0 >> 3);
        if (col0 + 512 < d)
            router_piece_scaled<N>(z, smem, kgroups, h1, reinterpret_cast<const uint32_t *>(lnw + ((col0 + 512) >> 3)),
                                   (col0 + 512) >> 3);
        for (int c0 = 1024; c0 < d; c0 += 512) {
            const int cc = c0 + col0;
            if (cc < d)
                router_piece_scaled<N>(z, smem, kgroups, ld16_stream<NTA>(hrow + cc),
                                       reinterpret_cast<const uint32_t *>(lnw + (cc >> 3)), cc >> 3);
        }
    } else {
        if (col0 < d)
            router_piece<N>(z, smem, kgroups, h0, col0 >> 3);
        if (col0 + 512 < d)
            router_piece<N>(z, smem, kgroups, h1, (col0 + 512) >> 3);
        for (int c0 = 1024; c0 < d; c0 += 512) {
            const int cc = c0 + col0;
            if (cc < d)
                router_piece<N>(z, smem, kgroups, ld16_stream<NTA>(hrow + cc), cc >> 3);
        }
    }
    float zz = Fold<N, 32>::run(z, lane) * rs;
    if constexpr (NREAL < N) {
        if (lane / LPJ >= NREAL)
            zz = -INFINITY;                 // a padded expert: gate exactly 0
    }
    const float m = span_reduce<32, LPJ, OpMax>(zz);
    const float e = __expf(zz - m);
    const float s = span_reduce<32, LPJ, OpAdd>(e);
    return e / s;
}

// the lane's pieces of h for the first two chunks (zero where the chunk does not exist)
template <bool NTA>
__device__ __forceinline__ void load_h2(uint4 &h0, uint4 &h1, const uint16_t *hrow, int d, int lane)
{
    const int col0 = lane * 8;
    h0 = col0 < d ? ld16_stream<NTA>(hrow + col0) : make_uint4(0, 0, 0, 0);
    h1 = col0 + 512 < d ? ld16_stream<NTA>(hrow + col0 + 512) : make_uint4(0, 0, 0, 0);
}

// acc[0..7] += g * (the 8 bf16 values of one 16-byte piece)
__device__ __forceinline__ void fma8(float (&acc)[8], float g, const uint4 &rr)
{
    acc[0] = fmaf(g, bf16lo(rr.x), acc[0]);
    acc[1] = fmaf(g, bf16hi(rr.x), acc[1]);
    acc[2] = fmaf(g, bf16lo(rr.y), acc[2]);
    acc[3] = fmaf(g, bf16hi(rr.y), acc[3]);
    acc[4] = fmaf(g, bf16lo(rr.z), acc[4]);
    acc[5] = fmaf(g, bf16hi(rr.z), acc[5]);
    acc[6] = fmaf(g, bf16lo(rr.w), acc[6]);
    acc[7] = fmaf(g, bf16hi(rr.w), acc[7]);
}

__device__ __forceinline__ void add8(float (&acc)[8], const uint4 &v)
{
    acc[0] += bf16lo(v.x);
    acc[1] += bf16hi(v.x);
    acc[2] += bf16lo(v.y);
    acc[3] += bf16hi(v.y);
    acc[4] += bf16lo(v.z);
    acc[5] += bf16hi(v.z);
    acc[6] += bf16lo(v.w);
    acc[7] += bf16hi(v.w);
}

__device__ __forceinline__ uint4 pack8(const float (&acc)[8])
{
    uint4 o;
    o.x = pack_bf16(acc[0], acc[1]);
    o.y = pack_bf16(acc[2], acc[3]);
    o.z = pack_bf16(acc[4], acc[5]);
    o.w = pack_bf16(acc[6], acc[7]);
    return o;
}

// eight fp32 values to bf16, round to nearest even, with the packed conversion instruction (one per pair);
// for the kernels that are bound by vector instruction issue: the integer sequence of pack8 costs about
// twelve instructions per pair.  (NaN inputs give the instruction's quiet NaN, not 0x7fc0.)
__device__ __forceinline__ uint4 pack8_cvt(const float (&acc)[8])
{
    return make_uint4(cvt_pk_bf16(acc[0], acc[1]), cvt_pk_bf16(acc[2], acc[3]), cvt_pk_bf16(acc[4], acc[5]),
                      cvt_pk_bf16(acc[6], acc[7]));
}

// ---- tile kernel of the bf16 forward (fwd_tile.hip): arguments and host-side launcher ----
struct TileArgs {
    const void *table;
    const int32_t *rowsrc;      // slot if given, else ids
    const void *h;
    const void *W_r;
    const void *shared;
    const void *residual;
    void *out;
    float *gates_dbg;
    int64_t *rows_dbg;
    int32_t *err_flag;
    const int32_t *plan;
    const void *ln_w;           // not NULL: h is the state before the RMSNorm, which is also the residual
    float ln_eps;
    int64_t table_stride, act_stride, rows;
    int T, d;
};
bool tile_forward_applies(int N, int d, int T, int L);
mole_status launch_tile_forward(const TileArgs &a, int N, int L, hipStream_t stream);
// steps 1 and 2 of the tile kernel alone, tokens in their own order: gates [L, T, N] fp32 = softmax(h . W_r), N = 32;
// ln_w not NULL: h is the state before the RMSNorm the router reads it through
mole_status launch_tile_router(const void *h, const void *W_r, const void *ln_w, float ln_eps, float *gates, int T,
                               int d, int N, int L, int64_t act_stride, hipStream_t stream);
// step 3 alone, gates given (a.gates_dbg is not used), one wave per token in the visiting order
mole_status launch_tile_gather(const TileArgs &a, const float *gates, int N, int L, hipStream_t stream);

}  // namespace mole
#endif
