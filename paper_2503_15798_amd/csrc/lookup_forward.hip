// mole_lookup_forward: fused router + softmax + row gather + gate-weighted sum + adds.
//
// Paper: Sec. 3.2 (router equation: full softmax over all N experts) and Sec. 3.3
// (inference-layer equation: h' = sum_j g_j v^id_j + FFN_shared(h) + h).
//
// The path is bound by HBM bandwidth (about 1.7 flop per byte); the streaming kernel below does its
// arithmetic on the vector ALU.  (The run kernel further down, for large batches that come with a
// plan, sums groups of tokens with equal ids on the matrix pipe.)
// One 64-lane wavefront owns a token:
//   * lane l owns columns [512*c + 8*l, +8) of every row: every table access is a 16-byte
//     load and a wavefront covers 1 KiB of a row per load;
//   * the N row registers form a ring that is refilled as it is consumed (next 512-column
//     chunk, or the wave's next token), so N loads per lane are in flight at all times;
//   * the router weight lives in LDS for the life of the workgroup, stored as (k, k+1) bf16
//     pairs so that the lane's 16-byte piece of h meets it without repacking
//     (v_dot2_f32_bf16: two multiply-adds per instruction, fp32 accumulation); the N partial
//     logits of the 64 lanes are folded with a halving butterfly (N/2 + N/4 + ... exchanges
//     instead of 6 per logit), softmax runs on the folded values, gates move to scalar
//     registers with v_readlane;
//   * the combine multiplies from registers and adds shared / residual in the epilogue, with
//     a single round-to-nearest-even to bf16 at the (non-temporal) store.
// Waves never synchronise with each other after the router weight is in LDS.
#include "fwd_common.h"

namespace {
using namespace mole;

struct FwdArgs {
    const void *table;
    const int32_t *ids;
    const int32_t *slot;
    const void *h;
    const void *W_r;
    const void *shared;
    const void *residual;
    void *out;
    float *gates_dbg;
    int64_t *rows_dbg;
    int32_t *err_flag;
    const int32_t *plan;
    const void *ln_w;       // [L, d] weight of the RMSNorm in front of the router, or NULL.  Not NULL: h is the
    float ln_eps;           // state BEFORE that norm; the kernel applies it and adds the state as the residual
    int64_t table_stride;   // per layer, elements
    int64_t act_stride;     // per layer, elements
    int64_t rows;
    int T, d, N, L;
};

// ------------------------------------------------------------------------------------------
// bf16 streaming kernel.  The wave's N row registers are a ring: as soon as the rows of the
// current 512-column chunk have been multiplied in, the same registers are re-loaded with the
// next chunk -- or with chunk 0 of the wave's NEXT token when this was the last chunk -- so N
// 16-byte loads per lane are in flight through the router, the multiply phase and the epilogue
// alike; the next token's router input is prefetched the same way.
// Table rows are loaded with plain (cacheable) loads: repeated ids are then served by L2 /
// Infinity Cache.  Rows that the plan marks as read-once use non-temporal loads.
// N in {2, 4, 8, 16, 32, 64}, d % 8 == 0, router weight fits in LDS.  grid = (workgroups, L).
// ------------------------------------------------------------------------------------------
template <int N, bool NT>
__device__ __forceinline__ void ring_load(uint4 (&r)[N], const uint16_t *base, int d, int col)
{
#pragma unroll
    for (int j = 0; j < N; ++j)
        r[j] = ld16_row<NT>(base + (int64_t)j * d + col);
}

// SPLIT: small launches are bound by latency, not bandwidth.  There a work item is one 512-column
// chunk of a token instead of a whole token, so that the chunks of a token are fetched and combined
// by different waves at the same time (each computes the token's gates itself: the router is cheap
// next to a second memory round trip).
// NORM: a.h is the state after attention and a.ln_w the weight of the RMSNorm the router reads it through;
// the state times the norm weight enters the router exactly (router_gate), the token's 1/rms scales the
// logits, and the same state is the residual of the epilogue.
// DBG: a.gates_dbg / a.rows_dbg are written.  A variant of its own: in the kernel that serves every other call the two
// pointers and their tests stay out of the loop's scalar registers (24 x 256 decode step 37.2 -> 36.9 us, with a
// plan 35.0 -> 34.5 us, 12 x 64 tokens 9.8 -> 9.4 us).
template <int N, int WPB, bool NTA, bool SPLIT, bool NORM, bool DBG>
__global__ __launch_bounds__(WPB * 64) __attribute__((amdgpu_waves_per_eu(N <= 32 ? 4 : 2)))
void fwd_bf16_stream_kernel(FwdArgs a)
{
    extern __shared__ uint4 smem[];
    constexpr int NR = N < 4 ? 4 : N;   // experts the router is computed for (N = 2 is padded to 4)
    constexpr int LPJ = 64 / NR;        // lanes per expert after the fold
    // row registers: above 16 experts a chunk's rows pass through in parts of 16 (of 8 in the N = 32 norm variant,
    // whose router keeps more values live: with 16 it spills 40 to 80 registers and takes 290 instead of 235 us on
    // the 16384-token prefill)
    constexpr int R = N > 16 ? (NORM && N == 32 ? 8 : 16) : N;
    constexpr int H = N / R;
    // NORM: the state is also the residual; below 16 experts its two pieces stay in registers through the
    // combine, from 16 experts on (kernels at their 128-register budget) they are read again (an L2 hit)
    constexpr bool HOLD_X = NORM && N < 16;
    const int d = a.d;
    const int kgroups = d >> 3;
    const int layer = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col0 = lane * 8;
    const int T = a.T;
    const int nch = SPLIT ? (d + 511) >> 9 : 1;     // items per token
    const int n_items = T * nch;

    const uint16_t *table = static_cast<const uint16_t *>(a.table) + (int64_t)layer * a.table_stride;
    const int64_t act_off = (int64_t)layer * a.act_stride;
    const uint16_t *hbase = static_cast<const uint16_t *>(a.h) + act_off;
    const uint16_t *sbase = a.shared ? static_cast<const uint16_t *>(a.shared) + act_off : nullptr;
    const uint16_t *rbase = a.residual ? static_cast<const uint16_t *>(a.residual) + act_off : nullptr;
    uint16_t *obase = static_cast<uint16_t *>(a.out) + act_off;
    const int32_t *rowsrc = a.slot ? a.slot : a.ids;
    const int stride = gridDim.x * WPB;
    const int32_t *order = nullptr;
    if (a.plan && plan_ok(a))      // a foreign plan: flagged, tokens visited in their own order
        order = a.plan + plan_layout(T).order;

    // Order of the first requests.  The longest chain is (plan entry ->) id -> rows, so the id is asked for first;
    // what depends on no id follows while it travels: the first item's router input and the router weight, which
    // goes to LDS as soon as it is there (its registers are free again before the row registers fill).  Memory
    // returns a wave's loads in order, so by then the id has arrived too and the rows are requested at once; the
    // router then runs while they travel.  An earlier version requested the rows first: router input and weight
    // arrived behind the 16 KB of row pieces, the router could not start before the rows were there, and on a
    // single-layer call of 256 tokens the waves spent a third of their life waiting that way.  Lanes past the end
    // of a ragged chunk load a clamped (valid) column; their results are never stored.
    const int dlast = d - 8;
    int item = blockIdx.x * WPB + wave;
    Visit cur = item < n_items ? visit(order, SPLIT ? item / nch : item) : Visit{0, false};
    int cbase = SPLIT ? (item % nch) << 9 : 0;      // first column of this item
    const int32_t id_first = item < n_items ? ld_scalar(rowsrc, cur.t) : -1;      // requested; used further down
    uint4 h0, h1;
    load_h2<NTA>(h0, h1, hbase + (int64_t)cur.t * d, d, lane);
    // NORM: the norm weight behind the router weight in LDS; it travels with the router weight (asked for behind the
    // rows it would arrive behind them, and the barrier below would wait for the rows)
    uint4 *lnw_fill = smem + router_lds_bytes(d, NR) / 16;
    const uint16_t *lnw_src = static_cast<const uint16_t *>(a.ln_w) + (int64_t)layer * d;
    uint4 lnw_first = make_uint4(0, 0, 0, 0);
    if constexpr (NORM)
        if ((int)threadIdx.x < kgroups)
            lnw_first = *reinterpret_cast<const uint4 *>(lnw_src + 8 * threadIdx.x);
    fill_router_lds<NR, N>(smem, static_cast<const uint16_t *>(a.W_r) + (int64_t)layer * d * N, kgroups, WPB * 64);
    if constexpr (NORM) {
        if ((int)threadIdx.x < kgroups)
            lnw_fill[threadIdx.x] = lnw_first;
        for (int i = threadIdx.x + WPB * 64; i < kgroups; i += WPB * 64)
            lnw_fill[i] = *reinterpret_cast<const uint4 *>(lnw_src + 8 * i);
    }
    // every load so far has arrived (the weight's were the last): said out loud, because a lane without a share of the
    // weight skips the fill's waits, and the compiler would then wait for the router input behind the rows
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0)

    int64_t row = (int64_t)__builtin_amdgcn_readfirstlane(id_first);
    bool valid = row >= 0 && row < a.rows;
    uint4 r[R];
    if (valid) {
        const uint16_t *rp0 = table + row * (int64_t)N * d;
        if (cur.single)
            ring_load<R, true>(r, rp0, d, min(cbase + col0, dlast));
        else
            ring_load<R, false>(r, rp0, d, min(cbase + col0, dlast));
    }
    const uint4 *lnw = lnw_fill;
    __syncthreads();

    // The first item's gates are computed here and every later item's at the bottom of the loop.  At this point the
    // compiler knows that the router input has arrived (it was waited for before the rows were requested), so the
    // router runs with the rows in flight.  At the head of a loop it cannot know: loads counted on different paths
    // meet there, and it waits for every load in flight, the row pieces included.
    float g = 0.f;
    if (item < n_items)
        g = router_gate<NR, NTA, NORM, N>(smem, kgroups, hbase + (int64_t)cur.t * d, d, lane, h0, h1, a.ln_eps, lnw);

    bool bad_seen = false;
    for (; item < n_items; item += stride) {
        const int t = cur.t;
        const int nitem = item + stride;
        const Visit nxt = nitem < n_items ? visit(order, SPLIT ? nitem / nch : nitem) : Visit{0, false};
        const int ncbase = SPLIT ? (nitem % nch) << 9 : 0;
        const int64_t nrow = nitem < n_items ? (int64_t)ld_scalar(rowsrc, nxt.t) : -1;
        const bool nvalid = nrow >= 0 && nrow < a.rows;
        const bool reporter = !SPLIT || cbase == 0;    // one item per token reports flags and debug outputs
        bad_seen |= !valid;                             // reported once, when the wave is done
        if (DBG && a.rows_dbg && layer == 0 && lane == 0 && reporter)
            a.rows_dbg[t] = valid ? row : -1;

        if (DBG && a.gates_dbg && reporter && (lane & (LPJ - 1)) == 0 && lane / LPJ < N)
            a.gates_dbg[((int64_t)layer * T + t) * N + lane / LPJ] = g;
        const uint4 x0 = h0, x1 = h1;                  // NORM: the residual of chunks 0 and 1
        // the next token's h goes in flight now; its latency hides behind this token's combine
        load_h2<NTA>(h0, h1, hbase + (int64_t)nxt.t * d, d, lane);
        // gates into scalar registers: expert j's gate sits in lane j * (64/N)
        float gs[R];
        if constexpr (H == 1) {
#pragma unroll
            for (int j = 0; j < N; ++j)
                gs[j] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, g), j * LPJ));
        }

        const uint16_t *rp = table + (valid ? row : 0) * (int64_t)N * d;
        const uint16_t *nrp = table + (nvalid ? nrow : 0) * (int64_t)N * d;
        const int cend = SPLIT ? min(cbase + 512, d) : d;
        for (int c0 = cbase; c0 < cend; c0 += 512) {
            const int cc = c0 + col0;
            const bool on = cc < d;
            const bool last = c0 + 512 >= cend;
            const int64_t off = (int64_t)t * d + cc;
            uint4 sv = make_uint4(0, 0, 0, 0), rv = make_uint4(0, 0, 0, 0);
            if (on && sbase)
                sv = ld16_stream<NTA>(sbase + off);
            if constexpr (NORM) {
                // the residual is the state itself: kept in registers unless that would spill (N = 16 with
                // non-temporal loads sits at its 128-register budget), else read a second time
                if (HOLD_X && c0 == 0)
                    rv = x0;
                else if (HOLD_X && c0 == 512)
                    rv = x1;
                else if (on)
                    rv = ld16_stream<NTA>(hbase + off);
            } else if (on && rbase) {
                rv = ld16_stream<NTA>(rbase + off);
            }
            float acc[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                acc[e] = 0.f;
            if constexpr (H == 1) {
                if (valid) {
    #pragma unroll
                    for (int j = 0; j < N; ++j)
                        fma8(acc, gs[j], r[j]);
                }
                // refill the ring: next chunk of this item, or the first chunk of the wave's next item
                const uint16_t *fb = last ? nrp : rp;                      // wave-uniform
                const int fcol = min(last ? ncbase + col0 : cc + 512, dlast);
                if (last ? nvalid : valid) {
                    if (last ? nxt.single : cur.single)
                        ring_load<R, true>(r, fb, d, fcol);
                    else
                        ring_load<R, false>(r, fb, d, fcol);
                }
            } else {
                // N > 16: the chunk's experts pass through the row registers in parts of R
#pragma unroll
                for (int hf = 0; hf < H; ++hf) {
#pragma unroll
                    for (int j = 0; j < R; ++j)
                        gs[j] = __builtin_bit_cast(
                            float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, g), (hf * R + j) * LPJ));
                    if (valid) {
#pragma unroll
                        for (int j = 0; j < R; ++j)
                            fma8(acc, gs[j], r[j]);
                    }
                    // refill: the next half of this chunk, else the next chunk / the wave's next item
                    const bool more_halves = hf + 1 < H;
                    const uint16_t *fb = more_halves ? rp + (int64_t)(hf + 1) * R * d : (last ? nrp : rp);
                    const int fcol = min(more_halves ? cc : (last ? ncbase + col0 : cc + 512), dlast);
                    if (more_halves || !last ? valid : nvalid) {
                        if (more_halves || !last ? cur.single : nxt.single)
                            ring_load<R, true>(r, fb, d, fcol);
                        else
                            ring_load<R, false>(r, fb, d, fcol);
                    }
                }
            }
            add8(acc, sv);
            add8(acc, rv);
            if (on)
                st16_stream(obase + off, N >= 32 ? pack8_cvt(acc) : pack8(acc));
        }
        if (nitem < n_items)        // the next item's gates (its rows are on their way)
            g = router_gate<NR, NTA, NORM, N>(smem, kgroups, hbase + (int64_t)nxt.t * d, d, lane, h0, h1, a.ln_eps, lnw);
        row = nrow;
        valid = nvalid;
        cur = nxt;
        cbase = ncbase;
    }
    // an id outside the table: one atomic per wave, here and not in the loop (a memory operation on a branch in
    // front of the router makes the compiler wait there for every load in flight, the row pieces included)
    if (bad_seen && lane == 0 && a.err_flag)
        atomicOr(a.err_flag, 1);
}

// ------------------------------------------------------------------------------------------
// Run kernel (MOLE_FLAG_RUNS; needs the plan of mole_dedup_ids): the plan lists the tokens in id order, so
// tokens with equal ids sit next to each other.  A wave takes 4 consecutive positions of that order (a span) and
// cuts them into groups with the same row block; an item is one 512-column chunk of one group:
//   * the N row pieces of the chunk are fetched once for the whole group, and the gate-weighted sums
//     of its (up to) 4 tokens are taken together on the matrix pipe: v_mfma_f32_4x4x4_16b_bf16
//     computes, in each of its 16 blocks of 4 lanes, a 4x4 product D[i][j] += sum_k A[i][k] B[k][j]
//     where lane 4b+i supplies row i of A, lane 4b+j supplies column j of B and receives column j of
//     D.  With A = the gates of the group's tokens for 4 experts and B = the lane's own column of
//     those 4 experts' rows, every lane gets the sums of its own columns for 4 tokens at once, from
//     bf16 table values as they are (no conversion on the vector ALU, which is what limits the
//     streaming kernel at N = 32: two instructions per table element);
//   * the matrix instruction takes bf16 operands, so each gate is split into hi + lo (hi = the gate
//     rounded to bf16, lo = the rounded rest: 16 significant bits; the products with bf16 table
//     values are still exact in fp32);
//   * router and softmax are the streaming kernel's; the gates of a span are computed one position
//     at a time between the items of the span before it and handed over through LDS;
//   * the registers of an expert quad are refilled with the next item's pieces as soon as the
//     quad's operands have been built, and the next item's shared / residual pieces are requested
//     after this item's stores, so both travel while this item and the gates run;
//   * shared / residual are added and the result is rounded and stored per token, as elsewhere.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Row pieces come through buffer loads: base and size of a row block sit in a scalar descriptor, the
// expert's offset in a scalar register, the lane's column offset is the only vector operand.  Lanes
// past the end of the block read zeros (ragged last chunk); their results are never stored.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_block_rsrc(const uint16_t *block, int bytes)
{
    constexpr int RAW_32BIT = 0x00020000;   // untyped buffer, 32-bit data format
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(block), 0, bytes, RAW_32BIT);
}

// the 16-byte pieces of experts J0 .. J0+CNT-1 of one 512-column chunk
template <int N, int J0, int CNT, bool NT>
__device__ __forceinline__ void rows_load_buf(uint4 (&r)[N], __amdgpu_buffer_rsrc_t rs, int d, uint32_t lane_bytes,
                                              int chunk_bytes)
{
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
#pragma unroll
    for (int j = J0; j < J0 + CNT && j < N; ++j) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_bytes, j * d * 2 + chunk_bytes, NT ? 2 : 0);
        r[j] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

typedef __attribute__((ext_vector_type(4))) short bf16x4_bits;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ uint32_t dword_of(const uint4 &v, int i)
{
    return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}

// B operands of expert quad Q: for each of the lane's 8 columns, the values of experts 4Q .. 4Q+3
template <int N, int Q>
__device__ __forceinline__ void quad_columns(bf16x4_bits (&bcol)[8], const uint4 (&r)[N])
{
    const uint4 zero = make_uint4(0, 0, 0, 0);
    const uint4 &r0 = r[4 * Q];
    const uint4 &r1 = 4 * Q + 1 < N ? r[4 * Q + 1] : zero;
    const uint4 &r2 = 4 * Q + 2 < N ? r[4 * Q + 2] : zero;
    const uint4 &r3 = 4 * Q + 3 < N ? r[4 * Q + 3] : zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        // column e of the four rows: the low or high halves of dword e/2
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        const uint32_t b01 = __builtin_amdgcn_perm(dword_of(r1, e >> 1), dword_of(r0, e >> 1), sel);
        const uint32_t b23 = __builtin_amdgcn_perm(dword_of(r3, e >> 1), dword_of(r2, e >> 1), sel);
        bcol[e] = __builtin_bit_cast(bf16x4_bits, make_uint2(b01, b23));
    }
}

// acc[e][i] += sum over the 4 experts of a quad of gate[token i][expert] * row[expert][lane's column e].
// ga: this lane's A operand (gates of token lane & 3: hi in x, y; lo in z, w).
__device__ __forceinline__ void quad_products(f32x4 (&acc)[8], const bf16x4_bits (&bcol)[8], const uint4 &ga)
{
    const bf16x4_bits ahi = __builtin_bit_cast(bf16x4_bits, make_uint2(ga.x, ga.y));
    const bf16x4_bits alo = __builtin_bit_cast(bf16x4_bits, make_uint2(ga.z, ga.w));
#pragma unroll
    for (int e = 0; e < 8; ++e)
        acc[e] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ahi, bcol[e], acc[e], 0, 0, 0);
#pragma unroll
    for (int e = 0; e < 8; ++e)
        acc[e] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(alo, bcol[e], acc[e], 0, 0, 0);
}

// One item: the products of all expert quads with the held row pieces; each quad's registers are
// refilled with the next item's pieces (if FETCH) as soon as its operands have been built, so those
// loads travel while the rest of this item runs.
template <int N, int Q>
__device__ __forceinline__ void item_quads(f32x4 (&acc)[8], uint4 (&r)[N], const uint4 *ga, bool compute, bool fetch,
                                           bool fetch_once, __amdgpu_buffer_rsrc_t next_rs, int d, uint32_t lane_bytes,
                                           int next_chunk_bytes)
{
    constexpr int NQ = (N + 3) / 4;
    if constexpr (Q < NQ) {
        bf16x4_bits bcol[8];
        if (compute)
            quad_columns<N, Q>(bcol, r);
        if (fetch) {
            if (fetch_once)     // rows the plan marks as read-once: non-temporal
                rows_load_buf<N, 4 * Q, 4, true>(r, next_rs, d, lane_bytes, next_chunk_bytes);
            else
                rows_load_buf<N, 4 * Q, 4, false>(r, next_rs, d, lane_bytes, next_chunk_bytes);
        }
        if (compute)
            quad_products(acc, bcol, ga[Q]);
        __builtin_amdgcn_sched_barrier(0);      // keep the quads apart: hoisting all operand builds would spill
        item_quads<N, Q + 1>(acc, r, ga, compute, fetch, fetch_once, next_rs, d, lane_bytes, next_chunk_bytes);
    }
}

constexpr int RUN_GROUP = 4;    // tokens per matrix instruction (its M dimension) = positions per span

// RES: a residual is added (NORM: the state itself, else a.residual)
template <int N, int WPB, bool NORM, bool RES>
__global__ __launch_bounds__(WPB * 64) __attribute__((amdgpu_waves_per_eu(2)))
void fwd_bf16_run_kernel(FwdArgs a)
{
    static_assert(RES || !NORM, "the norm variant always adds the state");
    constexpr int G = RUN_GROUP;
    extern __shared__ uint4 smem[];
    constexpr int NR = N < 4 ? 4 : N;
    constexpr int NQ = NR / 4;
    constexpr int LPJ = 64 / NR;
    const int d = a.d;
    const int kgroups = d >> 3;
    const int layer = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col0 = lane * 8;
    const int T = a.T;
    const int nch = (d + 511) >> 9;
    const int nspans = (T + G - 1) / G;

    const uint16_t *table = static_cast<const uint16_t *>(a.table) + (int64_t)layer * a.table_stride;
    const int64_t act_off = (int64_t)layer * a.act_stride;
    const uint16_t *hbase = static_cast<const uint16_t *>(a.h) + act_off;
    const uint16_t *sbase = a.shared ? static_cast<const uint16_t *>(a.shared) + act_off : nullptr;
    const uint16_t *rbase = a.residual ? static_cast<const uint16_t *>(a.residual) + act_off : nullptr;
    uint16_t *obase = static_cast<uint16_t *>(a.out) + act_off;
    const int32_t *rowsrc = a.slot ? a.slot : a.ids;
    const int stride = gridDim.x * WPB;
    // a foreign plan is flagged and replaced by the identity order (every token its own group)
    const int32_t *order = plan_ok(a) ? a.plan + plan_layout(T).order : nullptr;
    // the wave's gates behind the router weight, for the span being combined and for the next one:
    // [2][G][NQ] pieces of 16 bytes = 4 experts x (hi, lo)
    const uint4 *lnw = smem + router_lds_bytes(d, NR) / 16;     // NORM: the norm weight, then the gates
    uint4 *gq = smem + (router_lds_bytes(d, NR) + (NORM ? norm_lds_bytes(d) : 0)) / 16 + wave * (2 * G * NQ);

    // Span descriptor: lane i holds position i's plan entry (token index, read-once flag in bit 31)
    // and row block; -1 = no such position / id outside the table.
    struct Span { int32_t t, row; };
    auto load_span = [&](int s) {
        Span sp{-1, -1};
        const int p = s * G + lane;
        if (s < nspans && lane < G && p < T) {
            sp.t = order ? order[p] : p;
            const int32_t rr = rowsrc[sp.t & ~PLAN_SINGLE];
            sp.row = rr >= 0 && rr < a.rows ? rr : -1;
        }
        return sp;
    };
    auto span_len = [&](int s) { return s < nspans ? min(G, T - s * G) : 0; };
    auto token_of = [&](const Span &sp, int i) { return (int)(__builtin_amdgcn_readlane(sp.t, i) & ~PLAN_SINGLE); };
    // group starting at position i: row block (wave-uniform), length 1..4, read-once flag
    struct Group { int32_t row; int len; bool single; };
    auto group_at = [&](const Span &sp, int i, int np) {
        Group g;
        g.row = __builtin_amdgcn_readlane(sp.row, i);
        g.single = (uint32_t)__builtin_amdgcn_readlane(sp.t, i) >> 31;
        g.len = 1;
        if (g.row >= 0) {
#pragma unroll
            for (int m = 1; m < G; ++m)
                if (g.len == m && i + m < np && __builtin_amdgcn_readlane(sp.row, i + m) == g.row)
                    g.len = m + 1;
        }
        return g;
    };
    uint4 r[N];
    auto issue_rows = [&](const Group &g, int c) {
        if (g.row < 0)
            return;
        const __amdgpu_buffer_rsrc_t rs = row_block_rsrc(table + (int64_t)g.row * N * d, N * d * 2);
        if (g.single)
            rows_load_buf<N, 0, N, true>(r, rs, d, lane * 16u, c << 10);
        else
            rows_load_buf<N, 0, N, false>(r, rs, d, lane * 16u, c << 10);
    };
    // router + softmax of position j of span sp (its router input is in h0 / h1); the gates go to gdst
    // as hi + lo bf16 pairs
    auto gates_of = [&](const Span &sp, int j, const uint4 &h0, const uint4 &h1, uint4 *gdst) {
        const int t = token_of(sp, j);
        const int32_t row = __builtin_amdgcn_readlane(sp.row, j);
        if (row < 0 && lane == 0 && a.err_flag)
            atomicOr(a.err_flag, 1);
        if (a.rows_dbg && layer == 0 && lane == 0)
            a.rows_dbg[t] = row;
        const float g = router_gate<NR, false, NORM, N>(smem, kgroups, hbase + (int64_t)t * d, d, lane, h0, h1, a.ln_eps, lnw);
        if ((lane & (LPJ - 1)) == 0) {
            const int e = lane / LPJ;
            if (a.gates_dbg && e < N)
                a.gates_dbg[((int64_t)layer * T + t) * N + e] = g;
            const uint32_t hi = f32_to_bf16_bits(g);
            const uint32_t lo = f32_to_bf16_bits(g - __uint_as_float(hi << 16));
            uint16_t *piece = reinterpret_cast<uint16_t *>(gdst) + ((j * NQ + (e >> 2)) << 3);
            piece[e & 3] = (uint16_t)hi;
            piece[4 + (e & 3)] = (uint16_t)lo;
        }
    };

    // shared / residual pieces of chunk c for the (up to) 4 tokens of the group at position i of span sp
    uint4 sv[G], rv[RES ? G : 1];
    int tok[G];
    auto load_act = [&](const Span &sp, int i, int len, int c) {
        const int cc = (c << 9) + col0;
#pragma unroll
        for (int m = 0; m < G; ++m) {
            sv[m] = make_uint4(0, 0, 0, 0);
            if constexpr (RES)
                rv[m] = make_uint4(0, 0, 0, 0);
            tok[m] = 0;
            if (m < len) {
                tok[m] = token_of(sp, i + m);
                const int64_t off = (int64_t)tok[m] * d + cc;
                if (cc < d && sbase)
                    sv[m] = ld16_stream<false>(sbase + off);
                if constexpr (RES) {
                    if (cc < d)
                        rv[m] = ld16_stream<false>((NORM ? hbase : rbase) + off);
                }
            }
        }
    };

    int s = blockIdx.x * WPB + wave;
    int ns = s + stride;
    Span cur_sp = load_span(s), nx_sp = load_span(ns);
    int np = span_len(s);
    Group cur = np > 0 ? group_at(cur_sp, 0, np) : Group{-1, 1, false};
    if (np > 0)
        issue_rows(cur, 0);
    uint4 h0 = make_uint4(0, 0, 0, 0), h1 = h0;
    if (np > 0)
        load_h2<false>(h0, h1, hbase + (int64_t)token_of(cur_sp, 0) * d, d, lane);

    fill_router_lds<NR, N>(smem, static_cast<const uint16_t *>(a.W_r) + (int64_t)layer * d * N, kgroups, WPB * 64);
    if constexpr (NORM)
        fill_norm_lds(smem + router_lds_bytes(d, NR) / 16, static_cast<const uint16_t *>(a.ln_w) + (int64_t)layer * d,
                      kgroups, WPB * 64);
    __syncthreads();

    // gates of the wave's first span; those of every later span are computed between the items of
    // the span before it, while that span's row pieces are in flight
    int buf = 0;
    for (int j = 0; j < np; ++j) {
        const uint4 c0 = h0, c1 = h1;
        if (j + 1 < np)
            load_h2<false>(h0, h1, hbase + (int64_t)token_of(cur_sp, j + 1) * d, d, lane);
        gates_of(cur_sp, j, c0, c1, gq);
    }
    wave_lds_fence();
    if (np > 0)
        load_act(cur_sp, 0, cur.len, 0);

    while (np > 0) {
        const int nns = ns + stride;
        const Span nn_sp = load_span(nns);      // descriptors run two spans ahead of their use
        const int nnp = span_len(ns);
        int rj = 0;                             // next position of the next span whose gates are due
        if (nnp > 0)
            load_h2<false>(h0, h1, hbase + (int64_t)token_of(nx_sp, 0) * d, d, lane);
        const uint4 *gcur = gq + buf * (G * NQ);
        uint4 *gnext = gq + (buf ^ 1) * (G * NQ);

        int i = 0, c = 0;
        while (i < np) {
            // the item after this one: next chunk of the group, else the next group of the span, else
            // the first group of the next span
            Group nxt = cur;
            int nc = c + 1;
            bool more = true;
            if (nc >= nch) {
                nc = 0;
                if (i + cur.len < np)
                    nxt = group_at(cur_sp, i + cur.len, np);
                else if (nnp > 0)
                    nxt = group_at(nx_sp, 0, nnp);
                else
                    more = false;
            }
            const int cc = (c << 9) + col0;
            const bool on = cc < d;

            f32x4 acc[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
            {
                // lane l supplies the gates of position min(i + (l & 3), G - 1); rows of D past the
                // group's length are not used.  The next item's pieces replace the held ones quad by
                // quad unless they are the same (same row block, same chunk).
                const uint4 *ga = gcur + min(i + (lane & 3), G - 1) * NQ;
                const bool fetch = more && nxt.row >= 0 && !(nxt.row == cur.row && nc == c);
                const __amdgpu_buffer_rsrc_t nrs =
                    row_block_rsrc(table + (int64_t)(fetch ? nxt.row : 0) * N * d, N * d * 2);
                item_quads<N, 0>(acc, r, ga, cur.row >= 0, fetch, nxt.single, nrs, d, lane * 16u, nc << 10);
            }

#pragma unroll
            for (int m = 0; m < G; ++m) {
                if (m < cur.len) {
                    float o[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        o[e] = acc[e][m];
                    add8(o, sv[m]);
                    if constexpr (RES)
                        add8(o, rv[m]);
                    if (on)
                        st16_stream(obase + (int64_t)tok[m] * d + cc, pack8_cvt(o));
                }
            }
            // the next item's shared / residual pieces go in flight now: they travel during the gates
            // below and the next item's products
            if (more) {
                if (nc != 0)
                    load_act(cur_sp, i, cur.len, nc);
                else if (i + cur.len < np)
                    load_act(cur_sp, i + cur.len, nxt.len, 0);
                else
                    load_act(nx_sp, 0, nxt.len, 0);
            }
            // while the row pieces travel: the gates of one position of the next span
            if (rj < nnp) {
                const uint4 c0 = h0, c1 = h1;
                if (rj + 1 < nnp)
                    load_h2<false>(h0, h1, hbase + (int64_t)token_of(nx_sp, rj + 1) * d, d, lane);
                gates_of(nx_sp, rj, c0, c1, gnext);
                ++rj;
            }
            if (nc == 0)
                i += cur.len;
            c = nc;
            cur = nxt;
        }
        for (; rj < nnp; ++rj) {
            const uint4 c0 = h0, c1 = h1;
            if (rj + 1 < nnp)
                load_h2<false>(h0, h1, hbase + (int64_t)token_of(nx_sp, rj + 1) * d, d, lane);
            gates_of(nx_sp, rj, c0, c1, gnext);
        }
        wave_lds_fence();
        buf ^= 1;
        s = ns;
        ns = nns;
        cur_sp = nx_sp;
        nx_sp = nn_sp;
        np = nnp;
    }
}

// ------------------------------------------------------------------------------------------
// Generic path: any 1 <= N <= 64, fp32 or bf16 storage, no LDS-resident router weight.
// One wavefront per token; lanes stride over k (router) and over columns (combine).
// ------------------------------------------------------------------------------------------
template <typename E> __device__ __forceinline__ float ldf(const E *p);
template <> __device__ __forceinline__ float ldf<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ldf<uint16_t>(const uint16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void stf(float *p, float v) { *p = v; }
__device__ __forceinline__ void stf(uint16_t *p, float v) { *p = (uint16_t)f32_to_bf16_bits(v); }

// 16-byte pieces of E: 8 bf16 or 4 fp32 values
template <typename E> struct Piece;
template <> struct Piece<uint16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ void unpack(float (&v)[8], const uint4 &p)
    {
        v[0] = bf16lo(p.x); v[1] = bf16hi(p.x); v[2] = bf16lo(p.y); v[3] = bf16hi(p.y);
        v[4] = bf16lo(p.z); v[5] = bf16hi(p.z); v[6] = bf16lo(p.w); v[7] = bf16hi(p.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&v)[8])
    {
        return make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
    }
};
template <> struct Piece<float> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ void unpack(float (&v)[4], const uint4 &p)
    {
        v[0] = __uint_as_float(p.x); v[1] = __uint_as_float(p.y); v[2] = __uint_as_float(p.z); v[3] = __uint_as_float(p.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&v)[4])
    {
        return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
    }
};

// One wavefront per token.  Router: lanes stride over k and keep the partial logits of 16 experts at a
// time (router rows are read in 16-byte pieces when a row of N values is a whole number of pieces);
// the 64 lanes' partial sums are folded with the butterfly of the streaming kernel and the logits meet
// in LDS for the softmax.  Combine: 16-byte pieces of the table rows, 8 rows in flight per lane, the
// gates broadcast from LDS.
template <typename E>
__global__ __launch_bounds__(256) void fwd_generic_kernel(FwdArgs a)
{
    constexpr int VEC = Piece<E>::VEC;
    constexpr int JB = 16;                  // experts per router pass
    __shared__ float gls[4][64];
    const int d = a.d, N = a.N;
    const int layer = blockIdx.y;
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    float *gl = gls[wave];

    const int32_t *order = nullptr;
    if (a.plan && plan_ok(a))      // a foreign plan: flagged, tokens visited in their own order
        order = a.plan + plan_layout(a.T).order;
    const E *table = static_cast<const E *>(a.table) + (int64_t)layer * a.table_stride;
    const int64_t act_off = (int64_t)layer * a.act_stride;
    const E *hbase = static_cast<const E *>(a.h) + act_off;
    const E *Wr = static_cast<const E *>(a.W_r) + (int64_t)layer * d * N;
    const E *lnw = a.ln_w ? static_cast<const E *>(a.ln_w) + (int64_t)layer * d : nullptr;
    const bool norm = lnw != nullptr;
    const E *sbase = a.shared ? static_cast<const E *>(a.shared) + act_off : nullptr;
    const E *rbase = a.residual ? static_cast<const E *>(a.residual) + act_off : nullptr;
    E *obase = static_cast<E *>(a.out) + act_off;
    const int32_t *rowsrc = a.slot ? a.slot : a.ids;
    const bool row_pieces = (N % VEC) == 0;     // router rows start on 16-byte boundaries

    for (int item = blockIdx.x * 4 + wave; item < a.T; item += gridDim.x * 4) {
        const int t = visit(order, item).t;
        const int64_t row = rowsrc[t];
        const bool valid = row >= 0 && row < a.rows;
        if (!valid && lane == 0 && a.err_flag)
            atomicOr(a.err_flag, 1);
        if (a.rows_dbg && layer == 0 && lane == 0)
            a.rows_dbg[t] = valid ? row : -1;
        const E *rp = table + (valid ? row : 0) * (int64_t)N * d;
        const E *hr = hbase + (int64_t)t * d;

        float rs = 1.f;            // with a norm in front of the router: 1 / rms of this token's state
        if (norm) {
            float ss = 0.f;
            for (int k = lane; k < d; k += 64)
                ss = fmaf(ldf(hr + k), ldf(hr + k), ss);
            ss = span_reduce<32, 1, OpAdd>(ss);
            rs = 1.0f / sqrtf(ss / (float)d + a.ln_eps);
        }
        // logits, 16 experts per pass; lane j of the pass's 16 ends up writing logit jb + j
        for (int jb = 0; jb < N; jb += JB) {
            float z[JB];
#pragma unroll
            for (int j = 0; j < JB; ++j)
                z[j] = 0.f;
            for (int k = lane; k < d; k += 64) {
                // with the norm: x_k * ln_w_k (exact in fp32 for bf16 storage), scaled by 1 / rms after the sum
                const float hk = norm ? ldf(hr + k) * ldf(lnw + k) : ldf(hr + k);
                const E *wk = Wr + (int64_t)k * N + jb;
                if (row_pieces) {
#pragma unroll
                    for (int p = 0; p < JB / VEC; ++p) {
                        if (jb + p * VEC < N) {
                            float w[VEC];
                            Piece<E>::unpack(w, *reinterpret_cast<const uint4 *>(wk + p * VEC));
#pragma unroll
                            for (int e = 0; e < VEC; ++e)
                                z[p * VEC + e] = fmaf(hk, w[e], z[p * VEC + e]);
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < JB; ++j)
                        if (jb + j < N)
                            z[j] = fmaf(hk, ldf(wk + j), z[j]);
                }
            }
            const float zz = Fold<JB, 32>::run(z, lane);      // logit jb + (lane >> 2), in all 4 lanes of the group
            if ((lane & 3) == 0 && jb + (lane >> 2) < N)
                gl[jb + (lane >> 2)] = zz * rs;
        }
        wave_lds_fence();
        const float zmine = lane < N ? gl[lane] : -INFINITY;   // lane j keeps logit j
        const float m = span_reduce<32, 1, OpMax>(zmine);
        const float e = lane < N ? expf(zmine - m) : 0.f;
        const float g = e / span_reduce<32, 1, OpAdd>(e);
        wave_lds_fence();
        if (lane < N) {
            gl[lane] = g;
            if (a.gates_dbg)
                a.gates_dbg[((int64_t)layer * a.T + t) * N + lane] = g;
        }
        wave_lds_fence();

        for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
            float acc[VEC];
#pragma unroll
            for (int e2 = 0; e2 < VEC; ++e2)
                acc[e2] = 0.f;
            if (valid) {
                for (int j0 = 0; j0 < N; j0 += 8) {
                    uint4 piece[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        piece[u] = j0 + u < N ? *reinterpret_cast<const uint4 *>(rp + (int64_t)(j0 + u) * d + c0)
                                              : make_uint4(0, 0, 0, 0);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        if (j0 + u < N) {
                            const float gj = gl[j0 + u];
                            float v[VEC];
                            Piece<E>::unpack(v, piece[u]);
#pragma unroll
                            for (int e2 = 0; e2 < VEC; ++e2)
                                acc[e2] = fmaf(gj, v[e2], acc[e2]);
                        }
                    }
                }
            }
            const int64_t off = (int64_t)t * d + c0;
            float v[VEC];
            if (sbase) {
                Piece<E>::unpack(v, *reinterpret_cast<const uint4 *>(sbase + off));
#pragma unroll
                for (int e2 = 0; e2 < VEC; ++e2)
                    acc[e2] += v[e2];
            }
            if (norm || rbase) {
                Piece<E>::unpack(v, *reinterpret_cast<const uint4 *>((norm ? hr + c0 : rbase + off)));
#pragma unroll
                for (int e2 = 0; e2 < VEC; ++e2)
                    acc[e2] += v[e2];
            }
            *reinterpret_cast<uint4 *>(obase + off) = Piece<E>::pack(acc);
        }
        wave_lds_fence();
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
constexpr size_t LDS_BYTES_PER_CU = 160 * 1024;

// Grid shape.  Every wave should get the same number of items, and all workgroups should be
// resident at once (a second round would stage the router weight again and leave CUs idle at the
// tail).  Residency per CU is bounded by LDS and by registers: the kernels fit 6 to 8 waves per SIMD for
// N <= 4 (asked for: 8; 24 layers x 256 tokens then run one token per wave, 17.5 -> 15.4 us at N = 4,
// 14.5 -> 12.7 us at N = 2), 4 for N <= 32, 2 above.  Returns the number of workgroups per layer.
template <int N, int WPB>
int64_t grid_x(int items, int L, size_t lds, int waves_per_cu = N <= 4 ? 32 : (N <= 32 ? 16 : 8), bool halve_items = false,
               bool oversubscribe = false)
{
    int per_cu = (int)(LDS_BYTES_PER_CU / lds);
    const int wave_cap = waves_per_cu / WPB;
    if (per_cu > wave_cap)
        per_cu = wave_cap;
    per_cu = knob_or(KNOB_FWD_WGS_PER_CU, per_cu);
    if (per_cu < 1)
        per_cu = 1;
    const int64_t resident = (int64_t)num_cus() * per_cu;
    int64_t cap = resident / L;
    if (cap < 1)
        cap = 1;
    // smallest items-per-wave whose grid fits: ceil(items / (WPB * ipw)) <= cap
    int64_t gx = (items + WPB - 1) / WPB;
    if (gx > cap) {
        int64_t ipw = (items + cap * WPB - 1) / (cap * WPB);
        // halve_items (the streaming kernel at N >= 32: eight-wave workgroups, two per CU): from four items per
        // wave on, twice as many workgroups with half the items each even out the tail (T = 16384: 211 ->
        // 202 us with uniform ids, 116 -> 108 us with Zipf ids; one item per wave is worse again)
        if (halve_items && ipw >= 4 && !knob(KNOB_FWD_WGS_PER_CU))
            ipw = (ipw + 1) / 2;
        // 8 and 16 experts, tokens in their own order: the all-resident grid is not always the best one.  More than
        // four items per wave is a static share so long that the launch ends with CUs waiting for the slowest (they
        // do not get equal shares of the memory system), and a grid that fills less than four fifths of the resident
        // places (N = 16, 24 x 256 tokens at two per wave: 768 of 1008) leaves wave slots empty for the whole launch.
        // In both cases: at most four items per wave, and as many as still give a grid of at least 1.4 rounds, the
        // dispatcher handing out what is not resident at once (just over one round is the worst case: a nearly empty
        // second one).  24 layers x 256 tokens: 36.8 -> 35.4 us, x 512: 67.1 -> 63.6 us, x 1024: 132 -> 116 us,
        // x 2048: 248 -> 208 us; N = 8, 24 x 1024: 78.1 -> 75.4 us.  In the order of a plan the all-resident grid
        // stays (measured 1 to 8 % better there up to 24 x 1024 tokens).
        if (oversubscribe && !halve_items && N >= 8 && N <= 16 && !knob(KNOB_FWD_WGS_PER_CU)) {
            auto wgs_at = [&](int64_t c) { return (items + WPB * c - 1) / (WPB * c) * L; };
            if (ipw > 4 || (N == 16 && ipw >= 2 && wgs_at(ipw) * 5 < resident * 4)) {
                int64_t c = ipw > 4 ? 4 : ipw - 1;
                while (c > 1 && wgs_at(c) * 10 < resident * 14)
                    --c;
                ipw = c;
            }
        }
        gx = (items + WPB * ipw - 1) / (WPB * ipw);
    }
    return gx < 1 ? 1 : gx;
}

template <int N, int WPB, bool NTA, bool SPLIT, bool NORM, bool DBG>
mole_status launch_fast_dbg(const FwdArgs &a, hipStream_t stream)
{
    const size_t lds = router_lds_bytes(a.d, N < 4 ? 4 : N) + (NORM ? norm_lds_bytes(a.d) : 0);
    static std::atomic<size_t> lds_seen{0};
    MOLE_HIP_CHECK(ensure_dynamic_lds(
        lds_seen, reinterpret_cast<const void *>(&fwd_bf16_stream_kernel<N, WPB, NTA, SPLIT, NORM, DBG>), lds));
    const int items = SPLIT ? a.T * ((a.d + 511) / 512) : a.T;
    dim3 grid((unsigned)grid_x<N, WPB>(items, a.L, lds, N <= 4 ? 32 : (N <= 32 ? 16 : 8), N >= 32, !SPLIT && !a.plan),
              (unsigned)a.L);
    hipLaunchKernelGGL((fwd_bf16_stream_kernel<N, WPB, NTA, SPLIT, NORM, DBG>), grid, dim3(WPB * 64), lds, stream, a);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

template <int N, int WPB, bool NTA, bool SPLIT, bool NORM>
mole_status launch_fast(const FwdArgs &a, hipStream_t stream)
{
    return a.gates_dbg || a.rows_dbg ? launch_fast_dbg<N, WPB, NTA, SPLIT, NORM, true>(a, stream)
                                     : launch_fast_dbg<N, WPB, NTA, SPLIT, NORM, false>(a, stream);
}

template <int N, int WPB, bool NTA, bool SPLIT>
mole_status launch_fast(const FwdArgs &a, hipStream_t stream)
{
    return a.ln_w ? launch_fast<N, WPB, NTA, SPLIT, true>(a, stream)
                  : launch_fast<N, WPB, NTA, SPLIT, false>(a, stream);
}

template <int N, int WPB, bool NORM, bool RES>
mole_status launch_run(const FwdArgs &a, hipStream_t stream)
{
    constexpr int NR = N < 4 ? 4 : N;
    const size_t lds = router_lds_bytes(a.d, NR) + (NORM ? norm_lds_bytes(a.d) : 0) +
                       (size_t)WPB * 2 * RUN_GROUP * NR * sizeof(float);
    static std::atomic<size_t> lds_seen{0};
    MOLE_HIP_CHECK(ensure_dynamic_lds(lds_seen, reinterpret_cast<const void *>(&fwd_bf16_run_kernel<N, WPB, NORM, RES>),
                                      lds));
    const int spans = (a.T + RUN_GROUP - 1) / RUN_GROUP;
    dim3 grid((unsigned)grid_x<N, WPB>(spans, a.L, lds, 8), (unsigned)a.L);    // two waves per SIMD
    hipLaunchKernelGGL((fwd_bf16_run_kernel<N, WPB, NORM, RES>), grid, dim3(WPB * 64), lds, stream, a);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

template <int N>
mole_status launch_fast_n(const FwdArgs &a, hipStream_t stream, bool long_runs)
{
    // wider workgroups when the router weight is large, so that LDS does not cap occupancy
    const size_t wbytes = (size_t)a.d * N * 2;
    int wpb = wbytes > 40 * 1024 ? 8 : 4;
    wpb = knob_or(KNOB_FWD_WPB, wpb);
    // MOLE_FLAG_RUNS (the caller expects long runs of equal ids in the plan): groups of equal ids share one
    // fetch of their rows and the weighted sum runs on the matrix pipe.  Against the streaming kernel in plan
    // order it wins from about eight tokens per distinct id on (N = 32, T = 16384: 54 against 73 us at 256
    // tokens per id, 73 against 77 us at 8) and loses below (130 against 122 us at 2; Zipf(1.1) ids over a
    // 50 k vocabulary: 105 against 100 us), which is why it is the caller's choice and not the default.
    // MOLE_FWD_RUN = 1 / 2 forces / forbids it (N = 64: rows and gates of one chunk would not fit the
    // register file).
    if constexpr (N <= 32) {
        constexpr size_t gate_lds = (size_t)4 * 2 * RUN_GROUP * 32 * sizeof(float);
        if (a.plan && knob_or(KNOB_FWD_RUN, long_runs ? 1 : 2) == 1 &&
            router_lds_bytes(a.d, N < 4 ? 4 : N) + norm_lds_bytes(a.d) + gate_lds <= LDS_BYTES_PER_CU) {
            if (a.ln_w)
                return launch_run<N, 4, true, true>(a, stream);
            return a.residual ? launch_run<N, 4, false, true>(a, stream) : launch_run<N, 4, false, false>(a, stream);
        }
    }
    // Large batches at N = 32 (at least eight tokens for each of two workgroups per CU): the tile kernel (router of
    // 32 tokens at a time on the matrix pipe, fwd_tile.hip).  d = 1024, against the streaming kernel, same process:
    // 16384 tokens with Zipf ids 112 against 119 us, with a plan 96 against 101 us; with the norm inside 115 against
    // 136 us and 101 against 119 us; 4096 tokens 33 against 35 us; uniform ids: within 2 % either way up to 12288
    // tokens, 222 against 212 us at 16384 (186 against 183 us with a plan), 272 against 280 us at 20000.
    // MOLE_FWD_TILE = 1 / 2 forces / forbids it.
    if constexpr (N == 32) {
        const int want = knob(KNOB_FWD_TILE);
        if (want == 1 || (want != 2 && tile_forward_applies(N, a.d, a.T, a.L))) {
            TileArgs t{a.table, a.slot ? a.slot : a.ids, a.h, a.W_r, a.shared, a.residual, a.out, a.gates_dbg, a.rows_dbg,
                       a.err_flag, a.plan, a.ln_w, a.ln_eps, a.table_stride, a.act_stride, a.rows, a.T, a.d};
            return launch_tile_forward(t, N, a.L, stream);
        }
    }
    // large batches at 32 experts and more: keep the read-once activations out of the caches (uniform ids, 16384
    // tokens: 201.5 against 204.3 us; not with a plan: there a token's activation rows are visited in id order and
    // the plain load measures 2.5 % faster).  Up to 16 experts the plain load is level or better at every size
    // (24 layers x 384 tokens 49.5 against 52.7 us, x 512 62.4 against 65.3, 1 x 16384 62.2 against 63.3).
    const bool nta = knob_or(KNOB_FWD_NTA, N >= 32 && (int64_t)a.T * a.L >= 8192 && !a.plan ? 1 : 2) == 1;
    // small launches: one chunk per item (latency regime); never together with the large-batch loads.  Up to 2048
    // tokens in the launch at 32 experts and more; up to 16 experts whole tokens win earlier (24 layers x 48 tokens:
    // 15.2 against 16.8 us, x 64: 15.8 against 17.4; 16 x 128 at N = 4, d = 2048: 13.6 against 15.2; one layer of 2048
    // tokens 14.8 against 15.9, but of 1536 tokens 13.6 against 12.8): up to 1024 tokens, 1536 for a single layer.
    const int64_t split_max = N >= 32 ? 2048 : (a.L == 1 ? 1536 : 1024);
    const bool split = knob_or(KNOB_FWD_SPLIT, (int64_t)a.T * a.L <= split_max ? 1 : 2) == 1 && a.d > 512;
    // chunk items of many layers in one launch: eight waves share a staged router weight instead of four
    // (24 layers x 32 tokens: 11.7 -> 11.2 us; a single layer is faster with the smaller workgroups)
    if (split && a.L >= 8 && (int64_t)a.T * ((a.d + 511) / 512) >= 64 && !knob(KNOB_FWD_WPB))
        wpb = 8;
    if (split)
        return wpb >= 8 ? launch_fast<N, 8, false, true>(a, stream) : launch_fast<N, 4, false, true>(a, stream);
    if (wpb >= 8)
        return nta ? launch_fast<N, 8, true, false>(a, stream) : launch_fast<N, 8, false, false>(a, stream);
    return nta ? launch_fast<N, 4, true, false>(a, stream) : launch_fast<N, 4, false, false>(a, stream);
}

mole_status forward_impl(const void *table, int64_t table_stride, const int32_t *ids, const int32_t *slot,
                         const void *h, const void *W_r, const void *shared_out, const void *residual,
                         void *out, int64_t act_stride, float *gates_dbg, int64_t *rows_dbg,
                         int32_t *err_flag, int L, int T, int64_t rows, int d, int N, mole_dtype dtype,
                         unsigned flags, const void *workspace, size_t workspace_bytes, void *hip_stream,
                         float ln_eps = 0.f, const void *ln_w = nullptr, bool with_norm = false)
{
    clear_error();
    if (dtype != MOLE_F32 && dtype != MOLE_BF16)
        return fail(MOLE_EINVAL, "mole_lookup_forward: unknown dtype %d", (int)dtype);
    if (T < 0 || L < 1 || rows < 1 || d < 1)
        return fail(MOLE_EINVAL, "mole_lookup_forward: bad size (T=%d, L=%d, rows=%lld, d=%d)", T, L,
                    (long long)rows, d);
    if (N < 1 || N > 64)
        return fail(MOLE_EUNSUPPORTED, "mole_lookup_forward: N=%d outside 1..64", N);
    const int dmul = dtype == MOLE_BF16 ? 8 : 4;
    if (d % dmul)
        return fail(MOLE_EUNSUPPORTED, "mole_lookup_forward: d=%d must be a multiple of %d", d, dmul);
    if (flags & ~unsigned(MOLE_FLAG_DEDUP | MOLE_FLAG_RUNS))
        return fail(MOLE_EINVAL, "mole_lookup_forward: unknown flags 0x%x", flags);
    if ((flags & MOLE_FLAG_RUNS) && !(flags & MOLE_FLAG_DEDUP))
        return fail(MOLE_EINVAL, "mole_lookup_forward: MOLE_FLAG_RUNS needs MOLE_FLAG_DEDUP and its plan");
    const bool long_runs = (flags & MOLE_FLAG_RUNS) != 0;
    if (T == 0)
        return MOLE_OK;
    if (!table || !ids || !h || !W_r || !out)
        return fail(MOLE_EINVAL, "mole_lookup_forward: table, ids, h, W_r and out must not be NULL");
    if (with_norm && !ln_w)
        return fail(MOLE_EINVAL, "mole_layer_forward: ln_w must not be NULL");
    if (with_norm && !(ln_eps >= 0.f))
        return fail(MOLE_EINVAL, "mole_layer_forward: ln_eps = %g must be >= 0", (double)ln_eps);
    if (ln_w && !aligned16(ln_w))
        return fail(MOLE_EINVAL, "mole_layer_forward: ln_w %p is not 16-byte aligned", ln_w);
    if (ln_w && L > 1 && ((int64_t)d * elem_bytes(dtype)) % 16)
        return fail(MOLE_EUNSUPPORTED, "mole_layer_forward: with L > 1 a norm-weight row of d=%d must be a 16-byte multiple", d);
    const void *ptrs[] = {table, h, W_r, shared_out, residual, out};
    for (const void *p : ptrs)
        if (p && !aligned16(p))
            return fail(MOLE_EINVAL, "mole_lookup_forward: tensor pointer %p is not 16-byte aligned", p);
    if (L > 1) {
        if (act_stride < (int64_t)T * d || table_stride < rows * N * (int64_t)d)
            return fail(MOLE_EINVAL, "mole_lookup_forward_layers: layer stride smaller than one layer");
        if ((act_stride * (int64_t)elem_bytes(dtype)) % 16 || (table_stride * (int64_t)elem_bytes(dtype)) % 16)
            return fail(MOLE_EINVAL, "mole_lookup_forward_layers: layer strides must keep 16-byte alignment");
        if (L > 65535)
            return fail(MOLE_EUNSUPPORTED, "mole_lookup_forward_layers: L=%d > 65535", L);
    }
    const int32_t *plan = nullptr;
    if (flags & MOLE_FLAG_DEDUP) {
        const size_t need = (size_t)plan_layout(T).words * 4;
        if (!workspace || workspace_bytes < need)
            return fail(MOLE_EWORKSPACE, "mole_lookup_forward: MOLE_FLAG_DEDUP needs a %zu-byte plan, got %zu",
                        need, workspace ? workspace_bytes : (size_t)0);
        plan = static_cast<const int32_t *>(workspace);
    }

    MOLE_ARCH_CHECK("mole_lookup_forward");
    FwdArgs a;
    a.table = table; a.ids = ids; a.slot = slot; a.h = h; a.W_r = W_r;
    a.shared = shared_out; a.residual = residual; a.out = out;
    a.gates_dbg = gates_dbg; a.rows_dbg = rows_dbg; a.err_flag = err_flag; a.plan = plan;
    a.ln_w = with_norm ? ln_w : nullptr; a.ln_eps = ln_eps;
    a.table_stride = table_stride; a.act_stride = act_stride; a.rows = rows;
    a.T = T; a.d = d; a.N = N; a.L = L;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    const size_t lds_fast = router_lds_bytes(d, N < 4 ? 4 : N) + (with_norm ? norm_lds_bytes(d) : 0);
    const bool fast = dtype == MOLE_BF16 && lds_fast <= LDS_BYTES_PER_CU && knob(KNOB_FWD_GENERIC) != 1;
    if (fast) {
        switch (N) {
        case 2: return launch_fast_n<2>(a, stream, long_runs);
        case 4: return launch_fast_n<4>(a, stream, long_runs);
        case 8: return launch_fast_n<8>(a, stream, long_runs);
        case 16: return launch_fast_n<16>(a, stream, long_runs);
        case 32: return launch_fast_n<32>(a, stream, long_runs);
        case 64: return launch_fast_n<64>(a, stream, long_runs);
        default: break;
        }
    }
    int64_t gx = (T + 3) / 4;
    int64_t cap = (int64_t)num_cus() * 8 / L;
    if (cap < 1)
        cap = 1;
    if (gx > cap)
        gx = cap;
    dim3 grid((unsigned)gx, (unsigned)L);
    if (dtype == MOLE_F32)
        hipLaunchKernelGGL(fwd_generic_kernel<float>, grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(fwd_generic_kernel<uint16_t>, grid, dim3(256), 0, stream, a);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

}  // namespace

extern "C" mole_status mole_lookup_forward(const void *table, const int32_t *ids, const int32_t *slot,
                                           const void *h, const void *W_r, const void *shared_out,
                                           const void *residual, void *out, float *gates_dbg,
                                           int64_t *rows_dbg, int32_t *err_flag, int T, int64_t rows, int d,
                                           int N, mole_dtype dtype, unsigned flags, const void *workspace,
                                           size_t workspace_bytes, void *hip_stream)
{
    return forward_impl(table, 0, ids, slot, h, W_r, shared_out, residual, out, 0, gates_dbg, rows_dbg,
                        err_flag, 1, T, rows, d, N, dtype, flags, workspace, workspace_bytes, hip_stream);
}

extern "C" mole_status mole_lookup_forward_layers(const void *table, int64_t table_stride, const int32_t *ids,
                                                  const int32_t *slot, const void *h, const void *W_r,
                                                  const void *shared_out, const void *residual, void *out,
                                                  int64_t act_stride, float *gates_dbg, int64_t *rows_dbg,
                                                  int32_t *err_flag, int L, int T, int64_t rows, int d, int N,
                                                  mole_dtype dtype, unsigned flags, const void *workspace,
                                                  size_t workspace_bytes, void *hip_stream)
{
    return forward_impl(table, table_stride, ids, slot, h, W_r, shared_out, residual, out, act_stride,
                        gates_dbg, rows_dbg, err_flag, L, T, rows, d, N, dtype, flags, workspace,
                        workspace_bytes, hip_stream);
}

extern "C" mole_status mole_layer_forward(const void *table, int64_t table_stride, const int32_t *ids,
                                          const int32_t *slot, const void *x, const void *ln_w, float ln_eps,
                                          const void *W_r, const void *shared_out, void *out, int64_t act_stride,
                                          float *gates_dbg, int64_t *rows_dbg, int32_t *err_flag, int L, int T,
                                          int64_t rows, int d, int N, mole_dtype dtype, unsigned flags,
                                          const void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return forward_impl(table, table_stride, ids, slot, x, W_r, shared_out, nullptr, out, act_stride, gates_dbg,
                        rows_dbg, err_flag, L, T, rows, d, N, dtype, flags, workspace, workspace_bytes, hip_stream,
                        ln_eps, ln_w, true);
}
