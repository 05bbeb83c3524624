// Tile kernel of the forward for large batches at N = 32.
//
// Paper: Sec. 3.2 (router equation) and Sec. 3.3 (inference-layer equation), as in lookup_forward.hip.
//
// For a batch of thousands of tokens the router h . W_r is a dense product [T, d] x [d, N], and the streaming
// kernel, which computes it token by token on the vector ALU (one dot-product instruction per two multiply-adds,
// then a fold over the 64 lanes), spends almost half of its instructions there.  Here a workgroup of eight
// waves works on a tile of 32 tokens at a time:
//   1. router on the matrix pipe: v_mfma_f32_32x32x16_bf16 with the router weight as its first operand (row =
//      expert) and the tokens' h as its second (row = token); wave w contracts the w-th eighth of d.  Lane l
//      supplies 8 consecutive k of token l % 32 (one 16-byte load) and the same 8 k of expert l % 32 (eight
//      2-byte loads from the [d, N] weight, which stays in L1 / L2: 64 KB for the whole launch).  Staging the
//      weight through LDS instead (16-byte loads, transposed there) measured 3 % slower: what this step waits
//      for is its h loads, queued behind the row loads of the whole chip.  The eight partial 32 x 32 products
//      meet in LDS;
//   2. wave w sums the partials of ITS four tokens, lane = expert, takes the softmax over the 32 lanes of a
//      half-wave (two tokens per pass), and leaves the gates in LDS;
//   3. gather and gate-weighted sum exactly as in the streaming kernel: one wave per token, 16-byte row pieces
//      through a ring of 8 registers that is refilled as it is consumed (the next token's, or the next tile's
//      first token's, pieces are in flight through steps 1 and 2), gates in scalar registers, shared / residual
//      added and one rounding at the store.
// Items are dealt out as in the streaming kernel (round `it`: wave w of workgroup g takes item (it * G + g) * 8 + w
// of the visiting order); a tile is four rounds of a workgroup.
// With the RMSNorm inside (NORM), the state times the norm weight enters step 1 exactly, as a bf16 hi + lo pair
// (two matrix instructions), and 1 / rms scales the logits in step 2.
#include "tile_router.h"

namespace {
using namespace mole;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int TILE = 32;        // tokens per tile = rows of the matrix instruction's second operand
constexpr int TILE_WPB = 8;     // waves per workgroup
constexpr int TPW = TILE / TILE_WPB;

template <int R, bool NT>
__device__ __forceinline__ void ring_load(uint4 (&r)[R], const uint16_t *base, int d, int col)
{
#pragma unroll
    for (int j = 0; j < R; ++j)
        r[j] = ld16_row<NT>(base + (int64_t)j * d + col);
}

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int N, bool NORM>
__global__ __launch_bounds__(TILE_WPB * 64) __attribute__((amdgpu_waves_per_eu(4)))
void fwd_bf16_tile_kernel(TileArgs a)
{
    constexpr int WPB = TILE_WPB;
    constexpr int R = 8;                // row registers (the ring)
    constexpr int H = N / R;
    constexpr int PROW = ROUTER_PROW;   // padded row of the partial-product array
    __shared__ float part[WPB][N][PROW];    // partial logits [wave = part of d][expert][token of the tile]
    __shared__ float ssq[NORM ? WPB : 1][64];
    __shared__ float gl[TILE][N];           // gates of the tile

    const int d = a.d;
    const int T = a.T;
    const int layer = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col0 = lane * 8;

    const uint16_t *table = static_cast<const uint16_t *>(a.table) + (int64_t)layer * a.table_stride;
    const int64_t act_off = (int64_t)layer * a.act_stride;
    const uint16_t *hbase = static_cast<const uint16_t *>(a.h) + act_off;
    const uint16_t *sbase = a.shared ? static_cast<const uint16_t *>(a.shared) + act_off : nullptr;
    const uint16_t *rbase = NORM ? hbase : (a.residual ? static_cast<const uint16_t *>(a.residual) + act_off : nullptr);
    uint16_t *obase = static_cast<uint16_t *>(a.out) + act_off;
    const uint16_t *Wr = static_cast<const uint16_t *>(a.W_r) + (int64_t)layer * d * N;
    const uint16_t *lnw = NORM ? static_cast<const uint16_t *>(a.ln_w) + (int64_t)layer * d : nullptr;
    const int32_t *order = nullptr;
    if (a.plan && plan_ok(a))
        order = a.plan + plan_layout(T).order;

    const int dlast = d - 8;
    // Items are dealt out as in the streaming kernel: in round `it` workgroup g's wave w takes item
    // (it * G + g) * 8 + w of the visiting order, so that at any time the whole grid works on one window of the
    // order (equal ids meet in L2) and every wave walks through the whole order (waves with cheap, repeated ids
    // and waves with ids seen once do not end up in different workgroups).  A tile is four rounds: column
    // 4w + q of the workgroup's k-th tile is the item of wave w in round 4k + q.
    const int G = gridDim.x, g = blockIdx.x;
    const int round_items = G * WPB;
    auto item_of = [&](int it, int w) { return (it * G + g) * WPB + w; };

    // the wave's first token: its first row pieces go in flight before anything else
    int item = item_of(0, wave);
    Visit cur = item < T ? visit(order, item) : Visit{0, false};
    int64_t row = item < T ? (int64_t)__builtin_amdgcn_readfirstlane(a.rowsrc[cur.t]) : -1;
    bool valid = row >= 0 && row < a.rows;
    uint4 r[R];
    auto first_fill = [&]() {
        if (valid) {
            const uint16_t *rp0 = table + row * (int64_t)N * d;
            if (cur.single)
                ring_load<R, true>(r, rp0, d, min(col0, dlast));
            else
                ring_load<R, false>(r, rp0, d, min(col0, dlast));
        }
    };
    first_fill();

    for (int k = 0; item_of(TPW * k, 0) < T; ++k) {
        // ---- 1. + 2. router of the tile: column c holds the item of wave c / TPW in round TPW * k + c % TPW; the
        //      gates stay in LDS for step 3
        router_tile<N, WPB, NORM>(
            &part[0][0][0], &ssq[0][0], hbase, Wr, lnw, a.ln_eps, d, wave, lane,
            [&](int c) {
                const int pitem = item_of(TPW * k + (c & (TPW - 1)), c / TPW);
                return pitem < T ? (order ? (int)((uint32_t)order[pitem] & ~PLAN_SINGLE) : pitem) : -1;
            },
            [&](int c, int tok, int j, float gj) {
                gl[c][j] = gj;
                if (a.gates_dbg && tok >= 0)
                    a.gates_dbg[((int64_t)layer * T + tok) * N + j] = gj;
            });
        wave_lds_fence();

        // ---- 3. gather and gate-weighted sum, one token at a time
        for (int q = 0; q < TPW; ++q) {
            if (item >= T)
                break;
            const int t = cur.t;
            const int nitem = item + round_items;
            const Visit nxt = nitem < T ? visit(order, nitem) : Visit{0, false};
            const int64_t nrow = nitem < T ? (int64_t)__builtin_amdgcn_readfirstlane(a.rowsrc[nxt.t]) : -1;
            const bool nvalid = nrow >= 0 && nrow < a.rows;
            if (!valid && lane == 0 && a.err_flag)
                atomicOr(a.err_flag, 1);
            if (a.rows_dbg && layer == 0 && lane == 0)
                a.rows_dbg[t] = valid ? row : -1;
            const float g = gl[wave * TPW + q][lane & (N - 1)];
            const uint16_t *rp = table + (valid ? row : 0) * (int64_t)N * d;
            const uint16_t *nrp = table + (nvalid ? nrow : 0) * (int64_t)N * d;
            for (int c0 = 0; c0 < d; c0 += 512) {
                const int cc = c0 + col0;
                const bool on = cc < d;
                const bool last = c0 + 512 >= d;
                const int64_t off = (int64_t)t * d + cc;
                uint4 sv = make_uint4(0, 0, 0, 0), rv = make_uint4(0, 0, 0, 0);
                if (on && sbase)
                    sv = ld16_stream<false>(sbase + off);
                if (on && rbase)
                    rv = ld16_stream<false>(rbase + off);
                float acc[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    acc[e] = 0.f;
#pragma unroll
                for (int hf = 0; hf < H; ++hf) {
                    float gs[R];
#pragma unroll
                    for (int j = 0; j < R; ++j)
                        gs[j] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, g), hf * R + j));
                    if (valid) {
#pragma unroll
                        for (int j = 0; j < R; ++j)
                            fma8(acc, gs[j], r[j]);
                    }
                    const bool more = hf + 1 < H;
                    const uint16_t *fb = more ? rp + (int64_t)(hf + 1) * R * d : (last ? nrp : rp);
                    const int fcol = min(more ? cc : (last ? col0 : cc + 512), dlast);
                    if (more || !last ? valid : nvalid) {
                        if (more || !last ? cur.single : nxt.single)
                            ring_load<R, true>(r, fb, d, fcol);
                        else
                            ring_load<R, false>(r, fb, d, fcol);
                    }
                }
                add8(acc, sv);
                add8(acc, rv);
                if (on)
                    st16_stream(obase + off, pack8_cvt(acc));
            }
            row = nrow;
            valid = nvalid;
            cur = nxt;
            item = nitem;
        }
        __syncthreads();    // the next tile's partial products overwrite what step 2 read
    }
}


// ------------------------------------------------------------------------------------------
// Steps 1 and 2 alone: gates [L, T, N] fp32 of all tokens, tiles of 32 consecutive tokens dealt round-robin to the
// workgroups.  Needs no plan, so it can run before (or beside) the dedup.
// ------------------------------------------------------------------------------------------
template <int N, bool NORM>
__global__ __launch_bounds__(TILE_WPB * 64) __attribute__((amdgpu_waves_per_eu(4)))
void tile_router_kernel(const uint16_t *__restrict__ h, const uint16_t *__restrict__ W_r, const uint16_t *__restrict__ ln_w,
                        float ln_eps, float *__restrict__ gates, int T, int d, int64_t act_stride)
{
    __shared__ float part[TILE_WPB][N][ROUTER_PROW];
    __shared__ float ssq[NORM ? TILE_WPB : 1][64];
    const int layer = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const uint16_t *hbase = h + (int64_t)layer * act_stride;
    const uint16_t *Wr = W_r + (int64_t)layer * d * N;
    const uint16_t *lnw = NORM ? ln_w + (int64_t)layer * d : nullptr;
    float *gl = gates + (int64_t)layer * T * N;
    for (int tok0 = blockIdx.x * ROUTER_TILE; tok0 < T; tok0 += gridDim.x * ROUTER_TILE) {
        router_tile<N, TILE_WPB, NORM>(
            &part[0][0][0], &ssq[0][0], hbase, Wr, lnw, ln_eps, d, wave, lane,
            [&](int c) { return tok0 + c < T ? tok0 + c : -1; },
            [&](int, int tok, int j, float gj) {
                if (tok >= 0)
                    gl[(int64_t)tok * N + j] = gj;
            });
        __syncthreads();    // the next tile's partial products overwrite what step 2 read
    }
}

// ------------------------------------------------------------------------------------------
// Gather kernel: step 3 alone, with the gates given ([L, T, N] fp32, written by the GATES variant above).  One wave
// per token and nothing shared between waves, so the hardware's workgroup dispatcher hands out the tokens: a CU
// that gets a smaller share of the memory system's bandwidth simply takes fewer tokens (the fused kernel's static
// partition waits for the slowest CU).  Tokens are taken in the visiting order.  (Giving each of the 8 XCDs one
// contiguous eighth of the order instead, so that the repeats of a row block meet in one L2, measured 3 % slower
// with Zipf ids; 8 row registers at eight waves per SIMD instead of 16 at five 2 % slower; a wave that takes four
// consecutive positions and fetches the rows of neighbours with equal ids once, one conversion for all of them,
// 20 % slower: a quarter of the waves, each with its fetches in a row.)
// ------------------------------------------------------------------------------------------
template <int N, int R, int WPB, bool NORM>
__global__ __launch_bounds__(WPB * 64) __attribute__((amdgpu_waves_per_eu(R <= 8 ? 8 : 4)))
void fwd_bf16_gather_kernel(TileArgs a, const float *__restrict__ gates)
{
    constexpr int H = N / R;
    const int d = a.d;
    const int T = a.T;
    const int layer = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col0 = lane * 8;

    const int item = blockIdx.x * WPB + wave;
    if (item >= T)
        return;

    const uint16_t *table = static_cast<const uint16_t *>(a.table) + (int64_t)layer * a.table_stride;
    const int64_t act_off = (int64_t)layer * a.act_stride;
    const uint16_t *hbase = static_cast<const uint16_t *>(a.h) + act_off;
    const uint16_t *sbase = a.shared ? static_cast<const uint16_t *>(a.shared) + act_off : nullptr;
    const uint16_t *rbase = NORM ? hbase : (a.residual ? static_cast<const uint16_t *>(a.residual) + act_off : nullptr);
    uint16_t *obase = static_cast<uint16_t *>(a.out) + act_off;
    const int32_t *order = nullptr;
    if (a.plan && plan_ok(a))
        order = a.plan + plan_layout(T).order;

    const int dlast = d - 8;
    const Visit cur = visit(order, item);
    const int t = cur.t;
    const int64_t row = (int64_t)__builtin_amdgcn_readfirstlane(a.rowsrc[t]);
    const bool valid = row >= 0 && row < a.rows;
    const float g = gates[((int64_t)layer * T + t) * N + (lane & (N - 1))];
    const uint16_t *rp = table + (valid ? row : 0) * (int64_t)N * d;
    uint4 r[R];
    if (valid) {
        if (cur.single)
            ring_load<R, true>(r, rp, d, min(col0, dlast));
        else
            ring_load<R, false>(r, rp, d, min(col0, dlast));
    } else if (lane == 0 && a.err_flag) {
        atomicOr(a.err_flag, 1);
    }
    if (a.rows_dbg && layer == 0 && lane == 0)
        a.rows_dbg[t] = valid ? row : -1;

    for (int c0 = 0; c0 < d; c0 += 512) {
        const int cc = c0 + col0;
        const bool on = cc < d;
        const bool last = c0 + 512 >= d;
        const int64_t off = (int64_t)t * d + cc;
        uint4 sv = make_uint4(0, 0, 0, 0), rv = make_uint4(0, 0, 0, 0);
        if (on && sbase)
            sv = ld16_stream<false>(sbase + off);
        if (on && rbase)
            rv = ld16_stream<false>(rbase + off);
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            acc[e] = 0.f;
#pragma unroll
        for (int hf = 0; hf < H; ++hf) {
            float gs[R];
#pragma unroll
            for (int j = 0; j < R; ++j)
                gs[j] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, g), hf * R + j));
            if (valid) {
#pragma unroll
                for (int j = 0; j < R; ++j)
                    fma8(acc, gs[j], r[j]);
            }
            const bool more = hf + 1 < H;
            if (valid && (more || !last)) {
                const uint16_t *fb = more ? rp + (int64_t)(hf + 1) * R * d : rp;
                const int fcol = min(more ? cc : cc + 512, dlast);
                if (cur.single)
                    ring_load<R, true>(r, fb, d, fcol);
                else
                    ring_load<R, false>(r, fb, d, fcol);
            }
        }
        add8(acc, sv);
        add8(acc, rv);
        if (on)
            st16_stream(obase + off, pack8_cvt(acc));
    }
}


}  // namespace

namespace mole {

bool tile_forward_applies(int N, int d, int T, int L)
{
    // every workgroup slot (two per CU) gets at least one round of eight tokens: below that the streaming
    // kernel, with its smaller work items, fills the chip better
    return N == 32 && d % 8 == 0 && (int64_t)((T + TILE_WPB - 1) / TILE_WPB) * L >= 2 * (int64_t)num_cus();
}

mole_status launch_tile_forward(const TileArgs &a, int N, int L, hipStream_t stream)
{
    if (N != 32)
        return fail(MOLE_EUNSUPPORTED, "tile forward: N=%d (only 32)", N);
    // Two workgroups of eight waves per CU (four waves per SIMD), all resident, and every one of them in every
    // round of eight items (a last tile of fewer than four rounds is cheaper than CUs with unequal numbers of
    // workgroups: 12288 tokens as 384 full tiles took 99 us, as 512 workgroups of three rounds 86 us).
    int64_t cap = (int64_t)num_cus() * knob_or(KNOB_FWD_WGS_PER_CU, 2) / L;
    if (cap < 1)
        cap = 1;
    int64_t gx = (a.T + TILE_WPB - 1) / TILE_WPB;      // one round each at least
    if (gx > cap)
        gx = cap;
    const dim3 grid((unsigned)gx, (unsigned)L), block(TILE_WPB * 64);
    if (a.ln_w)
        hipLaunchKernelGGL((fwd_bf16_tile_kernel<32, true>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((fwd_bf16_tile_kernel<32, false>), grid, block, 0, stream, a);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

mole_status launch_tile_router(const void *h, const void *W_r, const void *ln_w, float ln_eps, float *gates, int T,
                               int d, int N, int L, int64_t act_stride, hipStream_t stream)
{
    if (N != 32 || d % 8 || !gates)
        return fail(MOLE_EUNSUPPORTED, "tile router: N=%d, d=%d", N, d);
    int64_t gx = (T + ROUTER_TILE - 1) / ROUTER_TILE;
    int64_t cap = (int64_t)num_cus() * 2 / L;
    if (cap < 1)
        cap = 1;
    if (gx > cap)
        gx = cap;
    const dim3 grid((unsigned)gx, (unsigned)L), block(TILE_WPB * 64);
    const uint16_t *hp = static_cast<const uint16_t *>(h), *wp = static_cast<const uint16_t *>(W_r);
    if (ln_w)
        hipLaunchKernelGGL((tile_router_kernel<32, true>), grid, block, 0, stream, hp, wp, static_cast<const uint16_t *>(ln_w),
                           ln_eps, gates, T, d, act_stride);
    else
        hipLaunchKernelGGL((tile_router_kernel<32, false>), grid, block, 0, stream, hp, wp, nullptr, 0.f, gates, T, d,
                           act_stride);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

mole_status launch_tile_gather(const TileArgs &a, const float *gates, int N, int L, hipStream_t stream)
{
    if (N != 32 || !gates)
        return fail(MOLE_EUNSUPPORTED, "tile gather: N=%d (only 32) and a gates buffer", N);
    constexpr int WPB = 4;
    const dim3 grid((unsigned)((a.T + WPB - 1) / WPB), (unsigned)L);
    if (a.ln_w)
        hipLaunchKernelGGL((fwd_bf16_gather_kernel<32, 16, WPB, true>), grid, dim3(WPB * 64), 0, stream, a, gates);
    else
        hipLaunchKernelGGL((fwd_bf16_gather_kernel<32, 16, WPB, false>), grid, dim3(WPB * 64), 0, stream, a, gates);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

}  // namespace mole
