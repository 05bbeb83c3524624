// NormalFloat-quantised lookup tables: quantiser and fused dequantising forward.
//
// Paper: Sec. 5.5 and Table 8 -- the 16-bit LUTs are post-training quantised to NF4 / NF3 (the
// data types of the QLoRA paper) with token-wise blocks of 768 / 128 elements, which cuts storage
// and per-token traffic to 25.3 % / 19.5 %.  Those ratios imply one 32-bit absmax per 768-element
// NF4 block and one 16-bit absmax per 128-element NF3 block; both widths are supported for both
// types (for a bf16 table the absmax is itself a bf16 value, so the 16-bit scale is exact).
//
// Format of one row (d elements) of expert j of id v:
//   NF4: d/2 bytes, two codes per byte, element 2i in the low nibble;
//   NF3: every 8 consecutive elements form a 24-bit word (element e in bits 3e..3e+2); the low 16
//        bits of all words come first (d/4 bytes), then their high 8 bits (d/8 bytes) -- so that a
//        lane's eight elements are one aligned 16-bit load and one 8-bit load, not a 3-byte access;
//   scales: [rows, N, d/block] fp32 or bf16, in a buffer of their own.
// Quantisation rule (every decision in fp32): s = max|x| over the block; xn = x / s (IEEE
// division, 0 if s == 0); code = number of level midpoints below xn (a tie goes down);
// dequantised value = level[code] * s.
//
// The forward kernel is the bf16 streaming kernel with the row ring replaced by code words: a
// lane's eight columns of one row are 4 bytes (NF4) or 3 bytes (NF3), so ALL rows of a token's
// 512-column chunk sit in N registers and the next chunk / next token is prefetched behind them.
// Levels are looked up two at a time (the same column of two experts) in a table of fp16 pairs in LDS and
// multiplied by the fp16 pair of the experts' weights in one dot-product instruction.
#include "fwd_common.h"
#include "nf_codebook.h"

namespace {
using namespace mole;

struct NfArgs {
    const uint8_t *codes;
    const void *scales;
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
    int64_t codes_stride;    // per layer, bytes
    int64_t scales_stride;   // per layer, elements
    int64_t act_stride;      // per layer, elements
    int64_t rows;
    int T, d, N, L;
    int block;               // elements per scale
    const void *ln_w;        // NORM variant: [L, d] weight of the RMSNorm in front of the router; h is the state
    float ln_eps;            // before that norm and is added as the residual
};

// A scale is fetched as a raw dword (the fp32 value, or the aligned dword holding the bf16 value) and
// decoded only where it is used: any arithmetic right behind a load makes the compiler wait for that
// load before it issues the next one, which serialises the N loads of a chunk (measured: 1.7x on the
// whole kernel).
//
// Every load of a chunk is written as (wave-uniform 64-bit base) + (32-bit unsigned lane offset): that is
// the scalar-base form of a global load, whose address costs no vector instruction.  With 64-bit lane
// addresses each of the 2N loads of a chunk took three to five 64-bit vector adds and shifts.
template <typename W> __device__ __forceinline__ uint32_t ld_uniform(const void *base, uint32_t lane_bytes)
{
    return *reinterpret_cast<const W *>(static_cast<const uint8_t *>(base) + (uint64_t)lane_bytes);
}
__device__ __forceinline__ float decode_scale(uint32_t raw, int scale_bytes, int odd)
{
    if (scale_bytes == 4)
        return __uint_as_float(raw);
    return odd ? bf16hi(raw) : bf16lo(raw);
}

// ------------------------------------------------------------------------------------------
// quantiser: one wavefront per table row (d elements); lane l holds pieces of 8 elements
// ------------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void nf_quantize_kernel(const uint16_t *__restrict__ table,
                                                           uint8_t *__restrict__ codes, void *__restrict__ scales,
                                                           int64_t n_rows, int d, int block, int scale_bytes)
{
    constexpr int NLEV = 1 << BITS;
    const float *mids = BITS == 4 ? NF4_MIDPOINTS : NF3_MIDPOINTS;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= n_rows)
        return;
    const uint16_t *src = table + row * d;
    const int row_bytes = d * BITS / 8;
    uint8_t *dst = codes + row * row_bytes;
    const int nblk = d / block;
    for (int c0 = 0; c0 < d; c0 += 512) {
        const int col = c0 + lane * 8;
        const bool on = col < d;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (on)
            v = *reinterpret_cast<const uint4 *>(src + col);
        float x[8] = {bf16lo(v.x), bf16hi(v.x), bf16lo(v.y), bf16hi(v.y),
                      bf16lo(v.z), bf16hi(v.z), bf16lo(v.w), bf16hi(v.w)};
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            amax = fmaxf(amax, fabsf(x[e]));
        // absmax of each block that touches this chunk.  Blocks are multiples of 8 elements, so a
        // lane's piece lies in one block.  When blocks cannot straddle a chunk boundary (block divides
        // 512) the lanes of equal block index are reduced; otherwise the block is re-scanned whole.
        const int blk = on ? col / block : -1;
        float s = 0.f;
        const int b_lo = c0 / block, b_hi = min(nblk - 1, (min(c0 + 512, d) - 1) / block);
        for (int b = b_lo; b <= b_hi; ++b) {
            float m = 0.f;
            if (512 % block == 0) {
                m = blk == b ? amax : 0.f;
            } else {
                for (int c1 = b * block + lane * 8; c1 < (b + 1) * block; c1 += 512) {
                    const uint4 u = *reinterpret_cast<const uint4 *>(src + c1);
                    m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(bf16lo(u.x)), fabsf(bf16hi(u.x))),
                                             fmaxf(fabsf(bf16lo(u.y)), fabsf(bf16hi(u.y)))),
                                       fmaxf(fmaxf(fabsf(bf16lo(u.z)), fabsf(bf16hi(u.z))),
                                             fmaxf(fabsf(bf16lo(u.w)), fabsf(bf16hi(u.w))))));
                }
            }
#pragma unroll
            for (int w = 32; w >= 1; w >>= 1)
                m = fmaxf(m, __shfl_xor(m, w));
            if (blk == b)
                s = m;
            if (lane == 0 && b * block >= c0 && b * block < c0 + 512) {   // once: by the chunk where the block starts
                const int64_t si = row * nblk + b;
                if (scale_bytes == 4)
                    static_cast<float *>(scales)[si] = m;
                else
                    static_cast<uint16_t *>(scales)[si] = (uint16_t)f32_to_bf16_bits(m);
            }
        }
        if (!on)
            continue;
        uint32_t code[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float xn = s > 0.f ? x[e] / s : 0.f;
            uint32_t c = 0;
#pragma unroll
            for (int i = 0; i < NLEV - 1; ++i)
                c += xn > mids[i] ? 1u : 0u;
            code[e] = c;
        }
        if (BITS == 4) {
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                w |= code[e] << (4 * e);
            *reinterpret_cast<uint32_t *>(dst + col / 2) = w;
        } else {
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                w |= code[e] << (3 * e);
            *reinterpret_cast<uint16_t *>(dst + col / 4) = (uint16_t)(w & 0xffffu);
            dst[d / 4 + col / 8] = (uint8_t)(w >> 16);
        }
    }
}

// ------------------------------------------------------------------------------------------
// fused dequantising forward
// ------------------------------------------------------------------------------------------
// code word of the lane's 8 columns of row j, chunk at column `col`: NF4 one dword (4 bits per
// element); NF3 the 24-bit word (3 bits per element) assembled from its two planes
// (the two NF3 planes are kept as loaded and joined where they are used, see ld_uniform)
template <int BITS>
__device__ __forceinline__ void load_codes(uint32_t &lo, uint32_t &hi, const uint8_t *rowp, uint32_t vo_lo, uint32_t vo_hi)
{
    if (BITS == 4) {
        lo = ld_uniform<uint32_t>(rowp, vo_lo);
        hi = 0;
    } else {
        lo = ld_uniform<uint16_t>(rowp, vo_lo);
        hi = ld_uniform<uint8_t>(rowp, vo_hi);
    }
}

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
constexpr size_t PAIR_TABLE_LDS = 1024;   // static LDS of the forward kernel: 256 pairs for NF4 (64 for NF3)

// acc[e] += ga * level[code e of wa] + gb * level[code e of wb], e = 0..7, for the code words of TWO experts
// and their weights gab = (ga, gb) as an fp16 pair.  The two codes of a column are merged into one index
// (2 * BITS bits), the pair table returns both levels as an fp16 pair, and one v_dot2_f32_f16 multiplies
// and adds both (products exact, fp32 accumulation).  Per element that is 1.4 vector instructions (index,
// half a lookup, half a dot product) against 3 (shift, mask, fma) with one lookup per code.  The pair
// table is a statically allocated LDS array: its address is a compile-time constant, so no base is added
// per lookup.
template <int BITS>
__device__ __forceinline__ void dequant_pair8(float (&acc)[8], half2_t gab, uint32_t wa, uint32_t wb, const uint32_t *pairs)
{
    const unsigned char *base = reinterpret_cast<const unsigned char *>(pairs);
    // x[0]: the merged indices of the even columns, x[1]: of the odd columns
    uint32_t x[2];
    constexpr int F = 2 * BITS;                                   // bits per merged index
    if (BITS == 4) {
        x[0] = (wa & 0x0F0F0F0Fu) | ((wb << 4) & 0xF0F0F0F0u);
        x[1] = ((wa >> 4) & 0x0F0F0F0Fu) | (wb & 0xF0F0F0F0u);
    } else {
        // the merged indices times 4 (the table's byte offsets): 6-bit fields at bits 2, 8, 14, 20
        constexpr uint32_t M0 = 0x1C71C7u;                        // bits 0-2 of every 6-bit field of a 24-bit word
        x[0] = ((wa << 2) & (M0 << 2)) | ((wb << 5) & (M0 << 5));
        x[1] = ((wa >> 1) & (M0 << 2)) | ((wb << 2) & (M0 << 5));
    }
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        uint32_t a[4];
        if (BITS == 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                a[k] = ((x[o] >> (F * k)) & ((1u << F) - 1u)) << 2;
        } else {
            // fields 0 and 2 in one word, 1 and 3 in another: with its neighbours cleared a field leaves as the
            // byte offset through ONE bit-field extract (8 bits from 2 below the field), 1.5 instructions per
            // look-up instead of shift + mask + shift
            const uint32_t ye = x[o] & 0x000FC0FCu, yo = x[o] & 0x03F03F00u;
            // (written as instructions: the compiler turns the builtin with constant arguments back into shift + mask)
            a[0] = ye & 0xFFu;
            asm("v_bfe_u32 %0, %1, 6, 8" : "=v"(a[1]) : "v"(yo));
            asm("v_bfe_u32 %0, %1, 12, 8" : "=v"(a[2]) : "v"(ye));
            asm("v_bfe_u32 %0, %1, 18, 8" : "=v"(a[3]) : "v"(yo));
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t lv = *reinterpret_cast<const uint32_t *>(base + a[k]);
            acc[2 * k + o] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, lv), gab, acc[2 * k + o], false);
        }
    }
}

// DBG: a.gates_dbg / a.rows_dbg are written (a variant of its own: the two pointers stay out of the scalar
// registers of the kernel that serves every other call)
template <int N, int BITS, int WPB, bool NORM, bool DBG>
__global__ __launch_bounds__(WPB * 64) void fwd_nf_kernel(NfArgs a, int scale_bytes)
{
    extern __shared__ uint4 smem[];
    constexpr int NR = N < 4 ? 4 : N;   // experts the router is computed for (N = 2 is padded to 4)
    constexpr int LPJ = 64 / NR;        // lanes per expert after the fold
    constexpr int NLEV = 1 << BITS;
    // The experts of a chunk pass through the code-word registers R at a time (NF4: 16, NF3, which holds two
    // words per expert: 8): with all N in registers the kernel runs at two waves per SIMD or fewer, in parts
    // it fits four.
    constexpr int R = N > 16 ? (BITS == 3 ? 8 : 16) : N;
    constexpr int H = N / R;
    const int d = a.d;
    const int kgroups = d >> 3;
    const int layer = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col0 = lane * 8;
    const int T = a.T;
    const int row_bytes = d * BITS / 8;
    const int nblk = d / a.block;

    const uint8_t *codes = a.codes + (int64_t)layer * a.codes_stride;
    const int64_t sc_off = (int64_t)layer * a.scales_stride;
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

    // pair table (static: see dequant_pair8): entry a | b << BITS holds (level[a], level[b]) as fp16
    __shared__ uint32_t cb2[NLEV * NLEV];
    uint4 *router = smem;
    for (int i = threadIdx.x; i < NLEV * NLEV; i += WPB * 64) {
        const float *lv = BITS == 4 ? NF4_LEVELS : NF3_LEVELS;
        const half2_t pr = {(_Float16)lv[i & (NLEV - 1)], (_Float16)lv[i >> BITS]};
        cb2[i] = __builtin_bit_cast(uint32_t, pr);
    }
    // Order of the first requests, as in the bf16 streaming kernel: the id of the wave's first token is asked for
    // first (the chain id -> code words is the longest), its router input and the router weight follow, the weight
    // goes to LDS when it is there (by then the id has arrived too: memory returns a wave's loads in order), then the
    // code words and scales are requested and the router runs while they travel.
    const int item_first = blockIdx.x * WPB + wave;
    const int t_first = item_first < T ? visit(order, item_first).t : 0;
    const int32_t id_first = item_first < T ? rowsrc[t_first] : -1;
    uint4 h0, h1;
    load_h2<false>(h0, h1, hbase + (int64_t)t_first * d, d, lane);
    fill_router_lds<NR, N>(router, static_cast<const uint16_t *>(a.W_r) + (int64_t)layer * d * N, kgroups, WPB * 64);
    const uint4 *lnw = smem + router_lds_bytes(d, NR) / 16;     // NORM: the norm weight behind the router weight
    if constexpr (NORM)
        fill_norm_lds(smem + router_lds_bytes(d, NR) / 16, static_cast<const uint16_t *>(a.ln_w) + (int64_t)layer * d,
                      kgroups, WPB * 64);

    // col / block by a multiplication: exact for col < d <= 65535 (col * block < 2^32)
    const uint32_t block_magic = (uint32_t)(0x100000000ull / (uint32_t)a.block) + 1u;
    const int sbytes_is4 = scale_bytes == 4;
    int sc_odd = 0;   // parity of the scale index of row 0 of the chunk held in sc[] (bf16 scales; per lane)
    // One block per row (block = d) and all experts in one part: a row's scale serves every chunk of the token, so it
    // is loaded with the token's first chunk only, and the weights gate x scale are formed there only (a tenth of a
    // chunk's vector instructions).  NF4 only: NF3 sits at its register limit without the values kept.
    const bool weights_once = BITS == 4 && H == 1 && nblk == 1;
    auto load_part = [&](uint32_t (&cw)[R], uint32_t (&ch)[R], uint32_t (&sc)[R], int64_t row, int col, int part,
                         bool with_scales) {
        const int64_t e_row = row * (int64_t)N + part * R;                              // first expert row of the part
        const uint8_t *rp = codes + e_row * row_bytes;                                  // uniform
        const int64_t s0 = sc_off + e_row * nblk;                                       // uniform: scale index of its block 0
        const uint32_t q = __umulhi((uint32_t)col, block_magic);                        // the lane's block within the row
        const uint32_t vo_lo = BITS == 4 ? (uint32_t)col >> 1 : (uint32_t)col >> 2;
        const uint32_t vo_hi = (uint32_t)(d >> 2) + ((uint32_t)col >> 3);
        // Expert j's data lie j row_bytes (codes) and j nblk scales further on: those steps go into the lane
        // offset (one 32-bit add per load) so that one base serves all R loads; a base per expert would
        // need 4R scalar registers.  bf16 scales are read as the aligned dword that holds them: with
        // e = p0 + q the lane's element index relative to the even element at or below s0, expert j's scale
        // is in dword (e + j nblk) >> 1, which advances by exactly nblk per two experts.
        const uint32_t p0 = sbytes_is4 ? 0u : (uint32_t)s0 & 1u;
        const uint32_t e0 = p0 + q;
        uint32_t vs[2] = {sbytes_is4 ? e0 << 2 : (e0 >> 1) << 2,
                          sbytes_is4 ? (e0 + (uint32_t)nblk) << 2 : ((e0 + (uint32_t)nblk) >> 1) << 2};
        const uint32_t vs_step = sbytes_is4 ? (uint32_t)nblk << 3 : (uint32_t)nblk << 2;   // bytes per two experts
        sc_odd = (int)(e0 & 1u);
        const uint8_t *sbase = static_cast<const uint8_t *>(a.scales) + (sbytes_is4 ? s0 << 2 : (s0 >> 1) << 2);
        uint32_t vc_lo = vo_lo, vc_hi = vo_hi;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            load_codes<BITS>(cw[j], ch[j], rp, vc_lo, vc_hi);
            vc_lo += (uint32_t)row_bytes;
            // keep these running sums: rewritten as offset + j * step they need a scalar register per product
            asm volatile("" : "+v"(vc_lo));
            if (with_scales) {
                sc[j] = ld_uniform<uint32_t>(sbase, vs[j & 1]);
                vs[j & 1] += vs_step;
                asm volatile("" : "+v"(vs[j & 1]));
            }
            if (BITS == 3) {
                vc_hi += (uint32_t)row_bytes;
                asm volatile("" : "+v"(vc_hi));
            }
        }
    };
    const int dlast = d - 8;
    int item = item_first;
    int t = t_first;
    int64_t row = (int64_t)__builtin_amdgcn_readfirstlane(id_first);
    bool valid = row >= 0 && row < a.rows;
    uint32_t cw[R], ch[R], sc[R];
    if (valid)
        load_part(cw, ch, sc, row, min(col0, dlast), 0, true);
    __syncthreads();    // pair table, router weight and norm weight are in LDS

    for (; item < T; item += stride) {
        const int nitem = item + stride;
        const int nt = nitem < T ? visit(order, nitem).t : 0;
        const int64_t nrow = nitem < T ? (int64_t)__builtin_amdgcn_readfirstlane(rowsrc[nt]) : -1;
        const bool nvalid = nrow >= 0 && nrow < a.rows;
        if (!valid && lane == 0 && a.err_flag)
            atomicOr(a.err_flag, 1);
        if (DBG && a.rows_dbg && layer == 0 && lane == 0)
            a.rows_dbg[t] = valid ? row : -1;

        const float g = router_gate<NR, false, NORM, N>(router, kgroups, hbase + (int64_t)t * d, d, lane, h0, h1, a.ln_eps, lnw);
        if (DBG && a.gates_dbg && (lane & (LPJ - 1)) == 0 && lane / LPJ < N)
            a.gates_dbg[((int64_t)layer * T + t) * N + lane / LPJ] = g;
        load_h2<false>(h0, h1, hbase + (int64_t)nt * d, d, lane);
        // gates into scalar registers: expert j's gate sits in lane j * LPJ.  NF4 takes them anew for every part of
        // every chunk: kept across the chunks they are spilled to vector-register lanes and fetched back, which
        // costs more than the readlanes (NF3, with fewer scalars live, keeps them)
        constexpr bool GS_ONCE = H == 1 && BITS == 3;
        float gs[R];
        if constexpr (GS_ONCE) {
#pragma unroll
            for (int j = 0; j < N; ++j)
                gs[j] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, g), j * LPJ));
        }

        half2_t gp[R / 2];      // weights_once: kept from the token's first chunk
        float m = 1.f;
        for (int c0 = 0; c0 < d; c0 += 512) {
            const int cc = c0 + col0;
            const bool on = cc < d;
            const bool last = c0 + 512 >= d;
            const int64_t off = (int64_t)t * d + cc;
            uint4 sv = make_uint4(0, 0, 0, 0), rv = make_uint4(0, 0, 0, 0);
            if (on && sbase)
                sv = ld16_stream<true>(sbase + off);
            if (on && (NORM || rbase))          // NORM: the state itself, read a second time (an L2 hit)
                rv = ld16_stream<true>((NORM ? hbase : rbase) + off);
            float acc[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                acc[e] = 0.f;
#pragma unroll
            for (int part = 0; part < H; ++part) {
                // the products gate x scale as fp16 pairs, then the registers are free for the next part's
                // words.  They are divided by their largest (m, restored at the end) so that any table scale
                // fits fp16: the largest weight is 1, and one below 6e-5 of it keeps an absolute error of 3e-8.
                uint32_t w[R];
#pragma unroll
                for (int j = 0; j < R; ++j)
                    w[j] = BITS == 4 ? cw[j] : (cw[j] | (ch[j] << 16));
                if (!weights_once || c0 == 0) {
                    if constexpr (!GS_ONCE) {
#pragma unroll
                        for (int j = 0; j < R; ++j)
                            gs[j] = __builtin_bit_cast(
                                float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, g), (part * R + j) * LPJ));
                    }
                    float gsc[R];
                    m = 1.17549435e-38f;
#pragma unroll
                    for (int j = 0; j < R; ++j) {
                        gsc[j] = gs[j] * decode_scale(sc[j], scale_bytes, (j & 1) ? sc_odd ^ (nblk & 1) : sc_odd);
                        m = fmaxf(m, fabsf(gsc[j]));
                    }
                    const float rm = __builtin_amdgcn_rcpf(m);
#pragma unroll
                    for (int j = 0; j < R; j += 2) {
                        // product rounded to fp32, then to fp16, in every variant of the kernel: left to itself the
                        // compiler fuses some of these into one mixed-precision instruction with a single rounding,
                        // and not the same ones in every variant
                        float p0 = gsc[j] * rm, p1 = gsc[j + 1] * rm;
                        asm volatile("" : "+v"(p0), "+v"(p1));
                        gp[j / 2] = half2_t{(_Float16)p0, (_Float16)p1};
                    }
                }
                // refill: the next part of this chunk, else the next chunk / the wave's next token
                const bool more = part + 1 < H;
                if (more || !last ? valid : nvalid)
                    load_part(cw, ch, sc, more || !last ? row : nrow,
                              min(more ? cc : (last ? col0 : cc + 512), dlast), more ? part + 1 : 0,
                              !weights_once || last);
                if (valid) {
                    float pa[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        pa[e] = 0.f;
#pragma unroll
                    for (int j = 0; j < R; j += 2)
                        dequant_pair8<BITS>(pa, gp[j / 2], w[j], w[j + 1], cb2);
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        acc[e] = fmaf(pa[e], m, acc[e]);
                }
            }
            if (sbase)                  // wave-uniform: a missing term costs no unpacking and adding of zeros
                add8(acc, sv);
            if (NORM || rbase)
                add8(acc, rv);
            if (on)
                st16_stream(obase + off, pack8_cvt(acc));
        }
        row = nrow;
        valid = nvalid;
        t = nt;
    }
}

mole_status nf_params_status(int d, int bits, int block, int scale_bytes, const char *who)
{
    if (bits != 3 && bits != 4)
        return fail(MOLE_EUNSUPPORTED, "%s: bits=%d, NF3 and NF4 are built", who, bits);
    if (scale_bytes != 2 && scale_bytes != 4)
        return fail(MOLE_EINVAL, "%s: scale_bytes=%d must be 2 (bf16) or 4 (fp32)", who, scale_bytes);
    const int dmul = bits == 3 ? 16 : 8;
    if (d < dmul || d % dmul || block < 8 || block % 8 || d % block)
        return fail(MOLE_EUNSUPPORTED, "%s: d=%d must be a multiple of %d and block=%d a multiple of 8 dividing d",
                    who, d, dmul, block);
    return MOLE_OK;
}

template <int N, int BITS, bool NORM, bool DBG>
mole_status launch_nf_dbg(const NfArgs &a, int scale_bytes, hipStream_t stream)
{
    // N >= 32: the router weight (64 KiB at N = 32, d = 1024) leaves room for two workgroups per CU, so the
    // waves that the registers allow (three or four per SIMD) have to come from larger workgroups
    constexpr int WPB = N >= 32 ? 8 : 4;
    const size_t lds = router_lds_bytes(a.d, N < 4 ? 4 : N) + (NORM ? norm_lds_bytes(a.d) : 0) + 64;
    static std::atomic<size_t> lds_seen{0};
    MOLE_HIP_CHECK(ensure_dynamic_lds(lds_seen, reinterpret_cast<const void *>(&fwd_nf_kernel<N, BITS, WPB, NORM, DBG>), lds));
    int per_cu = (int)((160 * 1024) / (lds + PAIR_TABLE_LDS));
    constexpr int WG_CAP = N <= 4 ? 8 : 4;       // waves per SIMD the registers allow (four-wave workgroups)
    if (per_cu > WG_CAP)
        per_cu = WG_CAP;
    if (per_cu < 1)
        per_cu = 1;
    int64_t cap = (int64_t)num_cus() * per_cu / a.L;
    if (cap < 1)
        cap = 1;
    int64_t gx = (a.T + WPB - 1) / WPB;
    if (gx > cap) {
        int64_t ipw = (a.T + cap * WPB - 1) / (cap * WPB);
        // NF4 at N >= 32: from four tokens per wave on, twice the workgroups with half the tokens each even out
        // the tail (T = 16384: 101 -> 92 us); NF3 gains nothing from it
        if (N >= 32 && BITS == 4 && ipw >= 4)
            ipw = (ipw + 1) / 2;
        // 16 experts, tokens in their own order: more than four tokens per wave is a static share so long that the
        // launch ends with CUs waiting for the slowest; four per wave (fewer if that grid would be just over one
        // round of the resident places) and the dispatcher handing out the rest (24 layers x 1024 tokens: NF4
        // 91.6 -> 77.0 us, NF3 97.4 -> 82.2 us).  Unlike the bf16 forward (lookup_forward.hip, grid_x) a grid that
        // leaves resident places empty is NOT made finer here: every workgroup builds the pair table and stages the
        // router weight, and this kernel is bound by instruction issue (24 x 256 at one token per wave: 24.5 -> 27.3 us).
        if (N == 16 && ipw > 4 && !a.plan && !knob(KNOB_FWD_WGS_PER_CU)) {
            const int64_t resident = (int64_t)num_cus() * per_cu;
            int64_t c = 4;
            while (c > 1 && (a.T + WPB * c - 1) / (WPB * c) * a.L * 10 < resident * 14)
                --c;
            ipw = c;
        }
        gx = (a.T + WPB * ipw - 1) / (WPB * ipw);
    }
    hipLaunchKernelGGL((fwd_nf_kernel<N, BITS, WPB, NORM, DBG>), dim3((unsigned)gx, (unsigned)a.L), dim3(WPB * 64), lds, stream,
                       a, scale_bytes);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

template <int N, int BITS, bool NORM>
mole_status launch_nf(const NfArgs &a, int scale_bytes, hipStream_t stream)
{
    return a.gates_dbg || a.rows_dbg ? launch_nf_dbg<N, BITS, NORM, true>(a, scale_bytes, stream)
                                     : launch_nf_dbg<N, BITS, NORM, false>(a, scale_bytes, stream);
}

template <int BITS, bool NORM>
mole_status launch_nf_n(const NfArgs &a, int scale_bytes, hipStream_t stream)
{
    switch (a.N) {
    case 2: return launch_nf<2, BITS, NORM>(a, scale_bytes, stream);
    case 4: return launch_nf<4, BITS, NORM>(a, scale_bytes, stream);
    case 8: return launch_nf<8, BITS, NORM>(a, scale_bytes, stream);
    case 16: return launch_nf<16, BITS, NORM>(a, scale_bytes, stream);
    case 32: return launch_nf<32, BITS, NORM>(a, scale_bytes, stream);
    case 64: return launch_nf<64, BITS, NORM>(a, scale_bytes, stream);
    default: return fail(MOLE_EUNSUPPORTED, "mole_lookup_forward_nf: N=%d, built for 2, 4, 8, 16, 32, 64", a.N);
    }
}

// shared by mole_lookup_forward_nf and mole_layer_forward_nf (ln_w given: h is the state x before the norm)
mole_status nf_forward_impl(const char *who, const void *codes, int64_t codes_stride, const void *scales,
                            int64_t scales_stride, const int32_t *ids, const int32_t *slot, const void *h,
                            const void *W_r, const void *shared_out, const void *residual, void *out,
                            int64_t act_stride, float *gates_dbg, int64_t *rows_dbg, int32_t *err_flag, int L, int T,
                            int64_t rows, int d, int N, int bits, int block, int scale_bytes, unsigned flags,
                            const void *workspace, size_t workspace_bytes, void *hip_stream, const void *ln_w,
                            float ln_eps)
{
    clear_error();
    const mole_status ps = nf_params_status(d, bits, block, scale_bytes, who);
    if (ps != MOLE_OK)
        return ps;
    if (T < 0 || L < 1 || L > 65535 || rows < 1)
        return fail(MOLE_EINVAL, "%s: bad size (T=%d, L=%d, rows=%lld)", who, T, L, (long long)rows);
    if (N != 2 && N != 4 && N != 8 && N != 16 && N != 32 && N != 64)
        return fail(MOLE_EUNSUPPORTED, "%s: N=%d, built for 2, 4, 8, 16, 32, 64", who, N);
    if (flags & ~unsigned(MOLE_FLAG_DEDUP))
        return fail(MOLE_EINVAL, "%s: unknown flags 0x%x", who, flags);
    const bool with_norm = ln_w != nullptr;
    if (with_norm && !(ln_eps >= 0.f))
        return fail(MOLE_EINVAL, "%s: ln_eps = %g must be >= 0", who, (double)ln_eps);
    if (with_norm && !aligned16(ln_w))
        return fail(MOLE_EINVAL, "%s: ln_w %p is not 16-byte aligned", who, ln_w);
    if (router_lds_bytes(d, N < 4 ? 4 : N) + (with_norm ? norm_lds_bytes(d) : 0) + 64 + PAIR_TABLE_LDS > 160 * 1024)
        return fail(MOLE_EUNSUPPORTED, "%s: router weight of %d x %d does not fit in LDS", who, d, N);
    if (T == 0)
        return MOLE_OK;
    if (!codes || !scales || !ids || !h || !W_r || !out)
        return fail(MOLE_EINVAL, "%s: codes, scales, ids, the state, the router weight and out must not be NULL", who);
    const void *ptrs[] = {codes, scales, h, W_r, shared_out, residual, out};
    for (const void *p : ptrs)
        if (p && !aligned16(p))
            return fail(MOLE_EINVAL, "%s: tensor pointer %p is not 16-byte aligned", who, p);
    if (L > 1) {
        const int64_t cb = (int64_t)mole_nf_codes_bytes(rows, N, d, bits);
        const int64_t se = rows * N * (int64_t)(d / block);
        if (codes_stride < cb || scales_stride < se || act_stride < (int64_t)T * d || codes_stride % 16 ||
            (scales_stride * scale_bytes) % 16 || (act_stride * 2) % 16)
            return fail(MOLE_EINVAL, "%s: layer strides too small or not 16-byte multiples", who);
    }
    const int32_t *plan = nullptr;
    if (flags & MOLE_FLAG_DEDUP) {
        const size_t need = (size_t)plan_layout(T).words * 4;
        if (!workspace || workspace_bytes < need)
            return fail(MOLE_EWORKSPACE, "%s: MOLE_FLAG_DEDUP needs a %zu-byte plan, got %zu", who, need,
                        workspace ? workspace_bytes : (size_t)0);
        plan = static_cast<const int32_t *>(workspace);
    }
    MOLE_ARCH_CHECK(who);
    NfArgs a;
    a.codes = static_cast<const uint8_t *>(codes); a.scales = scales; a.ids = ids; a.slot = slot; a.h = h; a.W_r = W_r;
    a.shared = shared_out; a.residual = residual; a.out = out; a.gates_dbg = gates_dbg; a.rows_dbg = rows_dbg;
    a.err_flag = err_flag; a.plan = plan; a.codes_stride = codes_stride; a.scales_stride = scales_stride;
    a.act_stride = act_stride; a.rows = rows; a.T = T; a.d = d; a.N = N; a.L = L; a.block = block; a.ln_w = ln_w; a.ln_eps = ln_eps;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (with_norm)
        return bits == 4 ? launch_nf_n<4, true>(a, scale_bytes, stream) : launch_nf_n<3, true>(a, scale_bytes, stream);
    return bits == 4 ? launch_nf_n<4, false>(a, scale_bytes, stream) : launch_nf_n<3, false>(a, scale_bytes, stream);
}

}  // namespace

extern "C" int mole_nf_codebook(int bits, float *levels_host)
{
    if (!levels_host || (bits != 3 && bits != 4))
        return 0;
    const float *src = bits == 4 ? NF4_LEVELS : NF3_LEVELS;
    for (int i = 0; i < (1 << bits); ++i)
        levels_host[i] = src[i];
    return 1 << bits;
}

extern "C" size_t mole_nf_codes_bytes(int64_t rows, int N, int d, int bits)
{
    if (rows < 0 || N < 1 || d < 8 || d % 8 || (bits != 3 && bits != 4))
        return 0;
    return (size_t)rows * N * (size_t)(d * bits / 8);
}

extern "C" size_t mole_nf_scales_bytes(int64_t rows, int N, int d, int block, int scale_bytes)
{
    if (rows < 0 || N < 1 || d < 8 || block < 8 || d % block || (scale_bytes != 2 && scale_bytes != 4))
        return 0;
    // rounded up to 16 bytes: bf16 scales are read as aligned dwords
    return ((size_t)rows * N * (size_t)(d / block) * scale_bytes + 15) & ~(size_t)15;
}

extern "C" mole_status mole_quantize_lut(const void *table, void *codes, void *scales, int64_t rows, int N, int d,
                                         int bits, int block, int scale_bytes, void *hip_stream)
{
    clear_error();
    const mole_status ps = nf_params_status(d, bits, block, scale_bytes, "mole_quantize_lut");
    if (ps != MOLE_OK)
        return ps;
    if (rows < 0 || N < 1 || N > 64)
        return fail(MOLE_EINVAL, "mole_quantize_lut: bad size (rows=%lld, N=%d)", (long long)rows, N);
    if (rows == 0)
        return MOLE_OK;
    if (!table || !codes || !scales)
        return fail(MOLE_EINVAL, "mole_quantize_lut: table, codes and scales must not be NULL");
    if (!aligned16(table) || !aligned16(codes) || !aligned16(scales))
        return fail(MOLE_EINVAL, "mole_quantize_lut: buffers must be 16-byte aligned");
    MOLE_ARCH_CHECK("mole_quantize_lut");
    const int64_t n_rows = rows * N;
    const unsigned blocks = (unsigned)((n_rows + 3) / 4);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (bits == 4)
        hipLaunchKernelGGL(nf_quantize_kernel<4>, dim3(blocks), dim3(256), 0, st, static_cast<const uint16_t *>(table),
                           static_cast<uint8_t *>(codes), scales, n_rows, d, block, scale_bytes);
    else
        hipLaunchKernelGGL(nf_quantize_kernel<3>, dim3(blocks), dim3(256), 0, st, static_cast<const uint16_t *>(table),
                           static_cast<uint8_t *>(codes), scales, n_rows, d, block, scale_bytes);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

extern "C" mole_status mole_lookup_forward_nf(const void *codes, int64_t codes_stride, const void *scales,
                                              int64_t scales_stride, const int32_t *ids, const int32_t *slot,
                                              const void *h, const void *W_r, const void *shared_out,
                                              const void *residual, void *out, int64_t act_stride, float *gates_dbg,
                                              int64_t *rows_dbg, int32_t *err_flag, int L, int T, int64_t rows, int d,
                                              int N, int bits, int block, int scale_bytes, unsigned flags,
                                              const void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return nf_forward_impl("mole_lookup_forward_nf", codes, codes_stride, scales, scales_stride, ids, slot, h, W_r,
                           shared_out, residual, out, act_stride, gates_dbg, rows_dbg, err_flag, L, T, rows, d, N, bits,
                           block, scale_bytes, flags, workspace, workspace_bytes, hip_stream, nullptr, 0.f);
}

extern "C" mole_status mole_layer_forward_nf(const void *codes, int64_t codes_stride, const void *scales,
                                             int64_t scales_stride, const int32_t *ids, const int32_t *slot,
                                             const void *x, const void *ln_w, float ln_eps, const void *W_r,
                                             const void *shared_out,
                                             void *out, int64_t act_stride, float *gates_dbg, int64_t *rows_dbg,
                                             int32_t *err_flag, int L, int T, int64_t rows, int d, int N, int bits,
                                             int block, int scale_bytes, unsigned flags, const void *workspace,
                                             size_t workspace_bytes, void *hip_stream)
{
    if (!ln_w) {
        clear_error();
        return fail(MOLE_EINVAL, "mole_layer_forward_nf: ln_w must not be NULL");
    }
    return nf_forward_impl("mole_layer_forward_nf", codes, codes_stride, scales, scales_stride, ids, slot, x, W_r,
                           shared_out, nullptr, out, act_stride, gates_dbg, rows_dbg, err_flag, L, T, rows, d, N, bits,
                           block, scale_bytes, flags, workspace, workspace_bytes, hip_stream, ln_w, ln_eps);
}
