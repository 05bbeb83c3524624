// mole_offload_fetch: pull the looked-up rows of an off-chip LUT into a device staging buffer.
//
// Paper: Sec. 3.3 (after re-parameterization the LUT is offloaded to a storage tier and only
// the d*N looked-up values per token and layer are loaded -- the LoadParam equation of Sec. 3.4)
// and the lookup line of the inference listing (gather on the storage device, asynchronous
// copy to the accelerator).
//
// Here the gather and the copy are one kernel: wavefronts read the pinned, GPU-mapped host
// table directly with 16-byte loads and write HBM.  Only the distinct ids of the batch are
// fetched (uniq / n_uniq from mole_dedup_ids), all L layers in one launch.  Each row block
// (N*d elements) is cut into pieces of 64 lanes x 16 bytes; pieces are spread over the whole
// grid so that many reads are in flight on the host link at once.
//
// mole_offload_fetch_idmajor reads a host table laid out [V, L, N, d]: token ids are known when a
// decoding step starts (the lookup is the first line of the inference listing), so the rows of every
// layer can be requested at once, and with this layout they are one contiguous block per id.
//
// mole_offload_fetch_nf does the same for NormalFloat-quantised tables (Sec. 5.5: quantising the LUT
// cuts what has to be loaded per token to a quarter or a fifth): the code rows and the scale rows of
// the distinct ids, two launches of the same kernel on byte rows.
#include "mole_internal.h"

namespace {
using namespace mole;

// ID_MAJOR: the host table is [V, L, N, d] (all layers of an id adjacent) and the work is ordered
// so that consecutive wavefronts read consecutive KiB of one id's L*N*d block; otherwise the host
// table is [L, V, N, d].  uniq == nullptr means uniq[u] = u (the host buffer already holds exactly
// the wanted rows, e.g. rows read from a file).
// P: the unit of the copy (16 bytes for bf16 / fp32 tables; quantised tables may need 4 or 2).  Strides
// and row16 count units of P.
template <bool ID_MAJOR, typename P = uint4>
__global__ __launch_bounds__(256) void fetch_kernel(const P *__restrict__ host, int64_t host_ls16,
                                                     int64_t host_rs16, const int32_t *__restrict__ uniq,
                                                     const int32_t *__restrict__ n_uniq_p,
                                                     P *__restrict__ staging, int64_t stage_ls16,
                                                     int32_t *err_flag, int L, int U_cap, int64_t V,
                                                     int row16 /* pieces of P per row block */)
{
    int U = *n_uniq_p;
    if (U > U_cap) {
        if (threadIdx.x == 0 && blockIdx.x == 0 && err_flag)
            *err_flag = 1;
        U = U_cap;
    }
    if (U < 0)
        U = 0;
    // work = (layer, u, 1 KiB piece); a wavefront takes one piece at a time
    const int pieces = (row16 + 63) >> 6;
    const int64_t total = (int64_t)L * U * pieces;
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t w = wave0; w < total; w += nwaves) {
        const int p = (int)(w % pieces);
        const int64_t lu = w / pieces;
        int u, l;
        if (ID_MAJOR) {
            l = (int)(lu % L);
            u = (int)(lu / L);
        } else {
            u = (int)(lu % U);
            l = (int)(lu / U);
        }
        const int64_t id = uniq ? (int64_t)uniq[u] : (int64_t)u;
        const int i16 = p * 64 + lane;
        if (i16 < row16 && id >= 0 && id < V) {
            const P v = host[l * host_ls16 + id * host_rs16 + i16];
            staging[l * stage_ls16 + (int64_t)u * row16 + i16] = v;
        }
    }
}

mole_status fetch_impl(const char *who, bool id_major, const void *host_table, int64_t host_layer_stride,
                       const int32_t *uniq, const int32_t *n_uniq, void *staging, int64_t staging_layer_stride,
                       int32_t *err_flag, int L, int U_cap, int64_t V, int d, int N, mole_dtype dtype,
                       void *hip_stream)
{
    clear_error();
    if (dtype != MOLE_F32 && dtype != MOLE_BF16 && dtype != MOLE_U8)
        return fail(MOLE_EINVAL, "%s: unknown dtype %d", who, (int)dtype);
    if (L < 1 || U_cap < 0 || V < 1 || d < 1 || N < 1)
        return fail(MOLE_EINVAL, "%s: bad size (L=%d, U_cap=%d, V=%lld, d=%d, N=%d)", who, L, U_cap, (long long)V,
                    d, N);
    const int64_t eb = (int64_t)elem_bytes(dtype);
    const int64_t row_bytes = (int64_t)N * d * eb;
    if (row_bytes % 16)
        return fail(MOLE_EUNSUPPORTED, "%s: a row block of %lld bytes is not a multiple of 16", who,
                    (long long)row_bytes);
    if (U_cap == 0)
        return MOLE_OK;
    if (!host_table || !n_uniq || !staging || (!uniq && !id_major))
        return fail(MOLE_EINVAL, "%s: host_table, uniq, n_uniq and staging must not be NULL", who);
    if (!aligned16(host_table) || !aligned16(staging))
        return fail(MOLE_EINVAL, "%s: host_table and staging must be 16-byte aligned", who);
    if (L > 1 && (staging_layer_stride < (int64_t)U_cap * N * d || (staging_layer_stride * eb) % 16))
        return fail(MOLE_EINVAL, "%s: staging layer stride too small or not a 16-byte multiple", who);
    if (!id_major && L > 1 && (host_layer_stride < V * N * (int64_t)d || (host_layer_stride * eb) % 16))
        return fail(MOLE_EINVAL, "%s: host layer stride too small or not a 16-byte multiple", who);
    MOLE_ARCH_CHECK(who);
    const int row16 = (int)(row_bytes / 16);
    const int pieces = (row16 + 63) / 64;
    int64_t waves = (int64_t)L * U_cap * pieces;
    int64_t blocks = (waves + 3) / 4;
    const int64_t cap = (int64_t)num_cus() * 8;
    if (blocks > cap)
        blocks = cap;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (id_major)
        hipLaunchKernelGGL(fetch_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const uint4 *>(host_table), (int64_t)row16, (int64_t)L * row16, uniq,
                           n_uniq, static_cast<uint4 *>(staging), staging_layer_stride * eb / 16, err_flag, L,
                           U_cap, V, row16);
    else
        hipLaunchKernelGGL(fetch_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const uint4 *>(host_table), host_layer_stride * eb / 16, (int64_t)row16,
                           uniq, n_uniq, static_cast<uint4 *>(staging), staging_layer_stride * eb / 16, err_flag,
                           L, U_cap, V, row16);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

// rows of `row_bytes` bytes from a layer-major host array [L][V][row_bytes] (layer stride in bytes) into
// staging [L][U_cap][row_bytes], in the largest unit that divides sizes, strides and addresses
template <typename P>
void launch_rows(const void *host, int64_t host_ls, const int32_t *uniq, const int32_t *n_uniq, void *staging,
                 int64_t stage_ls, int32_t *err_flag, int L, int U_cap, int64_t V, int64_t row_bytes, hipStream_t stream)
{
    const int64_t u = (int64_t)sizeof(P);
    const int rowp = (int)(row_bytes / u);
    const int pieces = (rowp + 63) / 64;
    int64_t blocks = ((int64_t)L * U_cap * pieces + 3) / 4;
    const int64_t cap = (int64_t)num_cus() * 8;
    if (blocks > cap)
        blocks = cap;
    hipLaunchKernelGGL((fetch_kernel<false, P>), dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<const P *>(host), host_ls / u, (int64_t)rowp, uniq, n_uniq, static_cast<P *>(staging),
                       stage_ls / u, err_flag, L, U_cap, V, rowp);
}

// the largest unit (16, 4 or 2 bytes) that divides a byte-row copy's sizes, strides and addresses; an
// error status if the layer strides are too small or something is odd
mole_status rows_unit(const char *who, const char *what, const void *host, int64_t host_ls, const void *staging,
                      int64_t stage_ls, int L, int U_cap, int64_t V, int64_t row_bytes, int *unit)
{
    if (L > 1 && (host_ls < V * row_bytes || stage_ls < (int64_t)U_cap * row_bytes))
        return fail(MOLE_EINVAL, "%s: %s layer stride smaller than one layer", who, what);
    const uintptr_t bits = (uintptr_t)row_bytes | reinterpret_cast<uintptr_t>(host) | reinterpret_cast<uintptr_t>(staging) |
                           (L > 1 ? (uintptr_t)host_ls | (uintptr_t)stage_ls : 0);
    if (bits % 2)
        return fail(MOLE_EUNSUPPORTED, "%s: %s rows of %lld bytes, strides and addresses must be even", who, what,
                    (long long)row_bytes);
    *unit = bits % 16 == 0 ? 16 : (bits % 4 == 0 ? 4 : 2);
    return MOLE_OK;
}

void fetch_rows(int unit, const void *host, int64_t host_ls, const int32_t *uniq, const int32_t *n_uniq, void *staging,
                int64_t stage_ls, int32_t *err_flag, int L, int U_cap, int64_t V, int64_t row_bytes, hipStream_t stream)
{
    if (unit == 16)
        launch_rows<uint4>(host, host_ls, uniq, n_uniq, staging, stage_ls, err_flag, L, U_cap, V, row_bytes, stream);
    else if (unit == 4)
        launch_rows<uint32_t>(host, host_ls, uniq, n_uniq, staging, stage_ls, err_flag, L, U_cap, V, row_bytes, stream);
    else
        launch_rows<uint16_t>(host, host_ls, uniq, n_uniq, staging, stage_ls, err_flag, L, U_cap, V, row_bytes, stream);
}

}  // namespace

extern "C" mole_status mole_offload_fetch_nf(const void *host_codes, int64_t host_codes_stride,
                                             const void *host_scales, int64_t host_scales_stride,
                                             const int32_t *uniq, const int32_t *n_uniq, void *staging_codes,
                                             int64_t staging_codes_stride, void *staging_scales,
                                             int64_t staging_scales_stride, int32_t *err_flag, int L, int U_cap,
                                             int64_t V, int d, int N, int bits, int block, int scale_bytes,
                                             void *hip_stream)
{
    const char *who = "mole_offload_fetch_nf";
    clear_error();
    if (bits != 3 && bits != 4)
        return fail(MOLE_EUNSUPPORTED, "%s: bits=%d, NF3 and NF4 are built", who, bits);
    if (scale_bytes != 2 && scale_bytes != 4)
        return fail(MOLE_EINVAL, "%s: scale_bytes=%d must be 2 (bf16) or 4 (fp32)", who, scale_bytes);
    if (L < 1 || U_cap < 0 || V < 1 || d < 1 || N < 1)
        return fail(MOLE_EINVAL, "%s: bad size (L=%d, U_cap=%d, V=%lld, d=%d, N=%d)", who, L, U_cap, (long long)V,
                    d, N);
    const int dmul = bits == 3 ? 16 : 8;
    if (d % dmul || block < 8 || block % 8 || d % block)
        return fail(MOLE_EUNSUPPORTED, "%s: d=%d must be a multiple of %d and block=%d a multiple of 8 dividing d",
                    who, d, dmul, block);
    if (U_cap == 0)
        return MOLE_OK;
    if (!host_codes || !host_scales || !uniq || !n_uniq || !staging_codes || !staging_scales)
        return fail(MOLE_EINVAL, "%s: tables, uniq, n_uniq and staging buffers must not be NULL", who);
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t code_row = (int64_t)N * d * bits / 8;
    const int64_t scale_row = (int64_t)N * (d / block) * scale_bytes;
    int code_unit = 0, scale_unit = 0;
    mole_status st = rows_unit(who, "codes", host_codes, host_codes_stride, staging_codes, staging_codes_stride, L,
                               U_cap, V, code_row, &code_unit);
    if (st != MOLE_OK)
        return st;
    st = rows_unit(who, "scales", host_scales, host_scales_stride * scale_bytes, staging_scales,
                   staging_scales_stride * scale_bytes, L, U_cap, V, scale_row, &scale_unit);
    if (st != MOLE_OK)
        return st;
    MOLE_ARCH_CHECK(who);
    fetch_rows(code_unit, host_codes, host_codes_stride, uniq, n_uniq, staging_codes, staging_codes_stride, err_flag, L,
               U_cap, V, code_row, stream);
    fetch_rows(scale_unit, host_scales, host_scales_stride * scale_bytes, uniq, n_uniq, staging_scales,
               staging_scales_stride * scale_bytes, err_flag, L, U_cap, V, scale_row, stream);
    MOLE_HIP_CHECK(hipGetLastError());
    return MOLE_OK;
}

extern "C" mole_status mole_offload_fetch(const void *host_table, int64_t host_layer_stride, const int32_t *uniq,
                                          const int32_t *n_uniq, void *staging, int64_t staging_layer_stride,
                                          int32_t *err_flag, int L, int U_cap, int64_t V, int d, int N,
                                          mole_dtype dtype, void *hip_stream)
{
    return fetch_impl("mole_offload_fetch", false, host_table, host_layer_stride, uniq, n_uniq, staging,
                      staging_layer_stride, err_flag, L, U_cap, V, d, N, dtype, hip_stream);
}

extern "C" mole_status mole_offload_fetch_idmajor(const void *host_table, const int32_t *uniq,
                                                  const int32_t *n_uniq, void *staging,
                                                  int64_t staging_layer_stride, int32_t *err_flag, int L,
                                                  int U_cap, int64_t V, int d, int N, mole_dtype dtype,
                                                  void *hip_stream)
{
    return fetch_impl("mole_offload_fetch_idmajor", true, host_table, 0, uniq, n_uniq, staging,
                      staging_layer_stride, err_flag, L, U_cap, V, d, N, dtype, hip_stream);
}
