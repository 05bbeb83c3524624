/*
 * libmole -- the inference hot path of Mixture of Lookup Experts (MoLE, arXiv 2503.15798)
 * for AMD MI355X (gfx950).  Plain C ABI: raw pointers and sizes, no framework types.
 *
 * The layer (paper Sec. 3.3, inference-layer equation, with the router of Sec. 3.2):
 *
 *     g      = SoftMax_j( h . r_j ),  j = 1..N            all N experts active, no top-k
 *     h'     = sum_j g_j * LUT[id, j, :] + FFN_shared(h) + residual
 *     LUT[i, j, :] = FFN_j(Embedding(i))                  built once, offline (LUT entry equation)
 *
 * Conventions for every call
 *   - "dev" pointers are device memory (or host memory the GPU can address: pinned + mapped);
 *     "host" pointers are ordinary host memory.  The caller owns every buffer and the stream.
 *   - All calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and return without synchronising.  The library allocates no device memory, keeps
 *     no global state besides a thread-local error string, the handles of mole_lut_file_* and
 *     process-wide caches of device properties and kernel launch attributes (set idempotently,
 *     so calls may come from several host threads, each on its own stream), and never frees
 *     caller memory.
 *   - Tensors are dense, row-major, in the element type named by `mole_dtype`
 *     (MOLE_BF16: bfloat16 storage, fp32 arithmetic, one round-to-nearest-even at the store;
 *      MOLE_F32: fp32 throughout).  Token ids, slots and maps are int32.
 *   - Tensor pointers must be 16-byte aligned; d must be a multiple of 8 (bf16) / 4 (fp32);
 *     1 <= N <= 64.
 *   - Errors that the host can see (null required pointer, bad size, misalignment, workspace
 *     too small, unsupported shape, a current device that is not a gfx950 part) return a status
 *     WITHOUT launching anything and set the message returned by mole_last_error().
 *   - Errors only the device can see cannot be returned synchronously; they set bits of
 *     *err_flag (the caller zeroes err_flag beforehand and reads it after synchronising):
 *       bit 0 (value 1): a token id (or slot) outside [0, rows): that token's routed term is
 *                        taken as zero; the rest of its output is computed as usual;
 *       bit 1 (value 2): MOLE_FLAG_DEDUP was given but `workspace` does not hold a plan that
 *                        mole_dedup_ids wrote for a batch of T tokens: the plan is ignored, the
 *                        tokens are visited in their own order and the output is the same as
 *                        without the flag.  (A plan of another batch of the same T is not
 *                        detected; it only changes the visiting order, never the result.)
 *     T == 0 is MOLE_OK and launches nothing.
 */
#ifndef MOLE_H
#define MOLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOLE_OK = 0,
    MOLE_EINVAL = 1,        /* bad argument (null, negative, misaligned, inconsistent)      */
    MOLE_EUNSUPPORTED = 2,  /* shape or dtype outside what the kernels are built for       */
    MOLE_EWORKSPACE = 3,    /* workspace missing or smaller than mole_*_workspace() says  */
    MOLE_EHIP = 4,          /* a HIP runtime call failed (message holds hipGetErrorString) */
    MOLE_EIO = 5            /* a file could not be created, opened, mapped or read (LUT files)  */
} mole_status;

typedef enum {
    MOLE_F32 = 0,
    MOLE_BF16 = 1,
    MOLE_U8 = 2     /* raw bytes (d counts bytes per expert row): only for moving quantised tables through
                       mole_lut_file_* and mole_offload_fetch / _idmajor; no arithmetic is defined on it */
} mole_dtype;
typedef enum { MOLE_GELU_ERF = 0, MOLE_GELU_TANH = 1 } mole_act;
typedef enum {
    MOLE_LAYOUT_LAYER_MAJOR = 0,   /* [L, V, N, d]: one table per layer                           */
    MOLE_LAYOUT_ID_MAJOR = 1       /* [V, L, N, d]: the rows of all layers of an id are adjacent  */
} mole_layout;

enum {
    MOLE_FLAG_DEDUP = 1u,   /* forward: `workspace` holds a plan written by mole_dedup_ids for
                               these ids; tokens are visited in id order so that a distinct id's
                               rows cross the memory fabric once                               */
    MOLE_FLAG_RUNS = 2u     /* with MOLE_FLAG_DEDUP, bf16, N <= 32: the caller expects long runs of
                               equal ids (about eight tokens per distinct id or more); tokens with
                               equal ids then share one fetch of their rows and are summed together
                               on the matrix pipe.  Ignored for other dtypes and N            */
};

/* Message of the last failing call on this thread ("" if none).  Never NULL. */
const char *mole_last_error(void);

/* ABI version, currently 2 (2: mole_layer_forward / _nf take the norm weight itself; mole_set_tuning;
 * a no-allocation entry point). */
int mole_version(void);

/* Tuning knobs, for experiments and tests; normal use needs none.  `name` is one of
 * "MOLE_FWD_WPB" (waves per workgroup of the forward kernels, 4 or 8), "MOLE_FWD_WGS_PER_CU",
 * "MOLE_FWD_NTA" (1 = non-temporal activation loads, 2 = plain), "MOLE_FWD_SPLIT" (1 = one
 * 512-column chunk per work item, 2 = whole tokens), "MOLE_FWD_RUN" (1 / 2 = force / forbid the
 * kernel of MOLE_FLAG_RUNS for planned calls), "MOLE_FWD_TILE" (1 / 2 = force / forbid the tile kernel, which
 * serves N = 32 only), "MOLE_FWD_GENERIC" (1 = generic forward kernel),
 * "MOLE_DEDUP_GENERIC" (1 = generic dedup kernel, 2 = never the eight-workgroup kernel), "MOLE_BUILD_HIDDEN" (1 = fp16, 2 = bf16 hi/lo
 * hidden activation), "MOLE_BUILD_SMALL_TILE" (1 = the 256 x 128 GEMM), "MOLE_FFN_GATHER_LAST" (1 = in
 * mole_shared_ffn_forward every workgroup gathers its table rows behind its main loop).  value 0 restores the
 * library's own choice.  Each knob starts from the environment variable of the same name, read once
 * when the first knob is looked up.  Process-wide; takes effect for calls issued afterwards.
 * MOLE_EINVAL for an unknown name or a negative value. */
mole_status mole_set_tuning(const char *name, int value);

/* ------------------------------------------------------------------------------------------
 * Re-parameterization (Sec. 3.3, LUT entry equation):
 *     LUT[v, j, :] = GELU(x_v . W1_j + b1_j) . W2_j + b2_j,   x_v = E[v]
 * The expert is a two-matrix, non-gated FFN (the 4dD flop / 2dD parameter counts of Sec. 3.4).
 * With norm_w != NULL, x_v = E[v] / sqrt(mean(E[v]^2) + norm_eps) * norm_w first (the RMSNorm
 * the training listing applies to embedding states).
 *   E [V,d] dev, W1 [N,d,D] dev, b1 [N,D] dev nullable, W2 [N,D,d] dev, b2 [N,d] dev nullable,
 *   norm_w [d] dev nullable, LUT [V,N,d] dev out.  d and D multiples of 16.
 * bf16: both GEMMs run on the matrix cores with fp32 accumulation.  The hidden activation is
 * not rounded to bf16 (that would show in the result): it is carried in fp16, with W2 converted to
 * fp16 (exact), whenever a bound computed on the device (max |x_v|_2 * max |W1 column|_2 +
 * max |b1|, and max |W2|) proves that nothing can leave the fp16 range; otherwise as a bf16
 * high/low pair at 1.5 x the matrix work.  The environment variable MOLE_BUILD_HIDDEN = f16 | split
 * forces either (for experiments).
 * workspace: dev, at least mole_build_lut_workspace() bytes (holds the hidden activations of a
 * slab of vocabulary rows).  Returns MOLE_EWORKSPACE if it is smaller.
 * ---------------------------------------------------------------------------------------- */
size_t mole_build_lut_workspace(int64_t V, int d, int D, int N, mole_dtype dtype);
mole_status mole_build_lut(const void *E, const void *W1, const void *b1,
                           const void *W2, const void *b2,
                           const void *norm_w, float norm_eps,
                           void *LUT,
                           int64_t V, int d, int D, int N, mole_dtype dtype, mole_act act,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Token-id dedup (an optimisation of the lookup of the inference listing; not in the paper):
 *     uniq  = the distinct in-range ids, ascending        [T] dev out, first *n_uniq valid
 *     inv[t] = index of ids[t] in uniq, -1 if out of range [T] dev out
 *     *n_uniq = U                                          [1] dev out
 * and, in `workspace`, a plan for mole_lookup_forward(MOLE_FLAG_DEDUP): the token indices sorted
 * by id, each marked if its id occurs once.  Presence bitmap in LDS; one workgroup, eight (each owning an id
 * range) for batches of more than 4096 tokens.
 * V <= 524288.  err_flag: [1] dev nullable, set to 1 if any id is outside [0, V).
 * workspace: dev, at least mole_dedup_workspace(T, V) bytes.
 * ---------------------------------------------------------------------------------------- */
size_t mole_dedup_workspace(int T, int64_t V);
mole_status mole_dedup_ids(const int32_t *ids, int T, int64_t V,
                           int32_t *uniq, int32_t *inv, int32_t *n_uniq, int32_t *err_flag,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Fused MoLE layer forward (Sec. 3.2 router equation + Sec. 3.3 inference-layer equation):
 *     z[t,j]  = sum_k h[t,k] * W_r[k,j]
 *     g[t,:]  = softmax(z[t,:])
 *     out[t,:] = sum_j g[t,j] * table[row(t), j, :] + shared_out[t,:] + residual[t,:]
 *     row(t)  = slot ? slot[t] : ids[t]
 *   table [rows,N,d] dev: the resident LUT (rows = V) or a staging buffer of fetched rows
 *         (rows = U_cap, slot = inv of mole_dedup_ids); may be pinned host memory
 *   ids [T] dev; slot [T] dev nullable; h [T,d] dev: router input (the post-attention-normed
 *   state); W_r [d,N] dev (transpose of an nn.Linear(d,N) weight); shared_out [T,d] dev
 *   nullable (= 0); residual [T,d] dev nullable (= 0); out [T,d] dev.
 *   gates_dbg [T,N] fp32 dev nullable: the gates; rows_dbg [T] int64 dev nullable: row(t), or -1
 *   if it was outside [0, rows).  err_flag [1] dev nullable.
 *   flags: MOLE_FLAG_DEDUP -> workspace = plan of mole_dedup_ids(ids, T, ...) (and, if slot is
 *   given, slot must be that call's inv).  Without the flag workspace may be NULL.  The flag does not
 *   change what is computed, and the result is bit-identical to the call without it.
 *   MOLE_FLAG_RUNS (only together with MOLE_FLAG_DEDUP) is a hint for batches with many tokens per
 *   distinct id; the weighted sum of tokens with equal ids is then taken together on the matrix
 *   pipe (gates enter as a pair of bf16 values, 16 significant bits), which changes the summation
 *   order: same tolerance, not the same bits.
 * ---------------------------------------------------------------------------------------- */
mole_status mole_lookup_forward(const void *table, const int32_t *ids, const int32_t *slot,
                                const void *h, const void *W_r,
                                const void *shared_out, const void *residual,
                                void *out, float *gates_dbg, int64_t *rows_dbg, int32_t *err_flag,
                                int T, int64_t rows, int d, int N, mole_dtype dtype,
                                unsigned flags,
                                const void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same forward for L layers that share one id batch, in ONE launch: layer l uses
 * table + l*table_stride, h + l*act_stride, W_r + l*d*N, shared_out/residual/out + l*act_stride
 * (strides in ELEMENTS; act_stride >= T*d, table_stride >= rows*N*d).  Layers are independent
 * here (each has its own h), which is what a decode-throughput measurement over a stack of
 * MoLE layers needs; a real decoder calls the single-layer entry once per layer.
 * gates_dbg [L,T,N], rows_dbg [T]. */
mole_status mole_lookup_forward_layers(const void *table, int64_t table_stride,
                                       const int32_t *ids, const int32_t *slot,
                                       const void *h, const void *W_r,
                                       const void *shared_out, const void *residual,
                                       void *out, int64_t act_stride,
                                       float *gates_dbg, int64_t *rows_dbg, int32_t *err_flag,
                                       int L, int T, int64_t rows, int d, int N, mole_dtype dtype,
                                       unsigned flags,
                                       const void *workspace, size_t workspace_bytes,
                                       void *hip_stream);

/* For callers that cannot allocate device memory and so have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same result as
 *     mole_dedup_ids(ids, T, V, ...) followed by mole_lookup_forward(..., MOLE_FLAG_DEDUP, plan)
 * (bit for bit the output of mole_lookup_forward without flags, rows read in id order), with the plan,
 * the distinct ids, the inverse map and their count kept in a fixed array of 393 KiB in device memory
 * that belongs to the library: each GPU the library runs on holds one copy until the process ends.
 * The call allocates nothing, on the device or through any library, and never synchronises.
 *   T <= MOLE_NOALLOC_MAX_T, else MOLE_EUNSUPPORTED (then use the two calls with a workspace of your own);
 *   V <= 524288 (as mole_dedup_ids); no slot indirection and no debug outputs; other arguments and
 *   err_flag as in mole_lookup_forward.
 * All calls on one GPU share that GPU's array, and the array keeps the last call's contents (every word
 * a call reads it has written itself first): calls that overlap in time on one GPU -- from several
 * streams or host threads -- race and must be serialised by the caller. */
#define MOLE_NOALLOC_MAX_T 16384
mole_status mole_lookup_forward_noalloc(const void *table, const int32_t *ids,
                                        const void *h, const void *W_r,
                                        const void *shared_out, const void *residual,
                                        void *out, int32_t *err_flag,
                                        int T, int64_t V, int d, int N, mole_dtype dtype,
                                        void *hip_stream);

/* The MoLE part of a decoder layer from the state AFTER attention, with the post-attention RMSNorm
 * and the residual inside the kernel (inference listing, "Shared Expert" / "Routed Expert"):
 *     hn[t,:]  = x[t,:] / sqrt(mean_k x[t,k]^2 + ln_eps) * ln_w
 *     g[t,:]   = softmax(hn[t,:] . W_r)
 *     out[t,:] = x[t,:] + shared_out[t,:] + sum_j g[t,j] * table[row(t), j, :]
 * The normed state is never materialised: hn . r_j = (1 / rms(x)) * sum_k (x_k ln_w_k) W_r[k,j], and the
 * products x_k ln_w_k enter the router exactly (bf16 storage: as a pair of bf16 values; fp32 storage:
 * one fp32 rounding), so the gates carry fp32 rounding errors only, as in mole_lookup_forward.  x, read
 * once, is both the norm's input and the residual.
 *   x [T,d] dev: the state after the attention residual add; ln_w [d] dev ([L,d] for L layers); ln_eps >= 0;
 *   W_r [d,N] dev ([L,d,N]); shared_out [T,d] dev nullable: FFN_shared(hn), computed by the caller from
 *   the same normed state.  Everything else as in mole_lookup_forward_layers (L = 1: strides ignored).
 * Saves the 2d bytes per token of reading hn next to x. */
mole_status mole_layer_forward(const void *table, int64_t table_stride,
                               const int32_t *ids, const int32_t *slot,
                               const void *x, const void *ln_w, float ln_eps, const void *W_r,
                               const void *shared_out,
                               void *out, int64_t act_stride,
                               float *gates_dbg, int64_t *rows_dbg, int32_t *err_flag,
                               int L, int T, int64_t rows, int d, int N, mole_dtype dtype,
                               unsigned flags,
                               const void *workspace, size_t workspace_bytes, void *hip_stream);

/* Dedup and forward as one call (the lut(input_ids) line of the inference listing, then Sec. 3.2 router equation
 * and Sec. 3.3 inference-layer equation).  The same results as
 *     mole_dedup_ids(ids, T, V, uniq, inv, n_uniq, err_flag, workspace, ...) followed by
 *     mole_lookup_forward_layers(..., MOLE_FLAG_DEDUP, workspace, ...)           (ln_w == NULL) or
 *     mole_layer_forward(..., x = h, ln_w, ln_eps, ..., MOLE_FLAG_DEDUP, workspace, ...)   (ln_w != NULL),
 * bit for bit (uniq, inv, n_uniq, out; the plan may list tokens with equal ids in another order).  For large
 * batches at N = 32 in bf16 (4096 < T <= 16384, L = 1: the prefill shape) the first launch runs the dedup on a
 * few workgroups and, beside it on all others, the router of every token on the matrix pipe (gates depend on a
 * token's own h only, not on the plan); a second launch gathers and combines in the plan's order.  The dedup's
 * time is hidden behind the router's.  Every other shape runs the two calls one after the other.
 *   h [T,d] dev: the router input, or (ln_w != NULL) the state before the RMSNorm, which is then also the
 *   residual (residual must be NULL); ln_w [d] dev nullable ([L,d]); uniq, inv [T], n_uniq [1] dev out as in
 *   mole_dedup_ids; no slot indirection, no debug outputs; strides in elements, ignored for L = 1.
 *   workspace: dev, mole_dedup_forward_workspace(T, V, N, L) bytes, 16-byte aligned.  After the call its first
 *   mole_dedup_workspace(T, V) bytes hold the plan, which serves further mole_lookup_forward(MOLE_FLAG_DEDUP)
 *   calls on the same ids (the other layers of a model); the rest is scratch (the gates). */
size_t mole_dedup_forward_workspace(int T, int64_t V, int N, int L);
mole_status mole_dedup_forward(const void *table, int64_t table_stride, const int32_t *ids,
                               const void *h, const void *ln_w, float ln_eps, const void *W_r,
                               const void *shared_out, const void *residual,
                               void *out, int64_t act_stride,
                               int32_t *uniq, int32_t *inv, int32_t *n_uniq, int32_t *err_flag,
                               int L, int T, int64_t V, int d, int N, mole_dtype dtype,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/* The layer with its shared expert evaluated inside the call (Sec. 3.3, inference-layer equation; the
 * "Shared Expert" and "Routed Expert" lines of the inference listing):
 *     s[t,:]   = GELU(h[t,:] . W1^T + b1) . W2^T + b2          FFN_shared(h): two matrices, as a routed expert
 *     g[t,:]   = softmax(h[t,:] . W_r)
 *     out[t,:] = residual[t,:] + s[t,:] + sum_j g[t,j] * table[row(t), j, :]
 * Both products run on the matrix cores; the gather and the gate-weighted sum run in the epilogue of the
 * second one, so s is never written to memory (mole_lookup_forward takes it as shared_out instead).
 *   h [T,d] dev: the router's and the shared expert's input (the post-attention-normed state);
 *   W1 [D_s,d], W2 [d,D_s] dev: the weights as a linear layer stores them ([out, in]); b1 [D_s], b2 [d] dev
 *   nullable; residual [T,d] dev nullable; table, ids, slot, W_r, gates_dbg, err_flag, rows as in
 *   mole_lookup_forward.  bf16 only; d and D_s multiples of 128; N in {2, 4, 8, 16, 32, 64} with the
 *   router weight fitting in LDS; other shapes return MOLE_EUNSUPPORTED.
 * The hidden activation is carried as in mole_build_lut: in fp16 when a bound computed on the device (max
 * |h_t|_2 * max |W1 row|_2 + max |b1|, and max |W2|) rules out fp16 overflow, else as a bf16 high + low pair;
 * fp32 accumulation, one rounding of out.  The knob MOLE_BUILD_HIDDEN forces either.
 * workspace: dev, mole_shared_ffn_workspace(T, d, D_s, N) bytes (hidden activation, gates, W2 as fp16). */
size_t mole_shared_ffn_workspace(int T, int d, int D_s, int N);
mole_status mole_shared_ffn_forward(const void *table, const int32_t *ids, const int32_t *slot,
                                    const void *h, const void *W_r,
                                    const void *W1, const void *b1, const void *W2, const void *b2,
                                    const void *residual, void *out, float *gates_dbg, int32_t *err_flag,
                                    int T, int64_t rows, int d, int D_s, int N, mole_dtype dtype, mole_act act,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Offloaded-LUT row fetch (Sec. 3.3: the LUT lives off-chip, only looked-up rows are moved;
 * the lookup line of the inference listing):
 *     staging[l, u, :, :] = host_table[l, uniq[u], :, :]     u < *n_uniq, l < L
 *   host_table: pinned, GPU-addressable host memory [L, V, N, d] (layer stride in elements)
 *   uniq [>= *n_uniq] dev, n_uniq [1] dev: from mole_dedup_ids.  staging [L, U_cap, N, d] dev.
 *   Rows u >= U_cap are not copied and set *err_flag.  The copy is done by a kernel reading
 *   host memory with 16-byte loads (no per-row DMA descriptors).
 * ---------------------------------------------------------------------------------------- */
mole_status mole_offload_fetch(const void *host_table, int64_t host_layer_stride,
                               const int32_t *uniq, const int32_t *n_uniq,
                               void *staging, int64_t staging_layer_stride,
                               int32_t *err_flag,
                               int L, int U_cap, int64_t V, int d, int N, mole_dtype dtype,
                               void *hip_stream);

/* The same fetch from a host table laid out [V, L, N, d] (MOLE_LAYOUT_ID_MAJOR).  Token ids are
 * known when a decoding step starts (the lookup is the first line of the inference listing), so
 * the rows of all L layers are requested together; in this layout they are one contiguous block
 * of L*N*d elements per id.  staging stays [L, U_cap, N, d] (what the forward reads).
 * uniq == NULL means uniq[u] = u: the host buffer holds exactly the wanted rows, in order (for
 * instance rows that mole_lut_file_read_rows has just put into pinned memory; then V = row count
 * of that buffer). */
mole_status mole_offload_fetch_idmajor(const void *host_table,
                                       const int32_t *uniq, const int32_t *n_uniq,
                                       void *staging, int64_t staging_layer_stride,
                                       int32_t *err_flag,
                                       int L, int U_cap, int64_t V, int d, int N, mole_dtype dtype,
                                       void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * LUT files: the tables as an artifact on a storage device (Sec. 3.3: the LUT is offloaded after
 * re-parameterization; Sec. 4.1 offloading setting; Sec. 4.2: the tables sit on large storage
 * devices).  The paper defines no format.  This one: a 4096-byte little-endian header
 * ("MOLELUT\0", u32 version = 1, u32 header bytes, u32 dtype, u32 layout, i64 V, i32 L, i32 N,
 * i32 d, u32 0, u64 payload bytes) followed by the raw table in the layout the header names.
 * A quantised table is stored as two files of raw bytes (dtype MOLE_U8, d = bytes per expert row:
 * d_model*bits/8 for the codes, (d_model/block)*scale_bytes for the scales).
 * Host-only calls: no GPU work, no stream.  These are the only calls that keep state: a
 * mole_lut_file owns a file descriptor, a mapping and its reader threads (started on first use,
 * kept for later calls) until mole_lut_file_close.  Calls on one handle are serialised.
 *   mole_lut_file_create: creates (truncates) `path`, sizes it, maps it read-write.
 *   mole_lut_file_open:   opens read-only, validates the header against the file size, fills
 *                         *desc (nullable).
 *   mole_lut_file_payload: the mapped table (host memory, NOT GPU-addressable), NULL for NULL.
 *   mole_lut_file_write_layer: copies one layer's table src_host [V, N, d] into its place in
 *                         either layout, with `threads` host threads.
 *   mole_lut_file_read_rows: dst_host[i, l, :, :] = table(l, ids_host[i]) for i < n, all l:
 *                         dst is [n, L, N, d] whatever the file's layout (one pread per id for an
 *                         id-major file, L for a layer-major one), `threads` reader threads
 *                         (clamped to 1..64).  An id outside [0, V) fails with MOLE_EINVAL before
 *                         anything is read.  dst_host may be pinned memory.
 *   mole_lut_file_close:  syncs a written file, unmaps, closes, frees the handle; NULL is a no-op.
 * ---------------------------------------------------------------------------------------- */
typedef struct mole_lut_file mole_lut_file;
typedef struct {
    int32_t dtype;      /* mole_dtype  */
    int32_t layout;     /* mole_layout */
    int32_t L, N, d;
    int32_t reserved;   /* 0 */
    int64_t V;
} mole_lut_desc;
mole_status mole_lut_file_create(const char *path, const mole_lut_desc *desc, mole_lut_file **file);
mole_status mole_lut_file_open(const char *path, mole_lut_file **file, mole_lut_desc *desc);
void *mole_lut_file_payload(mole_lut_file *file);
mole_status mole_lut_file_write_layer(mole_lut_file *file, int layer, const void *src_host, int threads);
mole_status mole_lut_file_read_rows(mole_lut_file *file, const int32_t *ids_host, int n,
                                    void *dst_host, int threads);
mole_status mole_lut_file_close(mole_lut_file *file);

/* ------------------------------------------------------------------------------------------
 * NormalFloat-quantised tables (Sec. 5.5, Table 8: NF4 / NF3 post-training quantisation of the
 * LUT with token-wise blocks of 768 / 128 elements -> 25.3 % / 19.5 % of the 16-bit size).
 *
 * NF-k levels: 2^k quantiles of N(0,1) normalised to [-1,1] with an exact zero (the data type of
 * the QLoRA paper; the outermost quantile is taken at probability 1 - 1/(2*2^k)).
 * mole_nf_codebook writes the 2^bits levels (ascending) to host memory and returns their count.
 *
 * Storage of a table [rows, N, d]:
 *   codes  [rows, N, d*bits/8] bytes.  NF4: two codes per byte, element 2i in the low nibble.
 *          NF3: every 8 consecutive elements form a 24-bit word (element e in bits 3e..3e+2);
 *          per row the low 16 bits of all words first (d/4 bytes), then their high 8 bits (d/8).
 *   scales [rows, N, d/block], fp32 (scale_bytes = 4) or bf16 (scale_bytes = 2): max |x| of the block
 *          (buffer size from mole_nf_scales_bytes, which rounds up to 16 bytes).
 * Rule: xn = x / scale in fp32 (0 if scale == 0); code = number of level midpoints below xn;
 * value = level[code] * scale.  bits in {3, 4}; d a multiple of 8 (NF4) / 16 (NF3); block a
 * multiple of 8 dividing d.  The paper's settings: (bits 4, block 768, scale_bytes 4) and
 * (bits 3, block 128, scale_bytes 2).
 *
 * mole_quantize_lut: table bf16 [rows,N,d] dev -> codes, scales dev (sizes from the two helpers).
 * mole_lookup_forward_nf: the fused forward of mole_lookup_forward_layers with the rows
 * dequantised on the fly; activations bf16; flags: MOLE_FLAG_DEDUP or 0 (MOLE_FLAG_RUNS is not
 * accepted here); codes_stride in BYTES per layer, scales_stride and
 * act_stride in ELEMENTS per layer (ignored for L == 1).  N in {2, 4, 8, 16, 32, 64}; the router
 * weight, d * max(N, 4) * 2 bytes, has to fit in LDS next to the level table (about 158 KiB),
 * else MOLE_EUNSUPPORTED.
 * Arithmetic: gates in fp32 (as reported through gates_dbg); the levels and, per 512-column chunk,
 * the products gate * scale divided by their largest are rounded to fp16, multiplied exactly and
 * accumulated in fp32 (relative error about 2^-10 per term, independent of the table's magnitude);
 * shared / residual terms are added in fp32 and the result is rounded once to bf16.
 * ---------------------------------------------------------------------------------------- */
int mole_nf_codebook(int bits, float *levels_host);
size_t mole_nf_codes_bytes(int64_t rows, int N, int d, int bits);
size_t mole_nf_scales_bytes(int64_t rows, int N, int d, int block, int scale_bytes);
mole_status mole_quantize_lut(const void *table, void *codes, void *scales,
                              int64_t rows, int N, int d, int bits, int block, int scale_bytes,
                              void *hip_stream);
mole_status mole_lookup_forward_nf(const void *codes, int64_t codes_stride,
                                   const void *scales, int64_t scales_stride,
                                   const int32_t *ids, const int32_t *slot,
                                   const void *h, const void *W_r,
                                   const void *shared_out, const void *residual,
                                   void *out, int64_t act_stride,
                                   float *gates_dbg, int64_t *rows_dbg, int32_t *err_flag,
                                   int L, int T, int64_t rows, int d, int N,
                                   int bits, int block, int scale_bytes, unsigned flags,
                                   const void *workspace, size_t workspace_bytes, void *hip_stream);

/* mole_layer_forward with a quantised table: x is the state after attention, ln_w [L,d] the weight of the
 * RMSNorm the router reads it through; out = x + shared_out + sum_j g_j * row_j with the rows dequantised
 * on the fly.  Other arguments as in mole_lookup_forward_nf. */
mole_status mole_layer_forward_nf(const void *codes, int64_t codes_stride,
                                  const void *scales, int64_t scales_stride,
                                  const int32_t *ids, const int32_t *slot,
                                  const void *x, const void *ln_w, float ln_eps, const void *W_r,
                                  const void *shared_out, void *out, int64_t act_stride,
                                  float *gates_dbg, int64_t *rows_dbg, int32_t *err_flag,
                                  int L, int T, int64_t rows, int d, int N,
                                  int bits, int block, int scale_bytes, unsigned flags,
                                  const void *workspace, size_t workspace_bytes, void *hip_stream);

/* Offloaded mode with a quantised table: the codes [L, V, N, d*bits/8] and scales [L, V, N, d/block]
 * of all layers sit in pinned, GPU-mapped host memory; the rows of the distinct ids (uniq / n_uniq of
 * mole_dedup_ids) are copied to staging_codes [L, U_cap, N, d*bits/8] and staging_scales
 * [L, U_cap, N, d/block] on the device, ready for mole_lookup_forward_nf with slot = inv and
 * rows = U_cap.  Code strides count BYTES per layer, scale strides ELEMENTS per layer, as in
 * mole_lookup_forward_nf (ignored for L == 1).  Row sizes, strides and addresses must be even; the copy
 * runs in units of 16 bytes when all of them allow it.  *n_uniq > U_cap sets *err_flag = 1 and
 * fetches the first U_cap ids, as mole_offload_fetch does. */
mole_status mole_offload_fetch_nf(const void *host_codes, int64_t host_codes_stride,
                                  const void *host_scales, int64_t host_scales_stride,
                                  const int32_t *uniq, const int32_t *n_uniq,
                                  void *staging_codes, int64_t staging_codes_stride,
                                  void *staging_scales, int64_t staging_scales_stride,
                                  int32_t *err_flag, int L, int U_cap, int64_t V, int d, int N,
                                  int bits, int block, int scale_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MOLE_H */
