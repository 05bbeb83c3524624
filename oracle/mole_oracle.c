/*
 * mole_oracle.c -- plain fp64 CPU definition of the Mixture-of-Lookup-Experts layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP library is
 * checked against; it is not part of the product.  Only the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg may call it.  It shares no
 * code, header, table or helper with the HIP path.
 *
 * Everything is written as the paper states it, in double precision, with
 * straight loops and no blocking, fusion or reordering:
 *   - router:   g = SoftMax({h . r_j}, j = 1..N), all N experts active, no top-k
 *               (Sec. 3.2, router equation)
 *   - table:    v^i_j = FFN_j(Embedding(i))                     (Sec. 3.3, LUT entry equation)
 *   - layer:    h' = sum_j g_j v^i_j + FFN_shared(h) + h        (Sec. 3.3, inference-layer equation)
 *   - training-form layer used for brute force lives in the tests, not here.
 * The only parallelism is an OpenMP "for" over independent units (tokens,
 * vocabulary rows); the arithmetic of one unit is untouched by it.
 *
 * Storage formats: every tensor argument comes with a dtype code
 *   0 = IEEE fp32, 1 = bfloat16 (uint16 bit pattern), 2 = IEEE fp64
 * and is widened exactly to double before use, so input rounding is never part
 * of an error budget.
 *
 * Readings where the paper is silent (each is listed in the design notes):
 *   - expert FFN = two matrices, not gated (the 4dD flop / 2dD parameter counts of the
 *     complexity section), activation GELU (erf form; tanh form selectable), optional biases;
 *   - optional RMSNorm of the embedding row before the experts (training listing);
 *   - softmax is evaluated max-subtracted (identical value);
 *   - an id outside [0,V) contributes a zero routed term and raises the error flag;
 *   - dedup map is the canonical one: distinct ids ascending, inv = position in that list.
 *
 *   - the shared expert FFN_shared is read the same way as a routed expert (its 4dD_s flop count in the
 *     complexity table): two matrices, GELU in between, optional biases; its weights are taken in the
 *     layout a linear layer stores them ([out, in]);
 *
 * Pins (tests/test_oracle_pins.py): brute force against running every expert FFN on the
 * embedding; gates sum to one; zero router -> mean of rows; N=1 -> plain row gather;
 * saturated router -> one expert's row exactly; linearity; numpy.unique; math.erf.
 * The paper prints no numeric example of an output, so every pin is a closed form, an invariant,
 * a special case that reduces to a library routine, or brute force from the training form; each
 * exported function has such pins (shared FFN: numpy matmul with all sizes distinct, math.erf, closed
 * forms for zero weights and zero input, linearity in the second matrix, planted mistakes).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };
enum { ORACLE_GELU_ERF = 0, ORACLE_GELU_TANH = 1 };

static double ld(const void *p, int dtype, int64_t i)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)p)[i];
    if (dtype == ORACLE_F64)
        return ((const double *)p)[i];
    /* bfloat16: the upper half of an fp32 */
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int mole_oracle_version(void) { return 1; }

/* GELU, exact form x*Phi(x) or the tanh approximation. */
double mole_oracle_gelu(double x, int act)
{
    if (act == ORACLE_GELU_TANH) {
        const double k = 0.79788456080286535588; /* sqrt(2/pi) */
        return 0.5 * x * (1.0 + tanh(k * (x + 0.044715 * x * x * x)));
    }
    return 0.5 * x * (1.0 + erf(x * 0.70710678118654752440));
}

/* Router equation: gates[t,j] = softmax_j( sum_k h[t,k] * W_r[k,j] ).  W_r is [d,N]. */
int mole_oracle_gates(const void *h, int h_dtype, const void *W_r, int w_dtype,
                      int64_t T, int d, int N, double *gates)
{
    if (!h || !W_r || !gates || T < 0 || d <= 0 || N <= 0)
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        double *g = gates + t * N;
        for (int j = 0; j < N; ++j) {
            double z = 0.0;
            for (int k = 0; k < d; ++k)
                z += ld(h, h_dtype, t * d + k) * ld(W_r, w_dtype, (int64_t)k * N + j);
            g[j] = z;
        }
        double m = g[0];
        for (int j = 1; j < N; ++j)
            if (g[j] > m)
                m = g[j];
        double s = 0.0;
        for (int j = 0; j < N; ++j) {
            g[j] = exp(g[j] - m);
            s += g[j];
        }
        for (int j = 0; j < N; ++j)
            g[j] /= s;
    }
    return 0;
}

/*
 * Inference-layer equation:
 *   out[t,c] = sum_j g[t,j] * table[ids[t], j, c] + shared[t,c] + residual[t,c]
 * table is [V,N,d]; shared / residual may be NULL (= 0).  rows[t] (nullable) receives the
 * row index read, or -1 for an id outside [0,V); *err (nullable) is set to 1 if any id is.
 * gates_out (nullable) receives the [T,N] gates.
 */
int mole_oracle_lookup_forward(const void *table, int table_dtype,
                               const int32_t *ids,
                               const void *h, const void *W_r,
                               const void *shared, const void *residual, int act_dtype,
                               int64_t T, int64_t V, int d, int N,
                               double *out, double *gates_out, int64_t *rows, int32_t *err)
{
    if (!table || !ids || !h || !W_r || !out || T < 0 || V <= 0 || d <= 0 || N <= 0)
        return 1;
    double *gates = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * (size_t)N);
    if (!gates)
        return 2;
    int rc = mole_oracle_gates(h, act_dtype, W_r, act_dtype, T, d, N, gates);
    if (rc) {
        free(gates);
        return rc;
    }
    int any_bad = 0;
#pragma omp parallel for schedule(static) reduction(| : any_bad)
    for (int64_t t = 0; t < T; ++t) {
        const int64_t id = ids[t];
        const int ok = (id >= 0 && id < V);
        if (!ok)
            any_bad |= 1;
        if (rows)
            rows[t] = ok ? id : -1;
        for (int c = 0; c < d; ++c) {
            double routed = 0.0;
            if (ok)
                for (int j = 0; j < N; ++j)
                    routed += gates[t * N + j] * ld(table, table_dtype, (id * N + j) * (int64_t)d + c);
            double v = routed;
            if (shared)
                v += ld(shared, act_dtype, t * d + c);
            if (residual)
                v += ld(residual, act_dtype, t * d + c);
            out[t * d + c] = v;
        }
    }
    if (gates_out)
        memcpy(gates_out, gates, sizeof(double) * (size_t)T * (size_t)N);
    if (err)
        *err = any_bad;
    free(gates);
    return 0;
}

/*
 * The MoLE part of the inference listing (Appendix, inference phase), from the state after attention:
 *   hn[t,:]  = x[t,:] / sqrt(mean_k x[t,k]^2 + eps) * ln_w          post-attention RMSNorm
 *   g[t,:]   = softmax(hn[t,:] . W_r)
 *   out[t,c] = x[t,c] + shared[t,c] + sum_j g[t,j] * table[ids[t], j, c]
 * x is both the norm's input and the residual.  hn is kept in fp64 (no rounding to storage).
 * shared may be NULL (= 0).  gates_out, hn_out, rows, err nullable.
 */
int mole_oracle_layer_forward(const void *table, int table_dtype, const int32_t *ids,
                              const void *x, const void *ln_w, double eps, const void *W_r,
                              const void *shared, int act_dtype,
                              int64_t T, int64_t V, int d, int N,
                              double *out, double *gates_out, double *hn_out, int64_t *rows, int32_t *err)
{
    if (!table || !ids || !x || !ln_w || !W_r || !out || T < 0 || V <= 0 || d <= 0 || N <= 0)
        return 1;
    double *hn = (double *)calloc((size_t)(T > 0 ? T : 1) * (size_t)d, sizeof(double));
    double *gates = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * (size_t)N);
    if (!hn || !gates) {
        free(hn);
        free(gates);
        return 2;
    }
    for (int64_t t = 0; t < T; ++t) {
        double ss = 0.0;
        for (int k = 0; k < d; ++k) {
            const double v = ld(x, act_dtype, t * d + k);
            ss += v * v;
        }
        const double rs = 1.0 / sqrt(ss / (double)d + eps);
        for (int k = 0; k < d; ++k)
            hn[t * d + k] = ld(x, act_dtype, t * d + k) * rs * ld(ln_w, act_dtype, k);
    }
    int rc = mole_oracle_gates(hn, 2, W_r, act_dtype, T, d, N, gates);
    if (rc) {
        free(hn);
        free(gates);
        return rc;
    }
    int any_bad = 0;
    for (int64_t t = 0; t < T; ++t) {
        const int64_t id = ids[t];
        const int ok = (id >= 0 && id < V);
        if (!ok)
            any_bad = 1;
        if (rows)
            rows[t] = ok ? id : -1;
        for (int c = 0; c < d; ++c) {
            double v = ld(x, act_dtype, t * d + c);
            if (shared)
                v += ld(shared, act_dtype, t * d + c);
            if (ok)
                for (int j = 0; j < N; ++j)
                    v += gates[t * N + j] * ld(table, table_dtype, (id * N + j) * (int64_t)d + c);
            out[t * d + c] = v;
        }
    }
    if (gates_out)
        memcpy(gates_out, gates, sizeof(double) * (size_t)T * (size_t)N);
    if (hn_out)
        memcpy(hn_out, hn, sizeof(double) * (size_t)T * (size_t)d);
    if (err)
        *err = any_bad;
    free(hn);
    free(gates);
    return 0;
}

/*
 * Canonical dedup map: uniq = distinct in-range ids, ascending; inv[t] = index of ids[t] in uniq
 * (-1 for an id outside [0,V), which also sets *err).  Written as the definition: mark, then rank.
 */
int mole_oracle_dedup(const int32_t *ids, int64_t T, int64_t V,
                      int32_t *uniq, int32_t *inv, int32_t *n_uniq, int32_t *err)
{
    if (!ids || !uniq || !inv || !n_uniq || T < 0 || V <= 0)
        return 1;
    int32_t *rank = (int32_t *)malloc(sizeof(int32_t) * (size_t)V);
    if (!rank)
        return 2;
    for (int64_t v = 0; v < V; ++v)
        rank[v] = -1;
    int bad = 0;
    for (int64_t t = 0; t < T; ++t) {
        if (ids[t] < 0 || ids[t] >= V)
            bad = 1;
        else
            rank[ids[t]] = 0;
    }
    int32_t U = 0;
    for (int64_t v = 0; v < V; ++v)
        if (rank[v] == 0) {
            rank[v] = U;
            uniq[U++] = (int32_t)v;
        }
    for (int64_t t = 0; t < T; ++t)
        inv[t] = (ids[t] < 0 || ids[t] >= V) ? -1 : rank[ids[t]];
    *n_uniq = U;
    if (err)
        *err = bad;
    free(rank);
    return 0;
}

/*
 * LUT entry equation: for every requested vocabulary row v and expert j
 *   x = E[v]                       (or RMSNorm(E[v]) = E[v] / sqrt(mean(E[v]^2) + eps) * norm_w)
 *   a[m] = sum_k x[k] * W1[j,k,m] + b1[j,m]
 *   LUT[v,j,c] = sum_m GELU(a[m]) * W2[j,m,c] + b2[j,c]
 * E [V,d], W1 [N,d,D], W2 [N,D,d], b1 [N,D], b2 [N,d], norm_w [d]; biases and norm_w nullable.
 * rows (nullable) selects n_rows vocabulary ids; with rows == NULL rows 0..n_rows-1 are built.
 * lut_out is [n_rows, N, d] in double.
 */
int mole_oracle_build_lut(const void *E, const void *W1, const void *b1,
                          const void *W2, const void *b2, const void *norm_w, double norm_eps,
                          int dtype, int64_t V, int d, int D, int N, int act,
                          const int32_t *rows, int64_t n_rows, double *lut_out)
{
    if (!E || !W1 || !W2 || !lut_out || V <= 0 || d <= 0 || D <= 0 || N <= 0 || n_rows < 0)
        return 1;
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t v = rows ? rows[r] : r;
        if (v < 0 || v >= V)
            return 1;
    }
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)d);
        double *a = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < n_rows; ++r) {
            const int64_t v = rows ? rows[r] : r;
            for (int k = 0; k < d; ++k)
                x[k] = ld(E, dtype, v * d + k);
            if (norm_w) {
                double ms = 0.0;
                for (int k = 0; k < d; ++k)
                    ms += x[k] * x[k];
                ms /= (double)d;
                const double inv_rms = 1.0 / sqrt(ms + norm_eps);
                for (int k = 0; k < d; ++k)
                    x[k] = x[k] * inv_rms * ld(norm_w, dtype, k);
            }
            for (int j = 0; j < N; ++j) {
                /* each sum runs over its index in ascending order; the loops are nested with the
                 * summed index outside only so that the weight matrices are walked along rows */
                double *o = lut_out + (r * N + j) * (int64_t)d;
                for (int m = 0; m < D; ++m)
                    a[m] = 0.0;
                for (int k = 0; k < d; ++k)
                    for (int m = 0; m < D; ++m)
                        a[m] += x[k] * ld(W1, dtype, ((int64_t)j * d + k) * D + m);
                for (int m = 0; m < D; ++m) {
                    if (b1)
                        a[m] += ld(b1, dtype, (int64_t)j * D + m);
                    a[m] = mole_oracle_gelu(a[m], act);
                }
                for (int c = 0; c < d; ++c)
                    o[c] = 0.0;
                for (int m = 0; m < D; ++m)
                    for (int c = 0; c < d; ++c)
                        o[c] += a[m] * ld(W2, dtype, ((int64_t)j * D + m) * d + c);
                if (b2)
                    for (int c = 0; c < d; ++c)
                        o[c] += ld(b2, dtype, (int64_t)j * d + c);
            }
        }
        free(x);
        free(a);
    }
    return 0;
}

/*
 * Shared expert of the layer (inference listing, "Shared Expert": shared_output = mlp(hidden_states); the
 * FFN_shared(h) term of the inference-layer equation), as a two-matrix FFN:
 *   a[m]     = sum_k x[t,k] * W1[m,k] + b1[m]          m = 0..D-1
 *   out[t,c] = sum_m GELU(a[m]) * W2[c,m] + b2[c]      c = 0..d-1
 * x [T,d]; W1 [D,d] and W2 [d,D] are stored as a linear layer stores its weight ([out, in]); b1 [D], b2 [d]
 * nullable.  out is [T,d] in double.
 */
int mole_oracle_shared_ffn(const void *x, const void *W1, const void *b1, const void *W2, const void *b2,
                           int dtype, int64_t T, int d, int D, int act, double *out)
{
    if (!x || !W1 || !W2 || !out || T < 0 || d <= 0 || D <= 0)
        return 1;
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 1)
        for (int64_t t = 0; t < T; ++t) {
            for (int m = 0; m < D; ++m) {
                double s = 0.0;
                for (int k = 0; k < d; ++k)
                    s += ld(x, dtype, t * d + k) * ld(W1, dtype, (int64_t)m * d + k);
                if (b1)
                    s += ld(b1, dtype, m);
                a[m] = mole_oracle_gelu(s, act);
            }
            for (int c = 0; c < d; ++c) {
                double s = 0.0;
                for (int m = 0; m < D; ++m)
                    s += a[m] * ld(W2, dtype, (int64_t)c * D + m);
                if (b2)
                    s += ld(b2, dtype, c);
                out[t * d + c] = s;
            }
        }
        free(a);
    }
    return 0;
}
