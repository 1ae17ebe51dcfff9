/*
 * TEST INFRASTRUCTURE -- not part of the product path.
 *
 * Plain fp64 CPU definition of softmax attention for the decode phase (the paper's
 * Eq. 1 in Section 2.1, with N_q = 1 as in the decode column of Table 1) and for short
 * query tiles (N_q > 1), one query row at a time:
 *
 *     s_t  = scale * sum_j q[j] * k[t][j]          for t < N
 *     w_t  = exp(s_t - max_t s_t)
 *     out  = (sum_t w_t * v[t]) / (sum_t w_t)
 *     lse  = max_t s_t + log(sum_t w_t)             (the L of Algorithm 2)
 *
 * Two passes over the context, no tiling, no splitting, no re-scaling
 * operator: this is the result LeanAttention must reach exactly (Section 4.1
 * claims the split/merge gives the same exact output for any split).
 *
 * Inputs are the raw 16-bit patterns (IEEE binary16 or bfloat16) the GPU
 * path reads, widened exactly to double, or plain doubles for hand-made
 * pins.  A query head h_q reads KV head h_q / (Hq / Hkv).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg call this
 * file.  It shares no code with the HIP path.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };
enum { ORACLE_KV_PADDED = 0, ORACLE_KV_PACKED = 1 };

static double widen_bf16(uint16_t bits) {
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double widen_f16(uint16_t bits) {
    int sign = (bits >> 15) & 1;
    int expo = (bits >> 10) & 0x1f;
    int frac = bits & 0x3ff;
    double mag;
    if (expo == 0) {
        mag = ldexp((double)frac, -24); /* zero and subnormals */
    } else if (expo == 31) {
        mag = frac ? NAN : INFINITY;
    } else {
        mag = ldexp((double)(1024 + frac), expo - 25);
    }
    return sign ? -mag : mag;
}

/* Widen one row of D elements starting at element offset `row_off`. */
static void widen_row(const void* base, int64_t row_off, int D, int dtype, double* dst) {
    if (dtype == ORACLE_F64) {
        memcpy(dst, (const double*)base + row_off, (size_t)D * sizeof(double));
        return;
    }
    const uint16_t* p = (const uint16_t*)base + row_off;
    for (int j = 0; j < D; ++j) dst[j] = dtype == ORACLE_BF16 ? widen_bf16(p[j]) : widen_f16(p[j]);
}

/*
 * One (query row, context) pair: `k_rows`/`v_rows` point at element offset
 * `kv_off` of the first cached row; rows are D elements apart.
 * `scores` is caller scratch of n doubles, `row` of D doubles.
 */
static void attend_one(const void* q, int64_t q_off, const void* k_rows, const void* v_rows,
                       int64_t kv_off, int64_t n, int D, int dtype, double scale, double* scores,
                       double* row, double* qrow, double* out, double* lse) {
    for (int j = 0; j < D; ++j) out[j] = 0.0;
    if (n <= 0) { /* empty context: defined as zeros, lse = -inf */
        if (lse) *lse = -INFINITY;
        return;
    }
    widen_row(q, q_off, D, dtype, qrow);
    double smax = -INFINITY;
    for (int64_t t = 0; t < n; ++t) {
        widen_row(k_rows, kv_off + t * D, D, dtype, row);
        double dot = 0.0;
        for (int j = 0; j < D; ++j) dot += qrow[j] * row[j];
        scores[t] = scale * dot;
        if (scores[t] > smax) smax = scores[t];
    }
    double z = 0.0;
    for (int64_t t = 0; t < n; ++t) {
        double w = exp(scores[t] - smax);
        z += w;
        widen_row(v_rows, kv_off + t * D, D, dtype, row);
        for (int j = 0; j < D; ++j) out[j] += w * row[j];
    }
    for (int j = 0; j < D; ++j) out[j] /= z;
    if (lse) *lse = smax + log(z);
}

/*
 * Query tiles (N_q >= 1 rows per sequence; Algorithm 2 counts C_m = ceil(N_q / T_m) output
 * tiles of them).  The query tokens of sequence b are its LAST q_len[b] cached tokens.
 *
 * q   : [sum_b q_len[b], Hq, D]: the query tokens of sequence 0, then of sequence 1, ...
 *       (with every q_len[b] = N_q this is [B, N_q, Hq, D])
 * k,v : PADDED [B, Hkv, n_stride, D]  (row t of (b,h) at ((b*Hkv+h)*n_stride + t)*D), or
 *       PACKED [Hkv, total, D] with total = sum(seqlens), sequence b starting at
 *       row cu[b] = sum_{b'<b} seqlens[b'] (n_stride ignored)
 * causal = 0: every query row attends to all N_b cached rows.
 * causal = 1: query row i (0-based) is token N_b - q_len[b] + i of its sequence and attends to
 *             the cached rows t <= N_b - q_len[b] + i, i.e. to N_b - q_len[b] + i + 1 rows.  (The
 *             paper does not discuss masking; this is the usual decoder mask aligned to the end of
 *             the context.)  Needs N_b >= q_len[b] or N_b == 0.
 * out : [sum_b q_len[b], Hq, D] doubles;  lse: [sum_b q_len[b], Hq] doubles or NULL
 * Returns the number of threads used, or a negative value for bad arguments.
 */
int oracle_attention_ragged(const void* q, const void* k, const void* v, const int32_t* seqlens,
                            const int32_t* q_lens, int B, int Hq, int Hkv, int D, int dtype,
                            int kv_layout, int64_t n_stride, double scale, int causal, double* out,
                            double* lse, int n_threads) {
    if (!q || !k || !v || !seqlens || !q_lens || !out) return -1;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0) return -2;
    if (dtype < 0 || dtype > 2 || kv_layout < 0 || kv_layout > 1) return -3;
    int64_t total = 0, nmax = 0, q_total = 0;
    int64_t* cu = (int64_t*)malloc((size_t)(2 * B + 2) * sizeof(int64_t));
    if (!cu) return -4;
    int64_t* cu_q = cu + B + 1;
    for (int b = 0; b < B; ++b) {
        if (seqlens[b] < 0 || q_lens[b] < 0) { free(cu); return -5; }
        if (causal && seqlens[b] != 0 && seqlens[b] < q_lens[b]) { free(cu); return -7; }
        cu[b] = total;
        cu_q[b] = q_total;
        total += seqlens[b];
        q_total += q_lens[b];
        if (seqlens[b] > nmax) nmax = seqlens[b];
    }
    cu[B] = total;
    cu_q[B] = q_total;
    if (kv_layout == ORACLE_KV_PADDED && n_stride < nmax) { free(cu); return -6; }
    const int group = Hq / Hkv;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
#endif
        double* scores = (double*)malloc((size_t)(nmax > 0 ? nmax : 1) * sizeof(double));
        double* row = (double*)malloc((size_t)D * sizeof(double));
        double* qrow = (double*)malloc((size_t)D * sizeof(double));
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t r = 0; r < q_total * Hq; ++r) {
            int64_t token = r / Hq; /* index into the concatenated query tokens */
            int hq = (int)(r % Hq);
            int b = 0;
            while (cu_q[b + 1] <= token) ++b; /* the sequence that owns this query token */
            int i = (int)(token - cu_q[b]);
            int h;
            h = hq / group;
            int64_t kv_off = kv_layout == ORACLE_KV_PADDED
                                 ? ((int64_t)(b * (int64_t)Hkv + h) * n_stride) * D
                                 : ((int64_t)h * total + cu[b]) * D;
            int64_t n_visible = seqlens[b];
            if (causal && n_visible > 0) n_visible = n_visible - q_lens[b] + i + 1;
            attend_one(q, r * D, k, v, kv_off, n_visible, D, dtype, scale, scores, row, qrow,
                       out + r * D, lse ? lse + r : NULL);
        }
        free(scores);
        free(row);
        free(qrow);
#ifdef _OPENMP
    }
#endif
    free(cu);
    return used;
}

/* The same with N_q query tokens for every sequence: q, out [B, N_q, Hq, D], lse [B, N_q, Hq]. */
int oracle_attention(const void* q, const void* k, const void* v, const int32_t* seqlens, int B,
                     int N_q, int Hq, int Hkv, int D, int dtype, int kv_layout, int64_t n_stride,
                     double scale, int causal, double* out, double* lse, int n_threads) {
    if (B <= 0 || N_q <= 0) return -2;
    int32_t* q_lens = (int32_t*)malloc((size_t)B * sizeof(int32_t));
    if (!q_lens) return -4;
    for (int b = 0; b < B; ++b) q_lens[b] = N_q;
    int rc = oracle_attention_ragged(q, k, v, seqlens, q_lens, B, Hq, Hkv, D, dtype, kv_layout,
                                     n_stride, scale, causal, out, lse, n_threads);
    free(q_lens);
    return rc;
}

/*
 * Decode: N_q = 1 (the mask plays no role).
 * q   : [B, Hq, D];  out : [B, Hq, D] doubles;  lse: [B, Hq] doubles or NULL
 */
int oracle_decode_attention(const void* q, const void* k, const void* v, const int32_t* seqlens,
                            int B, int Hq, int Hkv, int D, int dtype, int kv_layout,
                            int64_t n_stride, double scale, double* out, double* lse,
                            int n_threads) {
    return oracle_attention(q, k, v, seqlens, B, 1, Hq, Hkv, D, dtype, kv_layout, n_stride, scale, 0,
                            out, lse, n_threads);
}
