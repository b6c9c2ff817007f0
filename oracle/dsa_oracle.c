/*
 * CPU oracle for the Dynamic Sparse Attention (DSA) forward path.
 *
 * TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the test-suite, the smoke check and
 * the benchmark's cpu_baseline leg call this file.  It shares no code with the HIP
 * library and is deliberately plain: one loop nest per equation, no blocking, no SIMD
 * intrinsics, no BLAS.  OpenMP only distributes independent (head, unit) problems over
 * threads; nothing inside a unit is reordered.
 *
 * What it computes, and where the paper defines it:
 *
 *   step 1  approximate scores  S~[i,j] = sum_c Q~[i,c] K~[j,c]  as exact integers
 *           (section 3.1: S~ = Q~ K~^T from the low-precision projections).
 *   step 2  vector-wise only: group score  Sg[g,j] = sum_{r<vec} S~[vec*g+r, j]
 *           (section 5.1, column-vector sparsity: one decision per vector of `vec`
 *           consecutive query rows and one key column; the aggregate is their sum).
 *   step 3  per unit (row or group) keep the `keep` keys with the largest score
 *           (section 3.1: mask from S~ "determined by top-k searching"; section 4.2 /
 *           5.2: the same count in every row).  Total order: larger score first, equal
 *           scores by lower key index first.  The kept indices are emitted ascending.
 *   step 4  S[i,t] = scale * sum_c Q[i,c] K[j_t,c]   (equation 2 at the kept positions:
 *           the SDDMM of section 3.4 / 5.1).
 *   step 5  P[i,t] = exp(S[i,t]-m) / sum_t exp(S[i,t]-m),  m = max_t S[i,t]
 *           (equation 4: masked entries get -c and so weight 0 -> softmax over kept only).
 *   step 6  O[i,:] = sum_t P[i,t] V[j_t,:]            (equation 3: the SpMM).
 *
 *   step 0  (the step in front of the path, section 3.1 equation 5: reduced-dimension, low-precision
 *           projections)  Y = X R,  Q~ = quantise(Y) symmetric per tensor to int8.  The paper
 *           fixes neither the precision of the projection nor the quantiser; because a rounding
 *           decides an integer code here, this step alone is evaluated in the kernel's precision:
 *           fp32, one chain of fused multiply-adds in increasing c, fp32 scale 127/max|Y|, round
 *           half to even.
 *
 * Floating point is double throughout the attention path; Q, K, V arrive as float (bfloat16 inputs are
 * widened exactly by the caller).  Every function can be restricted to a list of units
 * / rows so that full-size workloads can be spot-checked.
 *
 * Layouts (all row-major, innermost last):
 *   Qt, Kt  int8   [N, L, k]        N = B*H
 *   Q, K, V float  [N, L, d]
 *   idx     int32  [N, L/vec, keep]
 * "unit id" u in [0, N*L/vec): head n = u / (L/vec), unit-in-head g = u % (L/vec).
 * "row id"  r in [0, N*L):     head n = r / L, row i = r % L, its unit g = i / vec.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int32_t dsao_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* keep = round-half-up(ratio * L), clamped to [1, L].  10% of 256 -> 26, of 512 -> 51;
 * 5% of 2048 -> 102, of 4096 -> 205; 1% of 8192 -> 82. */
int32_t dsao_keep_from_ratio(int32_t L, double ratio)
{
    double x = floor(ratio * (double)L + 0.5);
    if (x < 1.0) x = 1.0;
    if (x > (double)L) x = (double)L;
    return (int32_t)x;
}

/* Steps 1-2 for one unit: out[j] for j in [0, L). */
static void unit_scores(const int8_t *Qt, const int8_t *Kt, int64_t L, int64_t k, int64_t vec,
                        int64_t n, int64_t g, int64_t *out)
{
    const int8_t *Kh = Kt + n * L * k;
    for (int64_t j = 0; j < L; ++j) {
        int64_t group_sum = 0;
        for (int64_t r = 0; r < vec; ++r) {
            const int8_t *q = Qt + (n * L + g * vec + r) * k;
            int64_t s = 0;                       /* step 1: one approximate score */
            for (int64_t c = 0; c < k; ++c)
                s += (int64_t)q[c] * (int64_t)Kh[j * k + c];
            group_sum += s;                      /* step 2 */
        }
        out[j] = group_sum;
    }
}

/* Steps 1-2, exported for the pins: scores [n_units, L] as int64. */
int32_t dsao_approx_scores(const int8_t *Qt, const int8_t *Kt, int32_t N, int32_t L, int32_t k,
                           int32_t vec, const int64_t *units, int64_t n_units, int64_t *scores)
{
    if (!Qt || !Kt || !scores || N < 1 || L < 1 || k < 1 || vec < 1 || L % vec) return 1;
    int64_t G = L / vec;
    if (!units) n_units = (int64_t)N * G;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < n_units; ++t) {
        int64_t u = units ? units[t] : t;
        unit_scores(Qt, Kt, L, k, vec, u / G, u % G, scores + t * (int64_t)L);
    }
    return 0;
}

typedef struct { int64_t score; int32_t j; } scored_key;

/* Total order of step 3: larger score first; equal scores: lower key index first. */
static int by_score_desc_then_index(const void *a, const void *b)
{
    const scored_key *x = (const scored_key *)a, *y = (const scored_key *)b;
    if (x->score != y->score) return x->score > y->score ? -1 : 1;
    return (x->j > y->j) - (x->j < y->j);
}

static int by_int32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Steps 1-3: idx [n_units, keep], each list ascending. */
int32_t dsao_predict_mask(const int8_t *Qt, const int8_t *Kt, int32_t N, int32_t L, int32_t k,
                          int32_t vec, int32_t keep, const int64_t *units, int64_t n_units,
                          int32_t *idx)
{
    if (!Qt || !Kt || !idx || N < 1 || L < 1 || k < 1 || vec < 1 || L % vec) return 1;
    if (keep < 1 || keep > L) return 1;
    int64_t G = L / vec;
    if (!units) n_units = (int64_t)N * G;
    int failed = 0;
#pragma omp parallel
    {
        int64_t *sc = (int64_t *)malloc(sizeof(int64_t) * (size_t)L);
        scored_key *keys = (scored_key *)malloc(sizeof(scored_key) * (size_t)L);
        if (!sc || !keys) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 16)
        for (int64_t t = 0; t < n_units; ++t) {
            if (!sc || !keys) continue;
            int64_t u = units ? units[t] : t;
            unit_scores(Qt, Kt, L, k, vec, u / G, u % G, sc);
            for (int32_t j = 0; j < L; ++j) { keys[j].score = sc[j]; keys[j].j = j; }
            qsort(keys, (size_t)L, sizeof(scored_key), by_score_desc_then_index);
            int32_t *out = idx + t * (int64_t)keep;
            for (int32_t a = 0; a < keep; ++a) out[a] = keys[a].j;
            qsort(out, (size_t)keep, sizeof(int32_t), by_int32);
        }
        free(sc);
        free(keys);
    }
    return failed;
}

/* Step 4 for the rows listed (all rows if rows == NULL): S [n_rows, keep] in double.
 * idx is the full [N, L/vec, keep] tensor. */
int32_t dsao_sddmm(const float *Q, const float *K, const int32_t *idx, int32_t N, int32_t L,
                   int32_t d, int32_t vec, int32_t keep, double scale, const int64_t *rows,
                   int64_t n_rows, double *S)
{
    if (!Q || !K || !idx || !S || N < 1 || L < 1 || d < 1 || vec < 1 || L % vec || keep < 1) return 1;
    int64_t G = L / vec;
    if (!rows) n_rows = (int64_t)N * L;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < n_rows; ++t) {
        int64_t r = rows ? rows[t] : t;
        int64_t n = r / L, i = r % L, g = i / vec;
        const float *q = Q + r * d;
        const int32_t *list = idx + (n * G + g) * keep;
        for (int32_t a = 0; a < keep; ++a) {
            const float *kr = K + (n * L + list[a]) * (int64_t)d;
            double acc = 0.0;
            for (int32_t c = 0; c < d; ++c) acc += (double)q[c] * (double)kr[c];
            S[t * keep + a] = scale * acc;
        }
    }
    return 0;
}

/* Step 5 on n_rows lists of `keep` scores. */
int32_t dsao_sparse_softmax(const double *S, int64_t n_rows, int32_t keep, double *P)
{
    if (!S || !P || keep < 1 || n_rows < 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_rows; ++t) {
        const double *s = S + t * keep;
        double *p = P + t * keep;
        double m = s[0];
        for (int32_t a = 1; a < keep; ++a) if (s[a] > m) m = s[a];
        double z = 0.0;
        for (int32_t a = 0; a < keep; ++a) { p[a] = exp(s[a] - m); z += p[a]; }
        for (int32_t a = 0; a < keep; ++a) p[a] = p[a] / z;
    }
    return 0;
}

/* Step 6 for the rows listed: O [n_rows, d] in double.  P is [n_rows, keep]. */
int32_t dsao_spmm(const double *P, const int32_t *idx, const float *V, int32_t N, int32_t L,
                  int32_t d, int32_t vec, int32_t keep, const int64_t *rows, int64_t n_rows,
                  double *O)
{
    if (!P || !idx || !V || !O || N < 1 || L < 1 || d < 1 || vec < 1 || L % vec || keep < 1) return 1;
    int64_t G = L / vec;
    if (!rows) n_rows = (int64_t)N * L;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < n_rows; ++t) {
        int64_t r = rows ? rows[t] : t;
        int64_t n = r / L, i = r % L, g = i / vec;
        const int32_t *list = idx + (n * G + g) * keep;
        double *o = O + t * d;
        for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
        for (int32_t a = 0; a < keep; ++a) {
            const float *vr = V + (n * L + list[a]) * (int64_t)d;
            double p = P[t * keep + a];
            for (int32_t c = 0; c < d; ++c) o[c] += p * (double)vr[c];
        }
    }
    return 0;
}

/* Steps 4-6 chained for the rows listed, given idx.  S, P may be NULL. */
int32_t dsao_masked_attention(const float *Q, const float *K, const float *V, const int32_t *idx,
                              int32_t N, int32_t L, int32_t d, int32_t vec, int32_t keep,
                              double scale, const int64_t *rows, int64_t n_rows, double *O,
                              double *S_out, double *P_out)
{
    if (!rows) n_rows = (int64_t)N * L;
    if (n_rows < 0 || keep < 1) return 1;
    double *S = S_out ? S_out : (double *)malloc(sizeof(double) * (size_t)n_rows * keep);
    double *P = P_out ? P_out : (double *)malloc(sizeof(double) * (size_t)n_rows * keep);
    int32_t rc = 1;
    if (S && P) {
        rc = dsao_sddmm(Q, K, idx, N, L, d, vec, keep, scale, rows, n_rows, S);
        if (!rc) rc = dsao_sparse_softmax(S, n_rows, keep, P);
        if (!rc) rc = dsao_spmm(P, idx, V, N, L, d, vec, keep, rows, n_rows, O);
    }
    if (!S_out) free(S);
    if (!P_out) free(P);
    return rc;
}

/* Step 0: Xt [rows, k] = quantise(X [rows, d] . R [d, k]); *amax = max |Y|.  fp32 by design (see
 * the header comment): y is built by fmaf in increasing c, exactly one rounding per term.
 * `bits` is the prediction precision (section 3.3 takes INT4, table 2 sweeps INT2 to INT16): the
 * codes are the integers of magnitude up to qmax = 2^(bits-1) - 1, one per int8 here. */
int32_t dsao_project_quantize_bits(const float *X, const float *R, int64_t rows, int32_t d, int32_t k,
                                   int32_t bits, int8_t *Xt, float *amax_out)
{
    if (!X || !R || !Xt || rows < 0 || d < 1 || k < 1 || bits < 2 || bits > 8) return 1;
    const float qmax = (float)((1 << (bits - 1)) - 1);
    float *Y = (float *)malloc(sizeof(float) * (size_t)rows * (size_t)k + 4);
    if (!Y) return 1;
    float amax = 0.0f;
#pragma omp parallel for schedule(static) reduction(max : amax)
    for (int64_t r = 0; r < rows; ++r) {
        for (int32_t j = 0; j < k; ++j) {
            float y = 0.0f;
            for (int32_t c = 0; c < d; ++c) y = fmaf(X[r * d + c], R[(int64_t)c * k + j], y);
            Y[r * k + j] = y;
            if (fabsf(y) > amax) amax = fabsf(y);
        }
    }
    const float s = amax > 0.0f ? qmax / amax : 0.0f;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < rows * (int64_t)k; ++t) {
        float v = rintf(Y[t] * s);            /* default rounding mode: halves to even */
        if (v > qmax) v = qmax;
        if (v < -qmax) v = -qmax;
        Xt[t] = (int8_t)v;
    }
    if (amax_out) *amax_out = amax;
    free(Y);
    return 0;
}

int32_t dsao_project_quantize(const float *X, const float *R, int64_t rows, int32_t d, int32_t k,
                              int8_t *Xt, float *amax_out)
{
    return dsao_project_quantize_bits(X, R, rows, d, k, 8, Xt, amax_out);
}

/* Storage of low-precision codes: 8/bits codes per byte, two's complement fields, code j of a row
 * in bits [bits * (j mod 8/bits), + bits) of byte j / (8/bits).  n = number of codes, a multiple of
 * 8/bits.  bits = 8 copies. */
int32_t dsao_pack_codes(const int8_t *codes, int64_t n, int32_t bits, uint8_t *packed)
{
    if (!codes || !packed || n < 0 || (bits != 2 && bits != 4 && bits != 8)) return 1;
    const int32_t per = 8 / bits;
    if (n % per) return 1;
    const int32_t lim = (1 << (bits - 1)) - 1;
    for (int64_t b = 0; b < n / per; ++b) {
        uint32_t byte = 0;
        for (int32_t f = 0; f < per; ++f) {
            const int32_t c = codes[b * per + f];
            if (bits < 8 && (c > lim || c < -lim)) return 2;      /* not representable */
            byte |= ((uint32_t)c & ((1u << bits) - 1u)) << (bits * f);
        }
        packed[b] = (uint8_t)byte;
    }
    return 0;
}

int32_t dsao_unpack_codes(const uint8_t *packed, int64_t n, int32_t bits, int8_t *codes)
{
    if (!codes || !packed || n < 0 || (bits != 2 && bits != 4 && bits != 8)) return 1;
    const int32_t per = 8 / bits;
    if (n % per) return 1;
    for (int64_t j = 0; j < n; ++j) {
        const uint32_t field = ((uint32_t)packed[j / per] >> (bits * (int32_t)(j % per))) & ((1u << bits) - 1u);
        const int32_t sign = 1 << (bits - 1);
        codes[j] = (int8_t)(((int32_t)field ^ sign) - sign);      /* sign extension of the field */
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------------
 * Threshold masks (section 3.1: the mask may also be predicted "using thresholds", the threshold
 * being a tuned constant).  The count per unit now varies, so the mask is stored in CSR form:
 *   row_ptr int64 [n_units + 1], col int32 [row_ptr[n_units]], each unit's keys ascending.
 * Step 3': unit u keeps every key j with score(u, j) >= theta (signed comparison of the exact
 * integer scores of steps 1-2).  A unit with no such key keeps its single best key (largest score,
 * lower index among equals): the softmax of its rows needs one entry, and that key is what a
 * lowered threshold would have admitted first.
 * With col == NULL only the counts are produced (row_ptr is filled); call again with col of
 * row_ptr[n_units] entries to get the keys. */
int32_t dsao_predict_mask_threshold(const int8_t *Qt, const int8_t *Kt, int32_t N, int32_t L, int32_t k,
                                    int32_t vec, int64_t theta, int64_t *row_ptr, int32_t *col)
{
    if (!Qt || !Kt || !row_ptr || N < 1 || L < 1 || k < 1 || vec < 1 || L % vec) return 1;
    const int64_t G = L / vec, n_units = (int64_t)N * G;
    int failed = 0;
    if (col == NULL) row_ptr[0] = 0;
#pragma omp parallel
    {
        int64_t *sc = (int64_t *)malloc(sizeof(int64_t) * (size_t)L);
        if (!sc) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 16)
        for (int64_t u = 0; u < n_units; ++u) {
            if (!sc) continue;
            unit_scores(Qt, Kt, L, k, vec, u / G, u % G, sc);
            int64_t count = 0;
            int32_t best = 0;
            for (int32_t j = 0; j < L; ++j) {
                if (sc[j] >= theta) {
                    if (col) col[row_ptr[u] + count] = j;
                    ++count;
                }
                if (sc[j] > sc[best]) best = j;          /* strict: the lower index wins among equals */
            }
            if (count == 0) {
                if (col) col[row_ptr[u]] = best;
                count = 1;
            }
            if (!col) row_ptr[u + 1] = count;            /* counts first; prefix sum below */
        }
        free(sc);
    }
    if (failed) return 1;
    if (!col)
        for (int64_t u = 0; u < n_units; ++u) row_ptr[u + 1] += row_ptr[u];
    return 0;
}

/* Steps 4-6 for a CSR mask (the same equations 2, 4, 3, per row over its unit's keys) for the rows
 * listed (all rows if rows == NULL): O [n_rows, d] in double. */
int32_t dsao_masked_attention_csr(const float *Q, const float *K, const float *V, const int64_t *row_ptr,
                                  const int32_t *col, int32_t N, int32_t L, int32_t d, int32_t vec,
                                  double scale, const int64_t *rows, int64_t n_rows, double *O)
{
    if (!Q || !K || !V || !row_ptr || !col || !O || N < 1 || L < 1 || d < 1 || vec < 1 || L % vec) return 1;
    const int64_t G = L / vec;
    if (!rows) n_rows = (int64_t)N * L;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < n_rows; ++t) {
        const int64_t r = rows ? rows[t] : t;
        const int64_t n = r / L, i = r % L, u = n * G + i / vec;
        const int32_t *list = col + row_ptr[u];
        const int64_t cnt = row_ptr[u + 1] - row_ptr[u];
        double *o = O + t * d;
        for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
        if (cnt < 1) continue;                            /* cannot happen for masks made above */
        double *p = (double *)malloc(sizeof(double) * (size_t)cnt);
        if (!p) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        const float *q = Q + r * d;
        double m = 0.0;
        for (int64_t a = 0; a < cnt; ++a) {               /* equation 2 at the kept positions */
            const float *kr = K + (n * L + list[a]) * (int64_t)d;
            double acc = 0.0;
            for (int32_t c = 0; c < d; ++c) acc += (double)q[c] * (double)kr[c];
            p[a] = scale * acc;
            if (a == 0 || p[a] > m) m = p[a];
        }
        double z = 0.0;
        for (int64_t a = 0; a < cnt; ++a) { p[a] = exp(p[a] - m); z += p[a]; }     /* equation 4 */
        for (int64_t a = 0; a < cnt; ++a) {               /* equation 3 */
            const float *vr = V + (n * L + list[a]) * (int64_t)d;
            const double w = p[a] / z;
            for (int32_t c = 0; c < d; ++c) o[c] += w * (double)vr[c];
        }
        free(p);
    }
    return failed;
}

/* Step 0 with the paper's own projection (section 3.1, equation 5): P in sqrt(3/k) * {-1, 0, 1}^(d x k),
 * a sparse random projection, so Y = X P needs additions and subtractions only.  P3 holds the signs
 * (-1, 0, 1).  The constant sqrt(3/k) > 0 multiplies every entry of Y and the quantiser's scale
 * qmax / max|Y| divides it out again, so it is left out; as for the dense projection the sums are
 * taken in fp32 in increasing c (one rounding per addition), because a rounding decides a code. */
int32_t dsao_project_quantize_ternary(const float *X, const int8_t *P3, int64_t rows, int32_t d, int32_t k,
                                      int32_t bits, int8_t *Xt, float *amax_out)
{
    if (!X || !P3 || !Xt || rows < 0 || d < 1 || k < 1 || bits < 2 || bits > 8) return 1;
    for (int64_t t = 0; t < (int64_t)d * k; ++t)
        if (P3[t] < -1 || P3[t] > 1) return 2;
    const float qmax = (float)((1 << (bits - 1)) - 1);
    float *Y = (float *)malloc(sizeof(float) * (size_t)rows * (size_t)k + 4);
    if (!Y) return 1;
    float amax = 0.0f;
#pragma omp parallel for schedule(static) reduction(max : amax)
    for (int64_t r = 0; r < rows; ++r) {
        for (int32_t j = 0; j < k; ++j) {
            float y = 0.0f;
            for (int32_t c = 0; c < d; ++c) {
                const int8_t sign = P3[(int64_t)c * k + j];
                if (sign > 0) y = y + X[r * d + c];
                else if (sign < 0) y = y - X[r * d + c];
            }
            Y[r * k + j] = y;
            if (fabsf(y) > amax) amax = fabsf(y);
        }
    }
    const float s = amax > 0.0f ? qmax / amax : 0.0f;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < rows * (int64_t)k; ++t) {
        float v = rintf(Y[t] * s);
        if (v > qmax) v = qmax;
        if (v < -qmax) v = -qmax;
        Xt[t] = (int8_t)v;
    }
    if (amax_out) *amax_out = amax;
    free(Y);
    return 0;
}
