/*
 * fq_oracle.c — CPU oracle for the FlattenQuant per-tensor-quantized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct statement of
 * what the method computes, written from the paper (arXiv 2402.17985).  It is used by the
 * tests, by the smoke check and by the benchmark's CPU-baseline leg.  The GPU library never
 * calls it, shares no header, table or helper with it, and must not be routed through it.
 *
 * Every function is the definition written out as loops: no blocking, no fusion, no
 * reordering beyond what the definition states.  The only parallelism is an OpenMP
 * "parallel for" over independent output rows.
 *
 * Conventions
 *   X   activations, M x K, row-major (K contiguous), fp32 (bf16/fp16 inputs are widened
 *       exactly to fp32 by the caller before they reach the oracle).
 *   W   weights in the nn.Linear storage layout, N x K row-major.  The paper writes
 *       Y = X W with W's j-th input channel matching X's j-th channel (Sec. 4.1, Eq. 4);
 *       "repeat weight channel j" is therefore "repeat column j of the N x K array".
 *   k   bit width, 8 or 4.  qmax = 2^(k-1) - 1 (Eq. 1), qmin = -2^(k-1).
 *   map src[p] (source channel of flattened slot p, -1 for padding) and rep[p] (n of that
 *       source channel, 0 for padding), p in [0, Kpad).
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py against values the
 * paper or plain arithmetic fixes (hand-worked examples, closed forms, brute force, the
 * X'W' = XW identity).  No function is "parity unpinned".
 *
 * Build: gcc -O3 -fopenmp -ffp-contract=off -shared -fPIC  (see oracle/build.py)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define FQO_OK 0
#define FQO_ERR_ARG 1
#define FQO_ERR_CAP 2
#define FQO_ERR_OVERFLOW 3

int fqo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int qmax_of(int bits) { return (1 << (bits - 1)) - 1; }
static int qmin_of(int bits) { return -(1 << (bits - 1)); }

/* ------------------------------------------------------------------------------------------
 * Flatten plan.  Sec. 4.1, Eq. 2: a channel whose calibrated max |x| exceeds the threshold T
 * receives extra channels; Eq. 3 fixes where they live: the original keeps index j, the
 * extras of channel j sit in an appended block starting at C + sum_{k<j} E_k, channels in
 * increasing j.  Reading taken for the count: total copies n_j = max(1, ceil(max_j / T)),
 * E_j = n_j - 1 (equals Eq. 2's floor except when max_j is an exact multiple of T, where
 * Eq. 2 would add one more, all-zero, channel).  The ratio is evaluated in float64.
 * The final channel count is rounded up to a multiple of `align` (Sec. 5.1 uses 32); padding
 * slots have src = -1, rep = 0.
 *
 * Call with cap = 0 (src, rep may be NULL) to obtain Kprime/Kpad only.
 * ---------------------------------------------------------------------------------------- */
int fqo_plan(const float *chmax, int K, float T, int align,
             int32_t *src, int32_t *rep, int cap, int *Kprime_out, int *Kpad_out)
{
    if (!chmax || K <= 0 || align <= 0 || !(T > 0.0f) || isinf(T)) return FQO_ERR_ARG;
    long long extra = 0;
    for (int j = 0; j < K; ++j) {
        float c = chmax[j];
        if (!(c >= 0.0f) || isinf(c)) return FQO_ERR_ARG;   /* NaN, negative, Inf */
        double r = (double)c / (double)T;
        long long n = (long long)ceil(r);
        if (n < 1) n = 1;
        extra += n - 1;
        if (extra > 0x3fffffff) return FQO_ERR_OVERFLOW;
    }
    long long Kprime = (long long)K + extra;
    long long Kpad = (Kprime + align - 1) / align * align;
    if (Kpad > 0x7fffffff) return FQO_ERR_OVERFLOW;
    if (Kprime_out) *Kprime_out = (int)Kprime;
    if (Kpad_out) *Kpad_out = (int)Kpad;
    if (cap == 0) return FQO_OK;
    if (!src || !rep) return FQO_ERR_ARG;
    if (cap < Kpad) return FQO_ERR_CAP;

    int next = K;                                   /* first free appended slot */
    for (int j = 0; j < K; ++j) {
        double r = (double)chmax[j] / (double)T;
        int n = (int)ceil(r);
        if (n < 1) n = 1;
        src[j] = j;                                 /* the original keeps its index */
        rep[j] = n;
        for (int e = 0; e < n - 1; ++e) {           /* its E_j extras, appended in channel order */
            src[next] = j;
            rep[next] = n;
            ++next;
        }
    }
    for (int p = next; p < (int)Kpad; ++p) { src[p] = -1; rep[p] = 0; }
    return FQO_OK;
}

/* max |v| over a buffer, fp32 (exact: max is order independent). */
float fqo_absmax(const float *v, long long count)
{
    float a = 0.0f;
    for (long long i = 0; i < count; ++i) {
        float t = fabsf(v[i]);
        if (t > a) a = t;
    }
    return a;
}

/* Round-half-to-even of an fp32 value to an integer, then clamp to the k-bit range.
 * Eq. 1's "round"; reading taken: ties to even (what rintf does in the default rounding
 * mode, and what torch.round does). */
static int round_clamp(float v, int bits)
{
    float r = rintf(v);
    int lo = qmin_of(bits), hi = qmax_of(bits);
    if (r < (float)lo) return lo;
    if (r > (float)hi) return hi;
    return (int)r;
}

/* ------------------------------------------------------------------------------------------
 * Weights, offline (Eq. 1 and Eq. 4).  s_w = max|W| / qmax.  The division by s_w is carried
 * out as one fp32 multiply by m_w = fl32(qmax / max|W|) (quotient formed in float64, rounded
 * once to fp32), then round-half-even, then clamp.  Column j of Wq is then repeated at every
 * slot p with src[p] = j; padding slots hold 0.  (Quantize-then-repeat equals
 * repeat-then-quantize because repetition does not change the maximum.)
 * An all-zero W gives all-zero output and s_w = 1.
 * ---------------------------------------------------------------------------------------- */
int fqo_flatten_weights(const float *W, int N, int K, const int32_t *src, int Kpad, int bits,
                        int8_t *Wq_out /* N x Kpad */, float *s_w_out)
{
    if (!W || !src || !Wq_out || !s_w_out || N <= 0 || K <= 0 || Kpad <= 0) return FQO_ERR_ARG;
    if (bits != 8 && bits != 4) return FQO_ERR_ARG;
    float a_w = fqo_absmax(W, (long long)N * K);
    int qmax = qmax_of(bits);
    float m_w, s_w;
    if (a_w == 0.0f) { m_w = 0.0f; s_w = 1.0f; }
    else {
        m_w = (float)((double)qmax / (double)a_w);
        s_w = (float)((double)a_w / (double)qmax);
    }
    *s_w_out = s_w;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int p = 0; p < Kpad; ++p) {
            int j = src[p];
            int q = 0;
            if (j >= 0) {
                float prod = W[(size_t)n * K + j] * m_w;      /* one IEEE fp32 multiply */
                q = round_clamp(prod, bits);
            }
            Wq_out[(size_t)n * Kpad + p] = (int8_t)q;
        }
    }
    return FQO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Dynamic per-tensor absmax of the flattened activation (Eq. 1's max|X| applied to X').
 * With the equal split each of the n_j copies of channel j holds x/n_j, so
 *     a' = max over slots p of  fl32( max_i |x[i, src[p]]| / (float)rep[p] ),
 * one IEEE fp32 division per slot.
 * ---------------------------------------------------------------------------------------- */
float fqo_act_absmax_dynamic(const float *X, int M, int K, int ldx,
                             const int32_t *src, const int32_t *rep, int Kpad)
{
    float *cmax = (float *)calloc((size_t)K, sizeof(float));
    for (int i = 0; i < M; ++i)
        for (int j = 0; j < K; ++j) {
            float t = fabsf(X[(size_t)i * ldx + j]);
            if (t > cmax[j]) cmax[j] = t;
        }
    float a = 0.0f;
    for (int p = 0; p < Kpad; ++p) {
        int j = src[p];
        if (j < 0) continue;
        float t = cmax[j] / (float)rep[p];
        if (t > a) a = t;
    }
    free(cmax);
    return a;
}

/* ------------------------------------------------------------------------------------------
 * Flatten + quantize the activation (Eq. 3 in the equal-split form, then Eq. 1).
 * Slot p of row i holds x[i, src[p]] / rep[p]; dividing that by s_x = a'/qmax is carried out as
 * one fp32 multiply by m_p = fl32( qmax / (rep[p] * a') ) (formed in float64, rounded once),
 * then round-half-even, then clamp to [qmin, qmax]; padding slots hold 0.
 * a' is the absmax of the flattened tensor: the caller passes either the dynamic value from
 * fqo_act_absmax_dynamic or a static (calibrated) one.  a' = 0 gives all zeros and s_x = 1.
 * ---------------------------------------------------------------------------------------- */
int fqo_flatten_quant_act(const float *X, int M, int K, int ldx,
                          const int32_t *src, const int32_t *rep, int Kpad, int bits,
                          float a_prime, int8_t *Xq_out /* M x Kpad */, float *s_x_out)
{
    if (!X || !src || !rep || !Xq_out || !s_x_out || M <= 0 || K <= 0 || Kpad <= 0) return FQO_ERR_ARG;
    if (bits != 8 && bits != 4) return FQO_ERR_ARG;
    if (!(a_prime >= 0.0f) || isinf(a_prime)) return FQO_ERR_ARG;
    int qmax = qmax_of(bits);
    *s_x_out = (a_prime == 0.0f) ? 1.0f : (float)((double)a_prime / (double)qmax);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        for (int p = 0; p < Kpad; ++p) {
            int j = src[p];
            int q = 0;
            if (j >= 0 && a_prime != 0.0f) {
                float m = (float)((double)qmax / ((double)rep[p] * (double)a_prime));
                float prod = X[(size_t)i * ldx + j] * m;      /* one IEEE fp32 multiply */
                q = round_clamp(prod, bits);
            }
            Xq_out[(size_t)i * Kpad + p] = (int8_t)q;
        }
    }
    return FQO_OK;
}

/* The unquantized flatten, float64, for the invariants (X'W' = XW, max|x'| <= T):
 * x'[i,p] = x[i,src[p]] / rep[p]; padding 0. */
void fqo_flatten_float(const float *X, int M, int K, int ldx, const int32_t *src,
                       const int32_t *rep, int Kpad, double *Xf_out /* M x Kpad */)
{
    (void)K;
    for (int i = 0; i < M; ++i)
        for (int p = 0; p < Kpad; ++p) {
            int j = src[p];
            Xf_out[(size_t)i * Kpad + p] = (j >= 0) ? (double)X[(size_t)i * ldx + j] / (double)rep[p] : 0.0;
        }
}

/* The unquantized weight repeat (Eq. 4), float64: W'[n,p] = W[n,src[p]]; padding 0. */
void fqo_repeat_weights_float(const float *W, int N, int K, const int32_t *src, int Kpad,
                              double *Wf_out /* N x Kpad */)
{
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < Kpad; ++p) {
            int j = src[p];
            Wf_out[(size_t)n * Kpad + p] = (j >= 0) ? (double)W[(size_t)n * K + j] : 0.0;
        }
}

/* The paper's own per-element split (Eq. 3 as printed, extended to negative values by
 * working on |x| and restoring the sign): slot e of channel j (e = 0 is the original
 * position, e >= 1 the appended copies in order) receives sign(x) * clamp(|x| - e*T, 0, T),
 * i.e. floor(|x|/T) slots hold T and the next one holds the remainder.  float64.
 * Used by the tests to show that both split rules satisfy the same two invariants. */
void fqo_flatten_float_peel(const float *X, int M, int K, int ldx, const int32_t *src,
                            int Kpad, double T, double *Xf_out /* M x Kpad */)
{
    int *seen = (int *)malloc((size_t)K * sizeof(int));
    for (int i = 0; i < M; ++i) {
        memset(seen, 0, (size_t)K * sizeof(int));
        /* e for slot p = number of earlier slots with the same source, taking the original
         * slot (p < K) first and appended slots after it in increasing p */
        for (int p = 0; p < Kpad; ++p) {
            int j = src[p];
            double v = 0.0;
            if (j >= 0) {
                int e = seen[j]++;
                double x = (double)X[(size_t)i * ldx + j];
                double mag = fabs(x) - (double)e * T;
                if (mag < 0.0) mag = 0.0;
                if (mag > T) mag = T;
                v = (x < 0.0) ? -mag : mag;
            }
            Xf_out[(size_t)i * Kpad + p] = v;
        }
    }
    free(seen);
}

/* ------------------------------------------------------------------------------------------
 * INT4 storage: two's-complement nibbles, two per byte along the flattened-channel axis,
 * even index in the low nibble.  (The paper leaves the storage format to its GEMM library;
 * this is the reading taken.)
 * ---------------------------------------------------------------------------------------- */
int fqo_pack_i4(const int8_t *q, long long rows, int Kpad, uint8_t *out /* rows x Kpad/2 */)
{
    if (!q || !out || Kpad <= 0 || (Kpad & 1)) return FQO_ERR_ARG;
    for (long long r = 0; r < rows; ++r)
        for (int b = 0; b < Kpad / 2; ++b) {
            int lo = q[r * Kpad + 2 * b], hi = q[r * Kpad + 2 * b + 1];
            if (lo < -8 || lo > 7 || hi < -8 || hi > 7) return FQO_ERR_ARG;
            out[r * (Kpad / 2) + b] = (uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));
        }
    return FQO_OK;
}

int fqo_unpack_i4(const uint8_t *packed, long long rows, int Kpad, int8_t *q /* rows x Kpad */)
{
    if (!q || !packed || Kpad <= 0 || (Kpad & 1)) return FQO_ERR_ARG;
    for (long long r = 0; r < rows; ++r)
        for (int b = 0; b < Kpad / 2; ++b) {
            int byte = packed[r * (Kpad / 2) + b];
            int lo = byte & 0xF, hi = (byte >> 4) & 0xF;
            q[r * Kpad + 2 * b] = (int8_t)(lo >= 8 ? lo - 16 : lo);
            q[r * Kpad + 2 * b + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
        }
    return FQO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Integer GEMM with int32 accumulation: acc[i,n] = sum_p Xq[i,p] * Wq[n,p].
 * Rows [row0, row0+rows) of the M x N result are produced (rows = M, row0 = 0 for all of it),
 * so that a bounded sample of a large problem can be computed.  acc_out holds `rows` rows.
 * The running sum is kept in int64 and checked against the int32 range.
 * ---------------------------------------------------------------------------------------- */
int fqo_gemm_i32(const int8_t *Xq, const int8_t *Wq, int M, int N, int Kpad,
                 int row0, int rows, int32_t *acc_out /* rows x N */)
{
    if (!Xq || !Wq || !acc_out || M <= 0 || N <= 0 || Kpad <= 0) return FQO_ERR_ARG;
    if (row0 < 0 || rows < 0 || row0 + rows > M) return FQO_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int i = 0; i < rows; ++i) {
        const int8_t *x = Xq + (size_t)(row0 + i) * Kpad;
        for (int n = 0; n < N; ++n) {
            const int8_t *w = Wq + (size_t)n * Kpad;
            int64_t s = 0;
            for (int p = 0; p < Kpad; ++p) s += (int32_t)x[p] * (int32_t)w[p];
            if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
            acc_out[(size_t)i * N + n] = (int32_t)s;
        }
    }
    return bad ? FQO_ERR_OVERFLOW : FQO_OK;
}

/* One accumulator, for sampled checks at full size. */
int32_t fqo_dot_i32(const int8_t *x, const int8_t *w, int Kpad)
{
    int64_t s = 0;
    for (int p = 0; p < Kpad; ++p) s += (int32_t)x[p] * (int32_t)w[p];
    return (int32_t)s;
}

/* Dequantize (the inverse of Eq. 1 applied to the product): y = acc * s_x * s_w, float64. */
void fqo_dequant(const int32_t *acc, long long count, float s_x, float s_w, double *y_out)
{
    for (long long i = 0; i < count; ++i)
        y_out[i] = (double)acc[i] * (double)s_x * (double)s_w;
}

/* Unquantized reference product Y = X W^T in float64 (what the layer approximates). */
void fqo_linear_f64(const float *X, const float *W, int M, int N, int K, int ldx, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i)
        for (int n = 0; n < N; ++n) {
            double s = 0.0;
            for (int j = 0; j < K; ++j) s += (double)X[(size_t)i * ldx + j] * (double)W[(size_t)n * K + j];
            Y[(size_t)i * N + n] = s;
        }
}

/* Product of two float64 row-major operands sharing their contiguous axis:
 * Y[i,n] = sum_p A[i,p] * B[n,p].  Used for X'W' in the identity test. */
void fqo_matmul_nt_f64(const double *A, const double *B, int M, int N, int Kpad, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i)
        for (int n = 0; n < N; ++n) {
            double s = 0.0;
            for (int p = 0; p < Kpad; ++p) s += A[(size_t)i * Kpad + p] * B[(size_t)n * Kpad + p];
            Y[(size_t)i * N + n] = s;
        }
}

/* ------------------------------------------------------------------------------------------
 * The whole layer on rows [row0, row0+rows): dynamic or static activation scale (a_static < 0
 * selects dynamic), flatten-quantize, (pack/unpack for k = 4), integer GEMM, dequantize.
 * Wq / s_w come from fqo_flatten_weights.  The dynamic absmax is always taken over ALL M rows
 * (it is a per-tensor quantity) even when only a sample of rows is multiplied.
 * Outputs: acc (rows x N int32), y (rows x N float64), s_x.
 * ---------------------------------------------------------------------------------------- */
int fqo_linear(const float *X, int M, int K, int ldx, const int32_t *src, const int32_t *rep,
               int Kpad, const int8_t *Wq, float s_w, int N, int bits, float a_static,
               int row0, int rows, int32_t *acc_out, double *y_out, float *s_x_out)
{
    if (row0 < 0 || rows <= 0 || row0 + rows > M) return FQO_ERR_ARG;
    float a_prime = (a_static >= 0.0f) ? a_static
                                       : fqo_act_absmax_dynamic(X, M, K, ldx, src, rep, Kpad);
    int8_t *Xq = (int8_t *)malloc((size_t)rows * Kpad);
    if (!Xq) return FQO_ERR_ARG;
    int rc = fqo_flatten_quant_act(X + (size_t)row0 * ldx, rows, K, ldx, src, rep, Kpad, bits,
                                   a_prime, Xq, s_x_out);
    if (rc == FQO_OK && bits == 4) {
        /* through the packed representation and back, as the stored tensors are */
        uint8_t *pk = (uint8_t *)malloc((size_t)rows * (Kpad / 2));
        rc = fqo_pack_i4(Xq, rows, Kpad, pk);
        if (rc == FQO_OK) rc = fqo_unpack_i4(pk, rows, Kpad, Xq);
        free(pk);
    }
    if (rc == FQO_OK) rc = fqo_gemm_i32(Xq, Wq, rows, N, Kpad, 0, rows, acc_out);
    if (rc == FQO_OK && y_out) fqo_dequant(acc_out, (long long)rows * N, *s_x_out, s_w, y_out);
    free(Xq);
    return rc;
}

/* ==========================================================================================
 * Offline policy helpers of the paper (host side; they only produce the hot path's inputs).
 * ======================================================================================== */

/* linear-interpolation quantile of a sorted array (position q*(n-1)); the paper only says the
 * quartiles split off the lowest and highest 25 %; this is the reading taken. */
static double quantile_sorted(const double *v, int n, double q)
{
    double pos = q * (double)(n - 1);
    int lo = (int)floor(pos);
    int hi = lo + 1 < n ? lo + 1 : lo;
    double frac = pos - (double)lo;
    return v[lo] + (v[hi] - v[lo]) * frac;
}
static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

/* ------------------------------------------------------------------------------------------
 * Truncation threshold (Sec. 4.2, Eq. 6-7): the channel maxima are clipped to the box-plot
 * fences [Q1 - 1.5 IQR, Q3 + 1.5 IQR] and T = beta * mean(clipped maxima).  float64, result
 * rounded to fp32.
 * ---------------------------------------------------------------------------------------- */
int fqo_threshold_boxplot(const float *chmax, int K, float beta, float *T_out)
{
    if (!chmax || !T_out || K <= 0 || !(beta > 0.0f) || isinf(beta)) return FQO_ERR_ARG;
    double *v = (double *)malloc((size_t)K * sizeof(double));
    for (int j = 0; j < K; ++j) {
        if (!(chmax[j] >= 0.0f) || isinf(chmax[j])) { free(v); return FQO_ERR_ARG; }
        v[j] = (double)chmax[j];
    }
    qsort(v, (size_t)K, sizeof(double), cmp_double);
    double q1 = quantile_sorted(v, K, 0.25), q3 = quantile_sorted(v, K, 0.75);
    double iqr = q3 - q1, lo = q1 - 1.5 * iqr, hi = q3 + 1.5 * iqr;
    double sum = 0.0;
    for (int j = 0; j < K; ++j) {
        double c = v[j];
        if (c < lo) c = lo;
        if (c > hi) c = hi;
        sum += c;
    }
    free(v);
    *T_out = (float)((double)beta * (sum / (double)K));
    return FQO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Channel smoothing factors (Sec. 4.2, Eq. 5):
 *   s_j = Sigmoid((max|X_j| - mu) / sigma)^alpha / Sigmoid((max|W_j| - mu) / sigma)^(1 - alpha)
 * with mu and sigma the mean and (population) standard deviation of the activation channel
 * maxima, as printed (the weight term is normalized with the same mu and sigma).
 * The smoothed operands are X diag(s)^-1 and diag(s) W.  sigma = 0 (all maxima equal) gives
 * s_j = 1.  float64, results rounded to fp32.
 * ---------------------------------------------------------------------------------------- */
int fqo_smooth_scales(const float *chmax_x, const float *chmax_w, int K, float alpha, float *s_out)
{
    if (!chmax_x || !chmax_w || !s_out || K <= 0 || !(alpha >= 0.0f) || !(alpha <= 1.0f)) return FQO_ERR_ARG;
    double mu = 0.0;
    for (int j = 0; j < K; ++j) mu += (double)chmax_x[j];
    mu /= (double)K;
    double var = 0.0;
    for (int j = 0; j < K; ++j) {
        double d = (double)chmax_x[j] - mu;
        var += d * d;
    }
    double sigma = sqrt(var / (double)K);
    for (int j = 0; j < K; ++j) {
        if (sigma == 0.0) { s_out[j] = 1.0f; continue; }
        double zx = ((double)chmax_x[j] - mu) / sigma, zw = ((double)chmax_w[j] - mu) / sigma;
        double sx = 1.0 / (1.0 + exp(-zx)), sw = 1.0 / (1.0 + exp(-zw));
        s_out[j] = (float)(pow(sx, (double)alpha) / pow(sw, 1.0 - (double)alpha));
    }
    return FQO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Calibration statistic (Sec. 4.2: the channel maxima that Eq. 2, Eq. 5 and Eq. 6 consume):
 *   chmax[j] = max(prev[j], max_i |x[i, j]|), prev = 0 when accumulate == 0, else the values
 * chmax holds on entry (a running maximum over calibration batches).
 * ---------------------------------------------------------------------------------------- */
int fqo_channel_absmax(const float *X, int M, int K, int ldx, int accumulate, float *chmax)
{
    if (!X || !chmax || M <= 0 || K <= 0 || ldx < K) return FQO_ERR_ARG;
    for (int j = 0; j < K; ++j) {
        float m = accumulate ? chmax[j] : 0.0f;
        for (int i = 0; i < M; ++i) {
            float t = fabsf(X[(size_t)i * ldx + j]);
            if (t > m) m = t;
        }
        chmax[j] = m;
    }
    return FQO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Batched integer matrix product (Sec. 5.1, the second quantized operator: the BMM of attention):
 *   acc[b, i, n] = sum_p Aq[b, i, p] * Bq[b, n, p],  b < batch, dense [batch, M, Kpad] and
 * [batch, N, Kpad] operands, int32 result (int64 running sum checked against the int32 range).
 * The paper gives no further detail; per-tensor scales apply to the whole batched tensor, so the
 * dequantized value is fqo_dequant of this.
 * ---------------------------------------------------------------------------------------- */
int fqo_bmm_i32(const int8_t *Aq, const int8_t *Bq, int batch, int M, int N, int Kpad, int32_t *acc_out)
{
    if (!Aq || !Bq || !acc_out || batch <= 0 || M <= 0 || N <= 0 || Kpad <= 0) return FQO_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int b = 0; b < batch; ++b)
        for (int i = 0; i < M; ++i)
            for (int n = 0; n < N; ++n) {
                const int8_t *x = Aq + ((size_t)b * M + i) * Kpad;
                const int8_t *w = Bq + ((size_t)b * N + n) * Kpad;
                int64_t s = 0;
                for (int p = 0; p < Kpad; ++p) s += (int32_t)x[p] * (int32_t)w[p];
                if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
                acc_out[((size_t)b * M + i) * N + n] = (int32_t)s;
            }
    return bad ? FQO_ERR_OVERFLOW : FQO_OK;
}

/* ==========================================================================================
 * The printed split of Eq. 3 ("peel") and flattening of the weights' own large channels
 * (Sec. 4.1, last paragraph).
 * ======================================================================================== */

/* ------------------------------------------------------------------------------------------
 * Two-sided plan.  Channel j is flattened on the activation side into nx_j = max(1,
 * ceil(max|X_j| / T_x)) shares (Eq. 2, reading as in fqo_plan) and, when chmax_w is given, on
 * the weight side into nw_j = max(1, ceil(max|W_j| / T_w)) shares (Sec. 4.1: the same
 * construction applied to the weights, the activation channel being the repeated one).  With
 * equal shares x/nx and w/nw the product x*w is recovered as the sum over nx*nw slots, so
 * channel j occupies c_j = nx_j * nw_j slots: index j and c_j - 1 appended slots, channels in
 * increasing j (Eq. 3's index rule).  Per slot: src, rep_x = nx, rep_w = nw, ord = the slot's
 * ordinal among its channel's slots (0 = the original position).  Padding: -1, 0, 0, 0.
 * chmax_w == NULL means no weight-side flattening (nw = 1); then src / rep_x equal fqo_plan's.
 * ---------------------------------------------------------------------------------------- */
int fqo_plan_xw(const float *chmax_x, float T_x, const float *chmax_w, float T_w, int K, int align,
                int32_t *src, int32_t *rep_x, int32_t *rep_w, int32_t *ord, int cap,
                int *Kprime_out, int *Kpad_out)
{
    if (!chmax_x || K <= 0 || align <= 0 || !(T_x > 0.0f) || isinf(T_x)) return FQO_ERR_ARG;
    if (chmax_w && (!(T_w > 0.0f) || isinf(T_w))) return FQO_ERR_ARG;
    long long total = 0;
    for (int j = 0; j < K; ++j) {
        if (!(chmax_x[j] >= 0.0f) || isinf(chmax_x[j])) return FQO_ERR_ARG;
        long long nx = (long long)ceil((double)chmax_x[j] / (double)T_x), nw = 1;
        if (nx < 1) nx = 1;
        if (chmax_w) {
            if (!(chmax_w[j] >= 0.0f) || isinf(chmax_w[j])) return FQO_ERR_ARG;
            nw = (long long)ceil((double)chmax_w[j] / (double)T_w);
            if (nw < 1) nw = 1;
        }
        if (nx > 0x3fffffff || nw > 0x3fffffff) return FQO_ERR_OVERFLOW;
        total += nx * nw;
        if (total > 0x3fffffff) return FQO_ERR_OVERFLOW;
    }
    long long Kpad = (total + align - 1) / align * align;
    if (Kprime_out) *Kprime_out = (int)total;
    if (Kpad_out) *Kpad_out = (int)Kpad;
    if (cap == 0) return FQO_OK;
    if (!src || !rep_x) return FQO_ERR_ARG;
    if (cap < Kpad) return FQO_ERR_CAP;
    int next = K;
    for (int j = 0; j < K; ++j) {
        int nx = (int)ceil((double)chmax_x[j] / (double)T_x), nw = 1;
        if (nx < 1) nx = 1;
        if (chmax_w) {
            nw = (int)ceil((double)chmax_w[j] / (double)T_w);
            if (nw < 1) nw = 1;
        }
        for (int e = 0; e < nx * nw; ++e) {
            int p = (e == 0) ? j : next++;
            src[p] = j;
            rep_x[p] = nx;
            if (rep_w) rep_w[p] = nw;
            if (ord) ord[p] = e;
        }
    }
    for (int p = next; p < (int)Kpad; ++p) {
        src[p] = -1;
        rep_x[p] = 0;
        if (rep_w) rep_w[p] = 0;
        if (ord) ord[p] = 0;
    }
    return FQO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Weights with their own channels flattened (Sec. 4.1, last paragraph; Eq. 1): slot p of row n
 * holds W[n, src[p]] / rep_w[p]; per-tensor absmax of that tensor
 *   a_w = max_p fl32( max_n |W[n, src[p]]| / (float)rep_w[p] ),
 * s_w = fl32(a_w / qmax), multiplier m_p = fl32(qmax / (rep_w[p] * a_w)) (float64 quotient), one
 * fp32 multiply, round-half-even, clamp.  The same arithmetic as the activation's equal split,
 * applied to the N x K weight array.
 * ---------------------------------------------------------------------------------------- */
int fqo_flatten_weights_split(const float *W, int N, int K, const int32_t *src, const int32_t *rep_w,
                              int Kpad, int bits, int8_t *Wq_out, float *s_w_out)
{
    if (!W || !src || !rep_w || !Wq_out || !s_w_out || N <= 0 || K <= 0 || Kpad <= 0) return FQO_ERR_ARG;
    float a_w = fqo_act_absmax_dynamic(W, N, K, K, src, rep_w, Kpad);
    return fqo_flatten_quant_act(W, N, K, K, src, rep_w, Kpad, bits, a_w, Wq_out, s_w_out);
}

/* ------------------------------------------------------------------------------------------
 * Eq. 3 as printed, quantized (Eq. 1).  The slot with ordinal e of channel j (e = 0 the
 * original position) holds  v = sign(x) * min(max(|x| - e*T, 0), T):  floor(|x|/T) slots of T,
 * then the remainder, then zeros (the paper prints the positive case; negative values are
 * treated through |x|).  All in fp32, in this order:
 *   t = fl32((float)e * T);  mag = fl32(|x| - t) clamped to [0, T];  v = +-mag;
 *   q = clamp(rne(fl32(v * m)), qmin, qmax),  m = fl32(qmax / a')  (float64 quotient).
 * a' is the absmax of the flattened tensor: at most T by construction; the caller passes T
 * (static, the paper's setting) or fqo_act_absmax_peel's value.  s_x = fl32(a' / qmax);
 * a' = 0 gives zeros and s_x = 1.  Weights are plainly repeated (Eq. 4) for this split.
 * ---------------------------------------------------------------------------------------- */
float fqo_act_absmax_peel(const float *X, int M, int K, int ldx, float T)
{
    float a = 0.0f;
    for (int i = 0; i < M; ++i)
        for (int j = 0; j < K; ++j) {
            float t = fabsf(X[(size_t)i * ldx + j]);
            if (t > a) a = t;
        }
    return a > T ? T : a;
}

int fqo_flatten_quant_act_peel(const float *X, int M, int K, int ldx, const int32_t *src,
                               const int32_t *ord, int Kpad, int bits, float T, float a_prime,
                               int8_t *Xq_out, float *s_x_out)
{
    if (!X || !src || !ord || !Xq_out || !s_x_out || M <= 0 || K <= 0 || Kpad <= 0) return FQO_ERR_ARG;
    if (bits != 8 && bits != 4) return FQO_ERR_ARG;
    if (!(T > 0.0f) || isinf(T) || !(a_prime >= 0.0f) || isinf(a_prime)) return FQO_ERR_ARG;
    int qmax = qmax_of(bits);
    *s_x_out = (a_prime == 0.0f) ? 1.0f : (float)((double)a_prime / (double)qmax);
    float m = (a_prime == 0.0f) ? 0.0f : (float)((double)qmax / (double)a_prime);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i)
        for (int p = 0; p < Kpad; ++p) {
            int j = src[p], q = 0;
            if (j >= 0) {
                float x = X[(size_t)i * ldx + j];
                float t = (float)ord[p] * T;
                float mag = fabsf(x) - t;
                if (mag < 0.0f) mag = 0.0f;
                if (mag > T) mag = T;
                float v = (x < 0.0f) ? -mag : mag;
                q = round_clamp(v * m, bits);
            }
            Xq_out[(size_t)i * Kpad + p] = (int8_t)q;
        }
    return FQO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Dequantize with the layer's bias: y[i, n] = acc[i, n] * s_x * s_w + bias[n], float64.  (The
 * paper replaces OPT's linear layers, which carry a bias, by quantized ones without spelling the
 * bias out; reading taken: it is added in floating point after the dequantization.)
 * ---------------------------------------------------------------------------------------- */
void fqo_dequant_bias(const int32_t *acc, int rows, int N, float s_x, float s_w, const float *bias,
                      double *y_out)
{
    for (int i = 0; i < rows; ++i)
        for (int n = 0; n < N; ++n)
            y_out[(size_t)i * N + n] = (double)acc[(size_t)i * N + n] * (double)s_x * (double)s_w + (double)bias[n];
}

/* ------------------------------------------------------------------------------------------
 * Second storage format of the 4-bit quantized tensors: each value q in [-8, 7] is stored as the
 * 6-bit floating-point code E3M2 (1 sign, 3 exponent bits with bias 3, 2 mantissa bits; value
 * (-1)^s * 2^(e-3) * (1 + m/4) for e >= 1, (-1)^s * 2^-2 * (m/4) for e = 0; no infinities or NaNs)
 * that represents the integer q exactly, 6 bits per slot, packed as a little-endian bit stream
 * along the flattened-channel axis (slot p occupies bits [6p, 6p+6) of its row; 16 slots = 12
 * bytes).  The paper leaves the storage of its 4-bit operands to its GEMM library; this format is
 * what the 6-bit matrix instructions of the target consume.  Kpad must be a multiple of 16.
 * ---------------------------------------------------------------------------------------- */
static int e3m2_code(int q)
{
    /* |q| = 0..8 as 2^(e-3) * (1 + m/4): 1 = 2^0, 2, 3 = 2 * 1.5, 4, 5 = 4 * 1.25, 6, 7, 8 = 2^3 */
    int a = q < 0 ? -q : q, e = 0, m = 0;
    if (a >= 1) {
        e = 3;
        while ((2 << (e - 3)) <= a) ++e;             /* 2^(e-3) <= a < 2^(e-2) */
        m = (4 * a) / (1 << (e - 3)) - 4;            /* a = 2^(e-3) * (1 + m/4), exact for a <= 8 */
    }
    return ((q < 0) ? 0x20 : 0) | (e << 2) | m;
}

int fqo_pack_e3m2(const int8_t *q, long long rows, int Kpad, uint8_t *out /* rows x Kpad*3/4 */)
{
    if (!q || !out || rows <= 0 || Kpad <= 0 || Kpad % 16) return FQO_ERR_ARG;
    long long rb = (long long)Kpad * 3 / 4;
    memset(out, 0, (size_t)(rows * rb));
    for (long long r = 0; r < rows; ++r)
        for (int p = 0; p < Kpad; ++p) {
            int v = q[r * Kpad + p];
            if (v < -8 || v > 8) return FQO_ERR_ARG;
            int c = e3m2_code(v);
            long long bit = 6LL * p;
            for (int b = 0; b < 6; ++b)
                if ((c >> b) & 1) out[r * rb + (bit + b) / 8] |= (uint8_t)(1u << ((bit + b) % 8));
        }
    return FQO_OK;
}

/* Decodes by the format's definition (not by inverting the table above). */
int fqo_unpack_e3m2(const uint8_t *packed, long long rows, int Kpad, double *out /* rows x Kpad */)
{
    if (!packed || !out || rows <= 0 || Kpad <= 0 || Kpad % 16) return FQO_ERR_ARG;
    long long rb = (long long)Kpad * 3 / 4;
    for (long long r = 0; r < rows; ++r)
        for (int p = 0; p < Kpad; ++p) {
            int c = 0;
            long long bit = 6LL * p;
            for (int b = 0; b < 6; ++b)
                if ((packed[r * rb + (bit + b) / 8] >> ((bit + b) % 8)) & 1) c |= 1 << b;
            int sgn = c >> 5, e = (c >> 2) & 7, m = c & 3;
            double v = (e == 0) ? 0.25 * (m / 4.0) : ldexp(1.0 + m / 4.0, e - 3);
            out[r * Kpad + p] = sgn ? -v : v;
        }
    return FQO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Dequantize to the layer's output type (the inverse of Eq. 1 applied to the product, Sec. 5.1:
 * the quantized layer hands a 16-bit floating-point tensor to the next operator).  The value is
 * defined in fp32, every step rounded once to nearest-even:
 *     f = fl32( fl32(acc) * fl32(s_x * s_w) )            fl32(acc): the int32 rounded to fp32
 *     f = fl32( f + bias[n] )                            only when a bias is given
 *     y = f rounded to the output type: fp32 (unchanged), IEEE half, or bfloat16.
 * The two 16-bit roundings are written out on the bit pattern of f (no compiler conversion is
 * relied on).  out_dtype: 0 = fp32 (out is float*), 1 = half, 2 = bfloat16 (out is uint16_t* and
 * receives the bit patterns).
 * ---------------------------------------------------------------------------------------- */
static uint32_t bits_of(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

/* fp32 -> bfloat16 (1 sign, 8 exponent, 7 fraction bits): keep the top 16 bits, round to nearest on
 * the 16 dropped bits, ties to the even kept pattern.  The carry of a round-up runs into the
 * exponent, which is what rounding up to the next binade (or to infinity) means. */
static uint16_t round_to_bf16(float f)
{
    uint32_t u = bits_of(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);   /* NaN stays NaN */
    uint32_t kept = u >> 16, dropped = u & 0xffffu;
    if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u))) kept += 1;
    return (uint16_t)kept;
}

/* fp32 -> IEEE half (1 sign, 5 exponent bits with bias 15, 10 fraction bits), nearest-even,
 * through the value: |f| = m * 2^e is placed on half's grid (spacing 2^(E-10) in the binade 2^E,
 * E >= -14; spacing 2^-24 below 2^-14) with rint (ties to even in the default rounding mode). */
static uint16_t round_to_f16(float f)
{
    uint32_t u = bits_of(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t mag = u & 0x7fffffffu;
    if (mag > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);        /* NaN */
    if (mag == 0x7f800000u) return (uint16_t)(sign | 0x7c00u);       /* infinity */
    double a = fabs((double)f);
    if (a == 0.0) return sign;
    int E;
    (void)frexp(a, &E);                 /* a = x * 2^E with 0.5 <= x < 1, so a lies in [2^(E-1), 2^E) */
    int binade = E - 1;
    if (binade < -14) binade = -14;     /* subnormal halves share the spacing of the lowest binade */
    double spacing = ldexp(1.0, binade - 10);
    double steps = rint(a / spacing);   /* exact division by a power of two; ties to even */
    double r = steps * spacing;
    if (r >= 65520.0) return (uint16_t)(sign | 0x7c00u);             /* beyond the largest half: infinity */
    /* r is on the grid: rebuild its pattern */
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)steps);               /* subnormal: steps of 2^-24 */
    int E2;
    (void)frexp(r, &E2);
    int e = E2 - 1;                                                   /* r in [2^e, 2^(e+1)) */
    uint32_t frac = (uint32_t)(r / ldexp(1.0, e - 10)) - 1024u;       /* 10 fraction bits */
    return (uint16_t)(sign | (uint32_t)((e + 15) << 10) | frac);
}

int fqo_dequant_out(const int32_t *acc, int rows, int N, float s_x, float s_w, const float *bias /* or NULL */,
                    int out_dtype, void *out)
{
    if (!acc || !out || rows <= 0 || N <= 0 || out_dtype < 0 || out_dtype > 2) return FQO_ERR_ARG;
    const float scale = s_x * s_w;                       /* one fp32 multiply */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < rows; ++i)
        for (int n = 0; n < N; ++n) {
            size_t at = (size_t)i * N + n;
            float a = (float)acc[at];                    /* int32 -> fp32, nearest-even */
            float f = a * scale;                         /* one fp32 multiply (the build forbids contraction) */
            if (bias) f = f + bias[n];                   /* one fp32 add */
            if (out_dtype == 0) ((float *)out)[at] = f;
            else if (out_dtype == 1) ((uint16_t *)out)[at] = round_to_f16(f);
            else ((uint16_t *)out)[at] = round_to_bf16(f);
        }
    return FQO_OK;
}
