/* Walks the CPU oracle through small ragged cases with every buffer allocated at its exact size, for a build with
 * -fsanitize=address,undefined (tests/test_oracle_sanitized.py compiles this file together with oracle/fq_oracle.c
 * and runs it): an access outside a buffer, a signed overflow or a misaligned access in the oracle ends the run
 * with a sanitizer report.  Values are not checked here (the pins in tests/test_oracle_*.py do that); only the
 * return codes are.  Test infrastructure, CPU only. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int fqo_plan(const float *chmax, int K, float T, int align, int32_t *src, int32_t *rep, int cap, int *Kprime_out, int *Kpad_out);
int fqo_flatten_weights(const float *W, int N, int K, const int32_t *src, int Kpad, int bits, int8_t *Wq_out, float *s_w_out);
float fqo_act_absmax_dynamic(const float *X, int M, int K, int ldx, const int32_t *src, const int32_t *rep, int Kpad);
int fqo_flatten_quant_act(const float *X, int M, int K, int ldx, const int32_t *src, const int32_t *rep, int Kpad, int bits,
                          float a_prime, int8_t *Xq_out, float *s_x_out);
int fqo_pack_i4(const int8_t *q, long long rows, int Kpad, uint8_t *out);
int fqo_unpack_i4(const uint8_t *packed, long long rows, int Kpad, int8_t *q);
int fqo_pack_e3m2(const int8_t *q, long long rows, int Kpad, uint8_t *out);
int fqo_unpack_e3m2(const uint8_t *packed, long long rows, int Kpad, double *out);
int fqo_gemm_i32(const int8_t *Xq, const int8_t *Wq, int M, int N, int Kpad, int row0, int rows, int32_t *acc_out);
int fqo_linear(const float *X, int M, int K, int ldx, const int32_t *src, const int32_t *rep, int Kpad, const int8_t *Wq,
               float s_w, int N, int bits, float a_static, int row0, int rows, int32_t *acc_out, double *y_out, float *s_x_out);
int fqo_threshold_boxplot(const float *chmax, int K, float beta, float *T_out);
int fqo_smooth_scales(const float *chmax_x, const float *chmax_w, int K, float alpha, float *s_out);
int fqo_channel_absmax(const float *X, int M, int K, int ldx, int accumulate, float *chmax);
int fqo_bmm_i32(const int8_t *Aq, const int8_t *Bq, int batch, int M, int N, int Kpad, int32_t *acc_out);
int fqo_plan_xw(const float *chmax_x, float T_x, const float *chmax_w, float T_w, int K, int align, int32_t *src,
                int32_t *rep_x, int32_t *rep_w, int32_t *ord, int cap, int *Kprime_out, int *Kpad_out);
int fqo_flatten_weights_split(const float *W, int N, int K, const int32_t *src, const int32_t *rep_w, int Kpad, int bits,
                              int8_t *Wq_out, float *s_w_out);
float fqo_act_absmax_peel(const float *X, int M, int K, int ldx, float T);
int fqo_flatten_quant_act_peel(const float *X, int M, int K, int ldx, const int32_t *src, const int32_t *ord, int Kpad,
                               int bits, float T, float a_prime, int8_t *Xq_out, float *s_x_out);
void fqo_dequant_bias(const int32_t *acc, int rows, int N, float s_x, float s_w, const float *bias, double *y_out);
int fqo_dequant_out(const int32_t *acc, int rows, int N, float s_x, float s_w, const float *bias, int out_dtype, void *out);

static uint64_t state = 0x9e3779b97f4a7c15ull;
static double uniform(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0;
}
static float *floats(long long n, double scale)
{
    float *p = (float *)malloc((size_t)n * sizeof(float));
    for (long long i = 0; i < n; ++i) p[i] = (float)((uniform() * 2.0 - 1.0) * scale);
    return p;
}
#define CHECK(call)                                                        \
    do {                                                                   \
        int rc_ = (call);                                                  \
        if (rc_ != 0) {                                                    \
            fprintf(stderr, "%s -> %d (case %d)\n", #call, rc_, case_no);  \
            return 1;                                                      \
        }                                                                  \
    } while (0)

static int one_case(int case_no, int M, int K, int N, int align, int bits)
{
    const int ldx = K + (case_no % 3);                       /* padded rows now and then */
    float *X = floats((long long)M * ldx, 1.0), *W = floats((long long)N * K, 0.1);
    for (int i = 0; i < M; ++i) X[(long long)i * ldx + (case_no % K)] *= 40.0f;       /* an outlier channel */
    float *chmax = (float *)malloc((size_t)K * sizeof(float)), *chw = (float *)malloc((size_t)K * sizeof(float));
    CHECK(fqo_channel_absmax(X, M, K, ldx, 0, chmax));
    CHECK(fqo_channel_absmax(X, M, K, ldx, 1, chmax));
    CHECK(fqo_channel_absmax(W, N, K, K, 0, chw));
    float T = 0.0f, *s = (float *)malloc((size_t)K * sizeof(float));
    CHECK(fqo_threshold_boxplot(chmax, K, 1.3f, &T));
    CHECK(fqo_smooth_scales(chmax, chw, K, 0.5f, s));
    if (!(T > 0.0f)) T = 1.0f;
    int Kp = 0, Kpad = 0;
    CHECK(fqo_plan(chmax, K, T, align, NULL, NULL, 0, &Kp, &Kpad));
    int32_t *src = (int32_t *)malloc((size_t)Kpad * 4), *rep = (int32_t *)malloc((size_t)Kpad * 4);
    CHECK(fqo_plan(chmax, K, T, align, src, rep, Kpad, &Kp, &Kpad));
    int8_t *Wq = (int8_t *)malloc((size_t)N * Kpad), *Xq = (int8_t *)malloc((size_t)M * Kpad);
    float s_w = 0, s_x = 0;
    CHECK(fqo_flatten_weights(W, N, K, src, Kpad, bits, Wq, &s_w));
    const float a = fqo_act_absmax_dynamic(X, M, K, ldx, src, rep, Kpad);
    CHECK(fqo_flatten_quant_act(X, M, K, ldx, src, rep, Kpad, bits, a > 0 ? a : 1.0f, Xq, &s_x));
    if (bits == 4) {
        uint8_t *pk = (uint8_t *)malloc((size_t)M * Kpad / 2);
        int8_t *back = (int8_t *)malloc((size_t)M * Kpad);
        CHECK(fqo_pack_i4(Xq, M, Kpad, pk));
        CHECK(fqo_unpack_i4(pk, M, Kpad, back));
        free(pk);
        free(back);
        if (Kpad % 4 == 0) {
            uint8_t *e = (uint8_t *)malloc((size_t)M * Kpad / 4 * 3);
            double *d = (double *)malloc((size_t)M * Kpad * sizeof(double));
            CHECK(fqo_pack_e3m2(Xq, M, Kpad, e));
            CHECK(fqo_unpack_e3m2(e, M, Kpad, d));
            free(e);
            free(d);
        }
    }
    const int row0 = M > 2 ? 1 : 0, rows = M - row0;
    int32_t *acc = (int32_t *)malloc((size_t)rows * N * 4);
    CHECK(fqo_gemm_i32(Xq, Wq, M, N, Kpad, row0, rows, acc));
    double *y = (double *)malloc((size_t)rows * N * sizeof(double));
    CHECK(fqo_linear(X, M, K, ldx, src, rep, Kpad, Wq, s_w, N, bits, case_no % 2 ? T : 0.0f, row0, rows, acc, y, &s_x));
    float *bias = floats(N, 2.0);
    fqo_dequant_bias(acc, rows, N, s_x, s_w, bias, y);
    for (int dt = 0; dt < 3; ++dt) {
        void *out = malloc((size_t)rows * N * (dt == 0 ? 4 : 2));
        CHECK(fqo_dequant_out(acc, rows, N, s_x, s_w, dt == 1 ? NULL : bias, dt, out));
        free(out);
    }
    /* two-sided plan, weight split, peel split */
    CHECK(fqo_plan_xw(chmax, T, chw, 0.07f, K, align, NULL, NULL, NULL, NULL, 0, &Kp, &Kpad));
    int32_t *src2 = (int32_t *)malloc((size_t)Kpad * 4), *rx = (int32_t *)malloc((size_t)Kpad * 4),
            *rw = (int32_t *)malloc((size_t)Kpad * 4), *ord = (int32_t *)malloc((size_t)Kpad * 4);
    CHECK(fqo_plan_xw(chmax, T, chw, 0.07f, K, align, src2, rx, rw, ord, Kpad, &Kp, &Kpad));
    int8_t *Wq2 = (int8_t *)malloc((size_t)N * Kpad), *Xq2 = (int8_t *)malloc((size_t)M * Kpad);
    CHECK(fqo_flatten_weights_split(W, N, K, src2, rw, Kpad, bits, Wq2, &s_w));
    CHECK(fqo_plan_xw(chmax, T, NULL, 0.0f, K, align, src2, rx, rw, ord, Kpad, &Kp, &Kpad));
    const float ap = fqo_act_absmax_peel(X, M, K, ldx, T);
    CHECK(fqo_flatten_quant_act_peel(X, M, K, ldx, src2, ord, Kpad, bits, T, ap > 0 ? ap : T, Xq2, &s_x));
    /* batched product */
    int8_t *Aq = (int8_t *)malloc((size_t)3 * M * 32), *Bq = (int8_t *)malloc((size_t)3 * N * 32);
    for (long long i = 0; i < 3LL * M * 32; ++i) Aq[i] = (int8_t)(uniform() * 255.0 - 128.0);
    for (long long i = 0; i < 3LL * N * 32; ++i) Bq[i] = (int8_t)(uniform() * 255.0 - 128.0);
    int32_t *accb = (int32_t *)malloc((size_t)3 * M * N * 4);
    CHECK(fqo_bmm_i32(Aq, Bq, 3, M, N, 32, accb));
    free(X); free(W); free(chmax); free(chw); free(s); free(src); free(rep); free(Wq); free(Xq); free(acc); free(y);
    free(bias); free(src2); free(rx); free(rw); free(ord); free(Wq2); free(Xq2); free(Aq); free(Bq); free(accb);
    return 0;
}

int main(void)
{
    static const int shapes[][5] = {{1, 1, 1, 32, 8},   {3, 5, 2, 32, 4},    {7, 33, 9, 32, 8},   {16, 64, 16, 128, 4},
                                    {5, 100, 3, 64, 8}, {33, 257, 17, 32, 4}, {2, 16, 70, 256, 4}, {64, 96, 5, 32, 8}};
    for (int c = 0; c < (int)(sizeof shapes / sizeof shapes[0]); ++c)
        if (one_case(c, shapes[c][0], shapes[c][1], shapes[c][2], shapes[c][3], shapes[c][4])) return 1;
    puts("oracle walk clean");
    return 0;
}
