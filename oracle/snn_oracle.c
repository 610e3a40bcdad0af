/*
 * CPU oracle for the sub-bit binary 3x3 convolution of "Sub-bit Neural Networks"
 * (arXiv 2110.09195).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition the GPU library is
 * checked against.  It is used by tests/, by __graft_entry__.smoke() and by the
 * cpu_baseline leg of bench.py, and by nothing else.  It shares no code, header, table or
 * helper with the HIP library and is never a fallback for it.
 *
 * What it computes (every function cites the passage it follows):
 *   - Sec. 4.1: a binary 3x3 kernel is one of 512 codes; flatten row-major, read as a
 *     binary number (+1 -> 1, -1 -> 0).  Paper index = code + 1 (all -1 -> 1, all +1 -> 512).
 *   - Sec. 3: a^i = lambda^i . (w_bar (*) a_bar^{i-1}), channel-wise scale lambda (alpha here),
 *     no bias.  The convolution is the usual CNN cross-correlation, 3x3, zero padding 1.
 *   - Sec. 4.2 Eq. 2 / Sec. 4.3 Eq. 5 / Alg. 1 forward: every (c_out, c_in) kernel is the
 *     member of the layer's subset P (the codebook) that its index selects / that is
 *     nearest to the real-valued kernel.
 *   - Sec. 4.5, Fig. 6: the shared ("two-stage") evaluation is a re-use of the same
 *     products, so its result is the direct convolution with the decoded kernels; the
 *     second routine below evaluates it in the two stages the figure shows.
 *
 * Readings where the paper is silent (kept identical in the library's header):
 *   - first flattened tap (top-left) is the most significant of the 9 bits;
 *   - taps outside the image contribute 0 (zero padding), also for +-1 activations;
 *   - sign(x) = +1 for x >= 0 (so +0, -0 -> +1) and -1 otherwise (NaN -> -1);
 *   - arg min over the codebook takes the lowest index among equal scores; scores are
 *     inner products accumulated in fp32, taps in order 0..8, add or subtract only.
 *
 * Pins: tests/test_oracle_*.py (brute force in pure Python, a library cross-correlation,
 * closed forms, the K=512 identity, two-stage == direct, Eq. 1, printed Bit-OPs columns).
 * All functions below are pinned there; none is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int snn_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sec. 4.1: 9-bit code -> +-1 taps, tap t = 3*dy + dx, bit (8 - t), 1 -> +1. */
void snn_oracle_decode(uint16_t code, int8_t w[9])
{
    for (int t = 0; t < 9; ++t)
        w[t] = ((code >> (8 - t)) & 1) ? 1 : -1;
}

/* Output size of a 3x3, pad 1 convolution with the given stride. */
int snn_oracle_out_size(int in, int stride)
{
    return (in - 1) / stride + 1;
}

/* Alg. 1 forward, sign(a^{i-1}): +1 where x >= 0, else -1. */
void snn_oracle_sign(const float *x, int8_t *s, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        s[i] = (x[i] >= 0.0f) ? 1 : -1;
}

/* Row-packed sign bits: out[n][c][h][ceil(W/32)], bit (w % 32) of word (w / 32),
 * 1 <-> +1, unused high bits zero. */
void snn_oracle_pack_rows(const float *x, uint32_t *out, int N, int C, int H, int W)
{
    const int WW = (W + 31) / 32;
    memset(out, 0, (size_t)N * C * H * WW * sizeof(uint32_t));
    for (int64_t r = 0; r < (int64_t)N * C * H; ++r)
        for (int w = 0; w < W; ++w)
            if (x[r * W + w] >= 0.0f)
                out[r * WW + w / 32] |= (uint32_t)1 << (w % 32);
}

/* Channel-packed sign bits: out[n][h][w][ceil(C/32)], bit (c % 32) of word (c / 32). */
void snn_oracle_pack_channels(const float *x, uint32_t *out, int N, int C, int H, int W)
{
    const int CW = (C + 31) / 32;
    memset(out, 0, (size_t)N * H * W * CW * sizeof(uint32_t));
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    if (x[(((int64_t)n * C + c) * H + h) * W + w] >= 0.0f)
                        out[(((int64_t)n * H + h) * W + w) * CW + c / 32] |= (uint32_t)1 << (c % 32);
}

/* Sec. 4.4: the stored layer is (subset, index per kernel); expanding it gives the
 * 9-bit code of every (c_out, c_in) kernel. */
void snn_oracle_expand(const uint16_t *codebook, const uint16_t *idx, int64_t n, uint16_t *codes)
{
    for (int64_t i = 0; i < n; ++i)
        codes[i] = codebook[idx[i]];
}

/*
 * Sec. 3 with +-1 activations (Alg. 1 forward, last line):
 *   S[n,co,ho,wo] = sum_ci sum_dy sum_dx W[co][ci][3dy+dx] * X[n,ci, s*ho+dy-1, s*wo+dx-1],
 *   X = 0 outside the image;  Y = (float)S * alpha[co]  (one fp32 multiply).
 * xs is NCHW int8 in {+1,-1}; codes is [C_out][C_in] 9-bit kernels.  S and Y may be NULL.
 */
void snn_oracle_conv_bin(const int8_t *xs, int N, int C_in, int C_out, int H, int W, int stride,
                         const uint16_t *codes, const float *alpha, int32_t *S, float *Y)
{
    const int Ho = snn_oracle_out_size(H, stride), Wo = snn_oracle_out_size(W, stride);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < C_out; ++co)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    int32_t s = 0;
                    for (int ci = 0; ci < C_in; ++ci) {
                        int8_t k[9];
                        snn_oracle_decode(codes[(int64_t)co * C_in + ci], k);
                        for (int dy = 0; dy < 3; ++dy)
                            for (int dx = 0; dx < 3; ++dx) {
                                const int h = stride * ho + dy - 1, w = stride * wo + dx - 1;
                                if (h < 0 || h >= H || w < 0 || w >= W)
                                    continue;
                                s += k[3 * dy + dx] * xs[(((int64_t)n * C_in + ci) * H + h) * W + w];
                            }
                    }
                    const int64_t o = (((int64_t)n * C_out + co) * Ho + ho) * Wo + wo;
                    if (S)
                        S[o] = s;
                    if (Y) {
                        const float sf = (float)s;
                        Y[o] = sf * alpha[co];
                    }
                }
}

/*
 * Same layer with real-valued activations (the W/A = x/32 rows of Tables 1-2, and the
 * deployment test of Table 4): binary/sub-bit weights, fp32 input.  Accumulated in
 * float64 in the order (ci, dy, dx); Y = (float)(alpha[co] * S).  Sd (float64 sums) may be NULL.
 */
void snn_oracle_conv_f32(const float *x, int N, int C_in, int C_out, int H, int W, int stride,
                         const uint16_t *codes, const float *alpha, double *Sd, float *Y)
{
    const int Ho = snn_oracle_out_size(H, stride), Wo = snn_oracle_out_size(W, stride);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < C_out; ++co)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    double s = 0.0;
                    for (int ci = 0; ci < C_in; ++ci) {
                        int8_t k[9];
                        snn_oracle_decode(codes[(int64_t)co * C_in + ci], k);
                        for (int dy = 0; dy < 3; ++dy)
                            for (int dx = 0; dx < 3; ++dx) {
                                const int h = stride * ho + dy - 1, w = stride * wo + dx - 1;
                                if (h < 0 || h >= H || w < 0 || w >= W)
                                    continue;
                                const double v = (double)x[(((int64_t)n * C_in + ci) * H + h) * W + w];
                                s += (k[3 * dy + dx] > 0) ? v : -v;
                            }
                    }
                    const int64_t o = (((int64_t)n * C_out + co) * Ho + ho) * Wo + wo;
                    if (Sd)
                        Sd[o] = s;
                    if (Y)
                        Y[o] = (float)((double)alpha[co] * s);
                }
}

/*
 * Sec. 4.5 / Fig. 6, evaluated the way the figure draws it, for +-1 activations:
 *   stage 1: T[ci][k][ho][wo] = response of input channel ci to subset kernel k;
 *   stage 2: S[co][ho][wo]    = sum_ci T[ci][ idx[co][ci] ][ho][wo].
 * One image at a time (T is N times smaller that way).  Returns 0, or -1 if the
 * temporary cannot be allocated.
 */
int snn_oracle_two_stage_bin(const int8_t *xs, int N, int C_in, int C_out, int H, int W, int stride,
                             const uint16_t *codebook, int K, const uint16_t *idx,
                             const float *alpha, int32_t *S, float *Y)
{
    const int Ho = snn_oracle_out_size(H, stride), Wo = snn_oracle_out_size(W, stride);
    const int64_t plane = (int64_t)Ho * Wo;
    int32_t *T = (int32_t *)malloc((size_t)C_in * K * plane * sizeof(int32_t));
    if (!T)
        return -1;
    for (int n = 0; n < N; ++n) {
        for (int ci = 0; ci < C_in; ++ci)
            for (int k = 0; k < K; ++k) {
                int8_t kw[9];
                snn_oracle_decode(codebook[k], kw);
                for (int ho = 0; ho < Ho; ++ho)
                    for (int wo = 0; wo < Wo; ++wo) {
                        int32_t r = 0;
                        for (int dy = 0; dy < 3; ++dy)
                            for (int dx = 0; dx < 3; ++dx) {
                                const int h = stride * ho + dy - 1, w = stride * wo + dx - 1;
                                if (h < 0 || h >= H || w < 0 || w >= W)
                                    continue;
                                r += kw[3 * dy + dx] * xs[(((int64_t)n * C_in + ci) * H + h) * W + w];
                            }
                        T[((int64_t)ci * K + k) * plane + (int64_t)ho * Wo + wo] = r;
                    }
            }
        for (int co = 0; co < C_out; ++co)
            for (int64_t p = 0; p < plane; ++p) {
                int32_t s = 0;
                for (int ci = 0; ci < C_in; ++ci)
                    s += T[((int64_t)ci * K + idx[(int64_t)co * C_in + ci]) * plane + p];
                const int64_t o = ((int64_t)n * C_out + co) * plane + p;
                if (S)
                    S[o] = s;
                if (Y) {
                    const float sf = (float)s;
                    Y[o] = sf * alpha[co];
                }
            }
    }
    free(T);
    return 0;
}

/* The same two stages with real-valued activations; T and the sums in float64. */
int snn_oracle_two_stage_f32(const float *x, int N, int C_in, int C_out, int H, int W, int stride,
                             const uint16_t *codebook, int K, const uint16_t *idx,
                             const float *alpha, double *Sd, float *Y)
{
    const int Ho = snn_oracle_out_size(H, stride), Wo = snn_oracle_out_size(W, stride);
    const int64_t plane = (int64_t)Ho * Wo;
    double *T = (double *)malloc((size_t)C_in * K * plane * sizeof(double));
    if (!T)
        return -1;
    for (int n = 0; n < N; ++n) {
        for (int ci = 0; ci < C_in; ++ci)
            for (int k = 0; k < K; ++k) {
                int8_t kw[9];
                snn_oracle_decode(codebook[k], kw);
                for (int ho = 0; ho < Ho; ++ho)
                    for (int wo = 0; wo < Wo; ++wo) {
                        double r = 0.0;
                        for (int dy = 0; dy < 3; ++dy)
                            for (int dx = 0; dx < 3; ++dx) {
                                const int h = stride * ho + dy - 1, w = stride * wo + dx - 1;
                                if (h < 0 || h >= H || w < 0 || w >= W)
                                    continue;
                                const double v = (double)x[(((int64_t)n * C_in + ci) * H + h) * W + w];
                                r += (kw[3 * dy + dx] > 0) ? v : -v;
                            }
                        T[((int64_t)ci * K + k) * plane + (int64_t)ho * Wo + wo] = r;
                    }
            }
        for (int co = 0; co < C_out; ++co)
            for (int64_t p = 0; p < plane; ++p) {
                double s = 0.0;
                for (int ci = 0; ci < C_in; ++ci)
                    s += T[((int64_t)ci * K + idx[(int64_t)co * C_in + ci]) * plane + p];
                const int64_t o = ((int64_t)n * C_out + co) * plane + p;
                if (Sd)
                    Sd[o] = s;
                if (Y)
                    Y[o] = (float)((double)alpha[co] * s);
            }
    }
    free(T);
    return 0;
}

/*
 * Eq. 2 / Eq. 5 / Alg. 1 forward: nearest member of the subset.  ||k||^2 = 9 for every
 * binary kernel, so arg min ||k - w||^2 = arg max <k, w>.  The inner product is built in
 * fp32 from 0, taps 0..8 in order, adding w_t where the code bit is 1 and subtracting it
 * where it is 0 (no multiplies); the lowest index wins among equal scores.
 * score_out (the winning score) may be NULL.
 */
void snn_oracle_project(const float *w, int64_t n, const uint16_t *codebook, int K,
                        uint16_t *idx_out, float *score_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n; ++c) {
        int best = 0;
        float best_score = 0.0f;
        for (int k = 0; k < K; ++k) {
            volatile float acc = 0.0f; /* volatile: every partial sum is rounded to fp32 */
            for (int t = 0; t < 9; ++t) {
                const float v = w[c * 9 + t];
                if ((codebook[k] >> (8 - t)) & 1)
                    acc = acc + v;
                else
                    acc = acc - v;
            }
            const float score = acc;
            if (k == 0 || score > best_score) {
                best = k;
                best_score = score;
            }
        }
        idx_out[c] = (uint16_t)best;
        if (score_out)
            score_out[c] = best_score;
    }
}
