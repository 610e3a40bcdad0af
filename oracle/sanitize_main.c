/*
 * Sanitizer run of the CPU oracle (test infrastructure only; see tests/test_oracle_sanitize.py).
 *
 * Built together with snn_oracle.c under -fsanitize=address,undefined and run as a program of its own:
 * every function of the oracle is called on heap buffers of exactly the size its comment states, on
 * shapes with ragged edges (rows of 1, 33 and 65 pixels, 33 channels, strides 1 and 2, one-pixel
 * images, subsets of 1 and of all 512 kernels), so that an access outside a buffer, a signed overflow
 * or a shift out of range in the oracle itself stops the run.  Prints a checksum and "ok".
 */
#include "snn_oracle.c"

#include <stdio.h>
#include <stdlib.h>

static uint32_t rng_state = 20211009u;
static uint32_t rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}
static float rndf(void) { return ((int)(rnd() % 2001) - 1000) / 500.0f; }

static double run_case(int N, int C_in, int C_out, int H, int W, int stride, int K)
{
    const int Ho = snn_oracle_out_size(H, stride), Wo = snn_oracle_out_size(W, stride);
    const size_t nx = (size_t)N * C_in * H * W, ny = (size_t)N * C_out * Ho * Wo, nk = (size_t)C_out * C_in;
    float *x = malloc(nx * sizeof(float));
    int8_t *xs = malloc(nx);
    uint32_t *pr = malloc((size_t)N * C_in * H * ((W + 31) / 32) * 4);
    uint32_t *pc = malloc((size_t)N * H * W * ((C_in + 31) / 32) * 4);
    uint16_t *cb = malloc((size_t)K * 2), *idx = malloc(nk * 2), *codes = malloc(nk * 2), *pidx = malloc(nk * 2);
    float *alpha = malloc((size_t)C_out * 4), *Y = malloc(ny * 4), *Y2 = malloc(ny * 4), *w = malloc(nk * 9 * 4), *score = malloc(nk * 4);
    int32_t *S = malloc(ny * 4), *S2 = malloc(ny * 4);
    double *Sd = malloc(ny * 8), *Sd2 = malloc(ny * 8);
    for (size_t i = 0; i < nx; ++i) x[i] = rndf();
    for (int k = 0; k < K; ++k) cb[k] = (uint16_t)(K == 512 ? k : (k * 37 + 5) % 512);
    for (size_t i = 0; i < nk; ++i) idx[i] = (uint16_t)(rnd() % (uint32_t)K);
    for (int c = 0; c < C_out; ++c) alpha[c] = 0.5f + (float)(rnd() % 1000) / 1000.0f;
    for (size_t i = 0; i < nk * 9; ++i) w[i] = rndf();
    snn_oracle_sign(x, xs, (int64_t)nx);
    snn_oracle_pack_rows(x, pr, N, C_in, H, W);
    snn_oracle_pack_channels(x, pc, N, C_in, H, W);
    snn_oracle_expand(cb, idx, (int64_t)nk, codes);
    snn_oracle_conv_bin(xs, N, C_in, C_out, H, W, stride, codes, alpha, S, Y);
    snn_oracle_conv_f32(x, N, C_in, C_out, H, W, stride, codes, alpha, Sd, Y2);
    const int ra = snn_oracle_two_stage_bin(xs, N, C_in, C_out, H, W, stride, cb, K, idx, alpha, S2, Y2);
    const int rb = snn_oracle_two_stage_f32(x, N, C_in, C_out, H, W, stride, cb, K, idx, alpha, Sd2, Y2);
    snn_oracle_project(w, (int64_t)nk, cb, K, pidx, score);
    double sum = (double)ra + rb;
    for (size_t i = 0; i < ny; ++i) {
        if (ra == 0 && S[i] != S2[i]) {
            fprintf(stderr, "two-stage and direct sums differ\n");
            exit(3);
        }
        sum += S[i] + Y[i] + Sd[i];
    }
    for (size_t i = 0; i < nk; ++i) sum += pidx[i] + score[i];
    sum += pr[0] + pc[0];
    free(x); free(xs); free(pr); free(pc); free(cb); free(idx); free(codes); free(pidx);
    free(alpha); free(Y); free(Y2); free(w); free(score); free(S); free(S2); free(Sd); free(Sd2);
    return sum;
}

int main(void)
{
    double sum = 0.0;
    sum += run_case(2, 3, 5, 7, 33, 1, 32);
    sum += run_case(1, 33, 4, 5, 65, 2, 16);
    sum += run_case(3, 2, 2, 1, 1, 1, 1);
    sum += run_case(1, 1, 1, 1, 1, 2, 2);
    sum += run_case(1, 4, 3, 6, 4, 2, 512);
    sum += run_case(2, 5, 6, 2, 31, 1, 64);
    int8_t k[9];
    snn_oracle_decode(511, k);
    snn_oracle_decode(0, k);
    printf("checksum %.6f threads %d\nok\n", sum, snn_oracle_threads());
    return 0;
}
