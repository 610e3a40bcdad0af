// Nearest-subset-member projection (Eq. 2 / Eq. 5, Alg. 1 forward):
//   idx[c] = arg max_k <P_k, w_c>   (lowest index among equal scores)
// with the inner product accumulated in fp32 from 0 over taps 0..8 in order, adding or
// subtracting w_t.  fma(w_t, +-1, acc) rounds exactly like acc +- w_t, so the chain below is
// that sum.  HBM-bound for the subset sizes of the paper (K <= 64): 36 B in, 2 B out per kernel.
#include "snn_internal.h"

namespace snn {

namespace {

constexpr int PROJ_THREADS = 256;

__global__ __launch_bounds__(PROJ_THREADS)
void project_kernel(const float *__restrict__ w, int64_t n, const uint16_t *__restrict__ codebook, int K,
                    uint16_t *__restrict__ idx_out)
{
    extern __shared__ float lds[];
    float *coef = lds;                       // [K][9]  +1.0f / -1.0f
    float *wl = lds + K * 9;                 // [PROJ_THREADS][9] staged kernels
    const int tid = threadIdx.x;

    for (int i = tid; i < K * 9; i += PROJ_THREADS) {
        const int k = i / 9, t = i - 9 * k;
        coef[i] = ((codebook[k] >> (8 - t)) & 1) ? 1.0f : -1.0f;
    }

    const int64_t c0 = (int64_t)blockIdx.x * PROJ_THREADS;
    const int cnt = (int)min((int64_t)PROJ_THREADS, n - c0);
    const float *src = w + c0 * 9;
    for (int i = tid; i < cnt * 9; i += PROJ_THREADS)
        wl[i] = src[i];
    __syncthreads();
    if (tid >= cnt) return;

    float wt[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
        wt[t] = wl[tid * 9 + t];

    int best = 0;
    float best_score = 0.0f;
    for (int k = 0; k < K; ++k) {
        const float *ck = coef + k * 9;
        float acc = 0.0f;
#pragma unroll
        for (int t = 0; t < 9; ++t)
            acc = __builtin_fmaf(wt[t], ck[t], acc);
        if (k == 0 || acc > best_score) {
            best = k;
            best_score = acc;
        }
    }
    idx_out[c0 + tid] = (uint16_t)best;
}

}  // namespace

int launch_project(const float *w, int64_t n, const uint16_t *codebook, int K, uint16_t *idx_out,
                   hipStream_t s)
{
    const int64_t blocks = (n + PROJ_THREADS - 1) / PROJ_THREADS;
    if (blocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;
    const size_t lds = (size_t)(K * 9 + PROJ_THREADS * 9) * sizeof(float);   // <= 27.6 KB
    hipLaunchKernelGGL(project_kernel, dim3((unsigned)blocks), dim3(PROJ_THREADS), lds, s, w, n, codebook, K,
                       idx_out);
    return check_launch();
}

}  // namespace snn
