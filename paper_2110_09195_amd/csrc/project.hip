// Nearest-subset-member projection (Eq. 2 / Eq. 5, Alg. 1 forward):
//   idx[c] = arg max_k <P_k, w_c>   (lowest index among equal scores)
// with the inner product accumulated in fp32 from 0 over taps 0..8 in order, adding or
// subtracting w_t (project_argmax in front_ops.h: fma(w_t, +-1, acc) rounds exactly like
// acc +- w_t).  HBM-bound for the subset sizes of the paper (K <= 64): 36 B in, 2 B out per kernel.
#include "front_ops.h"

namespace snn {

namespace {

constexpr int PROJ_THREADS = 256;
constexpr int PROJ_PER = 2;                  // kernels per thread: one coefficient read serves two chains
constexpr int PROJ_BLOCK = PROJ_THREADS * PROJ_PER;

__global__ __launch_bounds__(PROJ_THREADS)
void project_kernel(const float *__restrict__ w, int64_t n, const uint16_t *__restrict__ codebook, int K,
                    uint16_t *__restrict__ idx_out)
{
    extern __shared__ __align__(16) float lds[];
    float *coef = lds;                       // [K][12]  +1.0f / -1.0f, taps 0..8 (+3 pad): three 16-byte reads
    float *wl = lds + K * 12;                // [PROJ_BLOCK][9] staged kernels
    const int tid = threadIdx.x;

    project_fill_coef(coef, codebook, K, tid, PROJ_THREADS);

    const int64_t c0 = (int64_t)blockIdx.x * PROJ_BLOCK;
    const int cnt = (int)min((int64_t)PROJ_BLOCK, n - c0);
    const float *src = w + c0 * 9;
    if (cnt == PROJ_BLOCK && (((uintptr_t)w) & 15) == 0) {
        // full block: 16-byte loads (the block starts at a multiple of 16 bytes)
        const float4 *s4 = (const float4 *)src;
#pragma unroll
        for (int i = tid; i < PROJ_BLOCK * 9 / 4; i += PROJ_THREADS) ((float4 *)wl)[i] = s4[i];
    } else {
        for (int i = tid; i < cnt * 9; i += PROJ_THREADS) wl[i] = src[i];
    }
    __syncthreads();

    // thread handles kernels tid and tid + 256 of the block (stride-9 LDS reads: no conflicts)
    float wt[PROJ_PER][9];
#pragma unroll
    for (int q = 0; q < PROJ_PER; ++q)
#pragma unroll
        for (int t = 0; t < 9; ++t)
            wt[q][t] = (q * PROJ_THREADS + tid < cnt) ? wl[(q * PROJ_THREADS + tid) * 9 + t] : 0.0f;

    int best[PROJ_PER];
    project_argmax<PROJ_PER>(wt, coef, K, best);
#pragma unroll
    for (int q = 0; q < PROJ_PER; ++q)
        if (q * PROJ_THREADS + tid < cnt) idx_out[c0 + q * PROJ_THREADS + tid] = (uint16_t)best[q];
}

}  // namespace

int launch_project(const float *w, int64_t n, const uint16_t *codebook, int K, uint16_t *idx_out,
                   hipStream_t s)
{
    const int64_t blocks = (n + PROJ_BLOCK - 1) / PROJ_BLOCK;
    if (blocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;
    const size_t lds = (size_t)(K * 12 + PROJ_BLOCK * 9) * sizeof(float);    // <= 43 KB
    hipLaunchKernelGGL(project_kernel, dim3((unsigned)blocks), dim3(PROJ_THREADS), lds, s, w, n, codebook, K,
                       idx_out);
    return check_launch();
}

}  // namespace snn
