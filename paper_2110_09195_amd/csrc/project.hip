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

// The same projection for the vectors of 8 input channels of a 1x1 layer (appendix, Table 5): members
// of a subset of {+-1}^8, element j at code bit 7 - j.  A vector is run through the 9-tap chain with
// a ninth element 0.0f: adding +-0 changes neither a sum nor a comparison, so the result is that of
// the sequential sum over the 8 elements.
__global__ __launch_bounds__(PROJ_THREADS)
void project8_kernel(const float *__restrict__ w, int64_t n, const uint16_t *__restrict__ codebook8, int K,
                     uint16_t *__restrict__ idx_out)
{
    extern __shared__ __align__(16) float lds[];
    float *coef = lds;                                       // [K][12]
    uint16_t *code9 = (uint16_t *)(lds + K * 12);            // [K]: the 8-bit codes as 9-bit ones, last tap +1
    const int tid = threadIdx.x;
    for (int k = tid; k < K; k += PROJ_THREADS) code9[k] = (uint16_t)(((codebook8[k] & 255u) << 1) | 1u);
    __syncthreads();
    project_fill_coef(coef, code9, K, tid, PROJ_THREADS);
    __syncthreads();
    const int64_t v = (int64_t)blockIdx.x * PROJ_THREADS + tid;
    if (v >= n) return;
    const float4 a = ((const float4 *)w)[2 * v], b = ((const float4 *)w)[2 * v + 1];     // 32-byte vectors: aligned
    const float wt[1][9] = {{a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w, 0.0f}};
    int best[1];
    project_argmax<1>(wt, coef, K, best);
    idx_out[v] = (uint16_t)best[0];
}

}  // namespace

int launch_project8(const float *w, int64_t n, const uint16_t *codebook8, int K, uint16_t *idx_out, hipStream_t s)
{
    const int64_t blocks = (n + PROJ_THREADS - 1) / PROJ_THREADS;
    if (blocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;
    const size_t lds = (size_t)K * 12 * sizeof(float) + (size_t)K * sizeof(uint16_t);      // <= 12.5 KB
    hipLaunchKernelGGL(project8_kernel, dim3((unsigned)blocks), dim3(PROJ_THREADS), lds, s, w, n, codebook8, K, idx_out);
    return check_launch();
}

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
