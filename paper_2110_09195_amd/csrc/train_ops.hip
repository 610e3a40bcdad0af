// Training-side operations of a sub-bit layer (Alg. 1 backward lines, Sec. 4.2 / 4.3):
//   * the straight-through estimator for the real-valued kernels (Eq. 3) together with the gradient of
//     the subset tensor p, which is the gradient of its sign memory m: per member, the sum of the
//     gradients of the binarised kernels assigned to it (backward of Eq. 5 / Eq. 6);
//   * the update of the sign memory m from p with the hysteresis threshold theta (Eq. 4), the 9-bit
//     codes of the refined subset, and the check for repeated members (Sec. 4.3).
// All of it is memory-bound streaming over [n][9] floats plus a K x 9 reduction.
#include "snn_internal.h"

namespace snn {

namespace {

constexpr int TB_THREADS = 256;
constexpr int TB_PER = 2;                            // kernels per thread
constexpr int TB_BLOCK = TB_THREADS * TB_PER;        // kernels per block

// Pass 1: g_w = g_wbar where w in (-1, 1) (element-wise), else 0; per block, the sums of g_wbar by
// member in LDS (float atomics), written as one partial [K][9] per block.
__global__ __launch_bounds__(TB_THREADS)
void project_backward_kernel(const float *__restrict__ w, const float *__restrict__ g_wbar,
                             const uint16_t *__restrict__ idx, int64_t n, int K, float *__restrict__ g_w,
                             float *__restrict__ partial)
{
    extern __shared__ float acc[];                   // [K][9]
    const int tid = threadIdx.x;
    for (int i = tid; i < K * 9; i += TB_THREADS) acc[i] = 0.0f;
    __syncthreads();
    const int64_t c0 = (int64_t)blockIdx.x * TB_BLOCK;
#pragma unroll
    for (int q = 0; q < TB_PER; ++q) {
        const int64_t c = c0 + q * TB_THREADS + tid;
        if (c < n) {
            const int k = min((int)idx[c], K - 1);
            float wv[9], gv[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                wv[t] = w[c * 9 + t];
                gv[t] = g_wbar[c * 9 + t];
            }
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                g_w[c * 9 + t] = (wv[t] > -1.0f && wv[t] < 1.0f) ? gv[t] : 0.0f;
                atomicAdd(&acc[k * 9 + t], gv[t]);
            }
        }
    }
    __syncthreads();
    float *dst = partial + (int64_t)blockIdx.x * K * 9;
    for (int i = tid; i < K * 9; i += TB_THREADS) dst[i] = acc[i];
}

// Pass 2: g_p[k][t] = sum of the block partials; one wave per entry: lane l adds the partials of
// blocks l, l + 64, ... in order, then the 64 lane sums are added in a fixed butterfly.
__global__ __launch_bounds__(TB_THREADS)
void reduce_partials_kernel(const float *__restrict__ partial, int64_t blocks, int K9, float *__restrict__ g_p)
{
    const int i = blockIdx.x * (TB_THREADS / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (i >= K9) return;                             // wave-uniform
    float s = 0.0f;
    for (int64_t b = lane; b < blocks; b += 64) s += partial[b * K9 + i];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d);
    if (lane == 0) g_p[i] = s;
}

// One block: m' (Eq. 4), codes, repeated members.
__global__ __launch_bounds__(TB_THREADS)
void subset_update_kernel(const float *__restrict__ p, int8_t *__restrict__ m, float theta, int K,
                          uint16_t *__restrict__ codebook, uint8_t *__restrict__ dup)
{
    __shared__ uint16_t codes[512];
    const int tid = threadIdx.x;
    for (int k = tid; k < K; k += TB_THREADS) {
        uint32_t code = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const float pv = p[k * 9 + t];
            int8_t mv = m[k * 9 + t];
            if (fabsf(pv) > theta) mv = pv > 0.0f ? 1 : -1;      // |p| > theta >= 0: p is not zero
            m[k * 9 + t] = mv;
            code |= (mv > 0 ? 1u : 0u) << (8 - t);
        }
        codes[k] = (uint16_t)code;
        codebook[k] = (uint16_t)code;
    }
    __syncthreads();
    for (int k = tid; k < K; k += TB_THREADS) {
        uint8_t d = 0;
        for (int j = 0; j < k; ++j) d |= codes[j] == codes[k] ? 1 : 0;
        dup[k] = d;
    }
}

}  // namespace

size_t project_backward_workspace_bytes(int64_t n, int K)
{
    const int64_t blocks = (n + TB_BLOCK - 1) / TB_BLOCK;
    return align_up((size_t)(blocks > 0 ? blocks : 1) * K * 9 * sizeof(float), 256);
}

int launch_project_backward(const float *w, const float *g_wbar, const uint16_t *idx, int64_t n, int K, float *g_w,
                            float *g_p, void *ws, hipStream_t s)
{
    const int64_t blocks = (n + TB_BLOCK - 1) / TB_BLOCK;
    if (blocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;
    if (blocks > 0)
        hipLaunchKernelGGL(project_backward_kernel, dim3((unsigned)blocks), dim3(TB_THREADS), (size_t)K * 9 * sizeof(float), s, w,
                           g_wbar, idx, n, K, g_w, (float *)ws);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((K * 9 + TB_THREADS / 64 - 1) / (TB_THREADS / 64))), dim3(TB_THREADS), 0, s,
                       (const float *)ws, blocks, K * 9, g_p);
    return check_launch();
}

int launch_subset_update(const float *p, int8_t *m, float theta, int K, uint16_t *codebook, uint8_t *dup, hipStream_t s)
{
    hipLaunchKernelGGL(subset_update_kernel, dim3(1), dim3(TB_THREADS), 0, s, p, m, theta, K, codebook, dup);
    return check_launch();
}

}  // namespace snn
