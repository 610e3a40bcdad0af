// Sign + bit-packing of fp32 activations (Alg. 1 forward: sign(a^{i-1})).
// HBM-bound: 4 bytes read and 1/8 byte written per element.
#include "snn_internal.h"

namespace snn {

namespace {

constexpr int PACK_THREADS = 256;
constexpr int PACK_CHUNK = 2048;   // elements whose sign bits are staged in LDS per pass (8 loads per thread)

// Coalesced loads -> wave ballots -> a flat bit stream in LDS -> one output word per thread,
// cut out of the stream at the row's bit offset (rows need not be multiples of 32 wide).
__global__ __launch_bounds__(PACK_THREADS)
void pack_rows_kernel(const float *__restrict__ x, uint32_t *__restrict__ out, int64_t rows, int W,
                      int WW, int rows_per_block)
{
    __shared__ uint32_t bits[PACK_CHUNK / 32 + 2];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int nrows = (int)min((int64_t)rows_per_block, rows - r0);
    if (nrows <= 0) return;

    // W <= PACK_CHUNK: one pass over nrows whole rows.  Otherwise rows_per_block == 1 and the
    // single row is cut into word-aligned segments of PACK_CHUNK elements.
    const int row_len = (W <= PACK_CHUNK) ? nrows * W : W;
    for (int seg = 0; seg < row_len; seg += PACK_CHUNK) {
        const int cnt = min(PACK_CHUNK, row_len - seg);
        const float *src = x + r0 * W + seg;
        // eight independent loads in flight per thread, then eight ballots
        constexpr int U = 8;
        for (int base = 0; base < cnt; base += PACK_THREADS * U) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = base + u * PACK_THREADS + tid;
                v[u] = i < cnt ? src[i] : -1.0f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = base + u * PACK_THREADS + tid;
                const unsigned long long m = __ballot(v[u] >= 0.0f);
                if ((tid & 63) == 0 && (i & ~63) < cnt) {
                    bits[(i >> 6) * 2] = (uint32_t)m;
                    bits[(i >> 6) * 2 + 1] = (uint32_t)(m >> 32);
                }
            }
        }
        __syncthreads();
        if (W <= PACK_CHUNK) {
            const int nwords = nrows * WW;
            for (int q = tid; q < nwords; q += PACK_THREADS) {
                const int rl = q / WW, j = q - rl * WW;
                const int o = rl * W + 32 * j;
                const int nb = min(32, W - 32 * j);
                const int sh = o & 31;
                uint32_t v = bits[o >> 5] >> sh;
                if (sh + nb > 32) v |= bits[(o >> 5) + 1] << (32 - sh);
                if (nb < 32) v &= (1u << nb) - 1u;
                out[r0 * WW + q] = v;
            }
        } else {
            const int nwords = (cnt + 31) >> 5;
            for (int q = tid; q < nwords; q += PACK_THREADS) {
                const int nb = min(32, cnt - 32 * q);
                uint32_t v = bits[q];
                if (nb < 32) v &= (1u << nb) - 1u;
                out[r0 * WW + (seg >> 5) + q] = v;
            }
        }
        __syncthreads();
    }
}

// One thread per (pixel, word of 32 channels): 32 loads that are coalesced across the wave
// (consecutive pixels of one channel plane), one word out.
__global__ __launch_bounds__(PACK_THREADS)
void pack_channels_kernel(const float *__restrict__ x, uint32_t *__restrict__ out, int64_t NHW, int C,
                          int HW, int CW)
{
    const int64_t pix = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    const int cw = blockIdx.y;
    if (pix >= NHW) return;
    const int64_t n = pix / HW;
    const int hw = (int)(pix - n * HW);
    const int c0 = cw * 32;
    const int nc = min(32, C - c0);
    const float *src = x + (n * C + c0) * HW + hw;
    uint32_t word = 0;
#pragma unroll 8
    for (int c = 0; c < nc; ++c)
        word |= (uint32_t)(src[(int64_t)c * HW] >= 0.0f) << c;
    out[pix * CW + cw] = word;
}

}  // namespace

int launch_pack_rows(const float *x, uint32_t *out, int64_t rows, int W, hipStream_t s)
{
    const int WW = (W + 31) / 32;
    const int rows_per_block = (W <= PACK_CHUNK) ? PACK_CHUNK / W : 1;
    const int64_t blocks = (rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;
    hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)blocks), dim3(PACK_THREADS), 0, s, x, out, rows, W,
                       WW, rows_per_block);
    return check_launch();
}

int launch_pack_channels(const float *x, uint32_t *out, int N, int C, int H, int W, hipStream_t s)
{
    const int HW = H * W;
    const int CW = (C + 31) / 32;
    const int64_t NHW = (int64_t)N * HW;
    const int64_t blocks = (NHW + PACK_THREADS - 1) / PACK_THREADS;
    if (blocks > 0x7fffffffLL || CW > 65535) return SNN_ERR_INVALID_ARG;
    hipLaunchKernelGGL(pack_channels_kernel, dim3((unsigned)blocks, (unsigned)CW), dim3(PACK_THREADS), 0, s, x,
                       out, NHW, C, HW, CW);
    return check_launch();
}

}  // namespace snn
