// Sign + bit-packing of fp32 activations (Alg. 1 forward: sign(a^{i-1})).
// HBM-bound: 4 bytes read and 1/8 byte written per element.
#include "snn_internal.h"

namespace snn {

namespace {

constexpr int PACK_THREADS = 256;
constexpr int PACK_U = 4;                                  // 16-byte loads in flight per thread
constexpr int PACK_CHUNK = PACK_THREADS * 4 * PACK_U;      // elements whose sign bits are staged in LDS per pass

// 16-byte loads -> four sign bits per lane -> eight lanes OR their nibbles into one word of a flat
// bit stream in LDS -> one output word per thread, cut out of the stream at the row's bit offset
// (rows need not be multiples of 32 wide).  `vec` says that every block's first element is 16-byte
// aligned; the last, partial group of four of a segment is read element by element.
__global__ __launch_bounds__(PACK_THREADS)
void pack_rows_kernel(const float *__restrict__ x, uint32_t *__restrict__ out, int64_t rows, int W,
                      int WW, int rows_per_block, int vec)
{
    __shared__ uint32_t bits[PACK_CHUNK / 32 + 2];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int nrows = (int)min((int64_t)rows_per_block, rows - r0);
    if (nrows <= 0) return;

    // W <= PACK_CHUNK: one pass over nrows whole rows.  Otherwise rows_per_block == 1 and the
    // single row is cut into word-aligned segments of PACK_CHUNK elements.
    const int row_len = (W <= PACK_CHUNK) ? nrows * W : W;
    for (int seg = 0; seg < row_len; seg += PACK_CHUNK) {
        const int cnt = min(PACK_CHUNK, row_len - seg);
        const float *src = x + r0 * W + seg;
        float4 v[PACK_U];
#pragma unroll
        for (int u = 0; u < PACK_U; ++u) {
            const int e = (u * PACK_THREADS + tid) * 4;
            if (vec && e + 3 < cnt) {
                v[u] = *(const float4 *)(src + e);
            } else {
                v[u].x = e < cnt ? src[e] : -1.0f;
                v[u].y = e + 1 < cnt ? src[e + 1] : -1.0f;
                v[u].z = e + 2 < cnt ? src[e + 2] : -1.0f;
                v[u].w = e + 3 < cnt ? src[e + 3] : -1.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < PACK_U; ++u) {
            const uint32_t nib = (v[u].x >= 0.0f ? 1u : 0u) | (v[u].y >= 0.0f ? 2u : 0u) | (v[u].z >= 0.0f ? 4u : 0u) |
                                 (v[u].w >= 0.0f ? 8u : 0u);
            uint32_t w = nib << (4 * (lane & 7));
            w |= __shfl_xor(w, 1);
            w |= __shfl_xor(w, 2);
            w |= __shfl_xor(w, 4);
            if ((lane & 7) == 0) bits[(u * PACK_THREADS + tid) >> 3] = w;
        }
        __syncthreads();
        if (W <= PACK_CHUNK) {
            const int nwords = nrows * WW;
            for (int q = tid; q < nwords; q += PACK_THREADS) {
                const int rl = q / WW, j = q - rl * WW;
                const int o = rl * W + 32 * j;
                const int nb = min(32, W - 32 * j);
                const int sh = o & 31;
                uint32_t wv = bits[o >> 5] >> sh;
                if (sh + nb > 32) wv |= bits[(o >> 5) + 1] << (32 - sh);
                if (nb < 32) wv &= (1u << nb) - 1u;
                out[r0 * WW + q] = wv;
            }
        } else {
            const int nwords = (cnt + 31) >> 5;
            for (int q = tid; q < nwords; q += PACK_THREADS) {
                const int nb = min(32, cnt - 32 * q);
                uint32_t wv = bits[q];
                if (nb < 32) wv &= (1u << nb) - 1u;
                out[r0 * WW + (seg >> 5) + q] = wv;
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
    // whole rows per block, a multiple of four of them so that every block starts 16-byte aligned
    int rows_per_block = 1;
    if (W <= PACK_CHUNK) {
        rows_per_block = PACK_CHUNK / W;
        if (rows_per_block >= 4) rows_per_block &= ~3;
    }
    const bool aligned_rows = ((int64_t)rows_per_block * W) % 4 == 0 && (W <= PACK_CHUNK || W % 4 == 0);
    const int vec = (((uintptr_t)x & 15) == 0 && aligned_rows) ? 1 : 0;
    const int64_t blocks = (rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;
    hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)blocks), dim3(PACK_THREADS), 0, s, x, out, rows, W,
                       WW, rows_per_block, vec);
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
