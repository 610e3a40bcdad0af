// Sign + bit-packing of fp32 activations (Alg. 1 forward: sign(a^{i-1})).
// HBM-bound: 4 bytes read and 1/8 byte written per element.
#include "front_ops.h"

namespace snn {

namespace {

// A workgroup packs a run of consecutive blocks of rows: one contiguous piece of the input per workgroup, the
// loads of the next two blocks in flight while the current one is packed.  (The memory system reads faster that
// way than when the workgroups in flight share one window of the tensor, 8 KB each: 7.1 against 5.9 TB/s for a
// read-only stream.)  Runs of four while the launch still has several thousand workgroups (measured on
// the ResNet-18 stack's 55 000 blocks: 86 us with single blocks, 79 us with runs of two or four, 83 with eight,
// 85 with sixteen - longer runs leave too few workgroups)
constexpr int PACK_RUN_MAX = 4;
inline int pack_run(int64_t blocks)
{
    int run = 1;
    while (run < PACK_RUN_MAX && blocks / (2 * run) >= 4096) run *= 2;
    return run;
}

__global__ __launch_bounds__(PACK_THREADS)
void pack_rows_kernel(const float *__restrict__ x, uint32_t *__restrict__ out, int64_t rows, int W,
                      int WW, int rows_per_block, int vec, int64_t blocks, int run)
{
    __shared__ uint32_t bits[2 * PACK_LDS_WORDS];
    const int64_t b0 = (int64_t)blockIdx.x * run, b1 = min(b0 + run, blocks);
    if (vec && W <= PACK_CHUNK) {
        pack_rows_stream(x, out, rows, W, WW, rows_per_block, b0, b1, bits);
        return;
    }
    for (int64_t b = b0; b < b1; ++b) pack_rows_block(x, out, rows, W, WW, rows_per_block, vec, b, bits);
}

// The same for up to PACK_MANY_MAX tensors in one launch: blocks [first_block[i], first_block[i + 1]) pack tensor i.
// (A stack's inputs are packed at a fifth of the memory rate when each is a launch of its own: most are
// smaller than what the chip moves in the time a launch takes to start and drain.)
constexpr int PACK_MANY_MAX = 32;
struct PackManyParams {
    int n, run;
    int first_block[PACK_MANY_MAX + 1];
    struct Item {
        const float *x;
        uint32_t *out;
        int64_t rows;
        int W, WW, rows_per_block, vec;
        int blocks;             // blocks of rows of this tensor; a workgroup takes `run` of them
    } item[PACK_MANY_MAX];
};

__global__ __launch_bounds__(PACK_THREADS)
void pack_rows_many_kernel(const PackManyParams p)
{
    __shared__ uint32_t bits[2 * PACK_LDS_WORDS];
    const int b = blockIdx.x;
    int i = 0;
    while (i + 1 < p.n && b >= p.first_block[i + 1]) ++i;      // block-uniform
    const PackManyParams::Item &k = p.item[i];
    const int b0 = (b - p.first_block[i]) * p.run, b1 = min(b0 + p.run, k.blocks);
    if (k.vec && k.W <= PACK_CHUNK) {
        pack_rows_stream(k.x, k.out, k.rows, k.W, k.WW, k.rows_per_block, (int64_t)b0, (int64_t)b1, bits);
        return;
    }
    for (int c = b0; c < b1; ++c) pack_rows_block(k.x, k.out, k.rows, k.W, k.WW, k.rows_per_block, k.vec, (int64_t)c, bits);
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
        word |= (uint32_t)(load_once(src + (int64_t)c * HW) >= 0.0f) << c;
    out[pix * CW + cw] = word;
}

}  // namespace

int launch_pack_rows(const float *x, uint32_t *out, int64_t rows, int W, hipStream_t s)
{
    const int WW = (W + 31) / 32;
    const PackRowsPlan pl = pack_rows_plan(x, rows, W);
    if (pl.blocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;
    const int run = pack_run(pl.blocks);
    hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)((pl.blocks + run - 1) / run)), dim3(PACK_THREADS), 0, s, x, out, rows, W,
                       WW, pl.rows_per_block, pl.vec, pl.blocks, run);
    return check_launch();
}

int launch_pack_rows_many(int n, const float *const *x, uint32_t *const *out, const int64_t *rows, const int *W, hipStream_t s)
{
    for (int i0 = 0; i0 < n; i0 += PACK_MANY_MAX) {
        PackManyParams pm;
        pm.n = n - i0 < PACK_MANY_MAX ? n - i0 : PACK_MANY_MAX;
        int64_t blocks = 0, row_blocks = 0;
        for (int j = 0; j < pm.n; ++j) row_blocks += pack_rows_plan(x[i0 + j], rows[i0 + j], W[i0 + j]).blocks;
        pm.run = pack_run(row_blocks);
        for (int j = 0; j < pm.n; ++j) {
            const int i = i0 + j;
            const PackRowsPlan pl = pack_rows_plan(x[i], rows[i], W[i]);
            if (pl.blocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
            pm.item[j] = {x[i], out[i], rows[i], W[i], (W[i] + 31) / 32, pl.rows_per_block, pl.vec, (int)pl.blocks};
            pm.first_block[j] = (int)blocks;
            blocks += (pl.blocks + pm.run - 1) / pm.run;
            if (blocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
        }
        for (int j = pm.n; j <= PACK_MANY_MAX; ++j) pm.first_block[j] = (int)blocks;
        if (blocks == 0) continue;
        hipLaunchKernelGGL(pack_rows_many_kernel, dim3((unsigned)blocks), dim3(PACK_THREADS), 0, s, pm);
        const int rc = check_launch();
        if (rc != SNN_OK) return rc;
    }
    return SNN_OK;
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
