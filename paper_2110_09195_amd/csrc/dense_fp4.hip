// The 1-bit layer of Sec. 3, a = lambda * (w_bar o a_bar), computed as a dense contraction on the
// matrix cores: a second baseline next to the XNOR / bit-count kernel, and the reference point for
// what the sharing of Sec. 4.5 has to beat on this chip.
//
//   S[p][co] = sum over taps t and input channels c of  x(p, t, c) * w(co, c, t)
//
// with x, w in {+1, -1} (0 for taps outside the image and for padding channels) held as FP4
// (e2m1: +1 = 0b0010, -1 = 0b1010, 0 = 0), v_mfma_f32_32x32x64_f8f6f4 with both operands FP4 and
// unit scales.  All products are +-1 or 0 and |S| <= 9 C_in <= 36864 < 2^24, so the fp32 accumulator
// holds S exactly and  y = (float)S * alpha  is the one rounding of the definition.
//
// One contraction step = one tap and 64 input channels: lane half h of the wave holds channels
// 64 s + 32 h .. + 31, i.e. one 32-bit word of the packed-channels input per pixel, which four
// v_perm_b32 pairs turn into the 32 FP4 codes (2 bits -> 1 byte through a 4-entry byte table; the
// table is zero where the tap lies outside the image).  The weights are expanded into the operand
// layout by a preparation kernel (16 bytes per lane and step; from 9-bit codes, or from indices into a
// layer's subset), and the four waves of a workgroup share them through LDS.  An optional epilogue
// replaces y by the next layer's sign bits in the packed-channels layout.
#include <cstdlib>

#include "snn_internal.h"

namespace snn {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t FP4_PAIR_TABLE = 0x222AA2AAu;   // byte j: the two FP4 codes of the sign pair j = (bit 2i+1, bit 2i)

struct DenseParams {
    const uint32_t *x;      // [N][H][W][CW]
    const u32x4 *wq;        // [co block][channel block of 64][tap][lane]: 32 FP4 codes
    const float *alpha;
    const float *beta;      // sign epilogue only
    float *y;
    uint32_t *sign_out;     // sign epilogue only: [N][Ho][Wo][ceil(C_out / 32)]
    Geom g;
    int ncb64;              // channel blocks of 64
    int n_cotiles;          // tiles of CB co blocks
    int n_pxtiles;          // tiles of PB pixel blocks
    int n_pxgroups;         // groups of four pixel tiles: one workgroup each (per co tile)
#ifdef SNN_DENSE_TRACE
    unsigned long long *trace;    // tuning builds: wall-clock samples of two workgroups, 8 per wave
#endif
};
#ifdef SNN_DENSE_TRACE
#define DENSE_TRACE(slot)                                                                       \
    do {                                                                                        \
        if ((blockIdx.x == 3 || blockIdx.x == gridDim.x / 2) && (threadIdx.x & 63) == 0)        \
            p.trace[((blockIdx.x == 3 ? 0 : 4) + (threadIdx.x >> 6)) * 8 + (slot)] = wall_clock64(); \
    } while (0)
#else
#define DENSE_TRACE(slot) do { } while (0)
#endif

// Buffer loads: the range check of the resource turns "no input here" into a load that returns 0
// without a branch (lanes pass an offset beyond the buffer).
constexpr uint32_t OFF_BIT = 0x80000000u;          // buffers here are shorter than 2 GiB
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// 32 sign bits -> 32 FP4 codes (bit j -> nibble j); `table` = FP4_PAIR_TABLE, or 0 for "no input here"
__device__ inline v8i expand_signs(uint32_t w, uint32_t table)
{
    const uint32_t w4 = w >> 4;
    v8i r = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        // byte 0 <- byte q of w, byte 2 <- byte q of w >> 4, bytes 1 and 3 <- 0
        const uint32_t y = __builtin_amdgcn_perm(w, w4, 0x0C000C00u | ((uint32_t)q << 16) | (uint32_t)(4 + q));
        // bit pairs (0,1) (2,3) (4,5) (6,7) of the byte at bits 0, 8, 16, 24
        const uint32_t sel = (y | (y << 6)) & 0x03030303u;
        r[q] = (int)__builtin_amdgcn_perm(0u, table, sel);
    }
    return r;
}

// weights -> operand layout.  One thread per (co block, channel block, lane): the lane's row is output
// channel 32 b + lane % 32, its 32 contraction slots are channels 64 s + 32 (lane / 32) + j.
__global__ __launch_bounds__(256)
void dense_fp4_prep_kernel(const uint16_t *__restrict__ codebook, int K, const uint16_t *__restrict__ w9, int C_in,
                           int C_out, int ncb64, int n_coblocks, u32x4 *__restrict__ wq)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)n_coblocks * ncb64 * 64) return;
    const int lane = (int)(i & 63);
    const int64_t bs = i >> 6;
    const int s = (int)(bs % ncb64), b = (int)(bs / ncb64);
    const int co = 32 * b + (lane & 31);
    const int c0 = 64 * s + 32 * (lane >> 5);
    uint32_t bits[9], have = 0;
#pragma unroll
    for (int t = 0; t < 9; ++t) bits[t] = 0;
    if (co < C_out) {
        // 32 independent loads in flight
        uint32_t code[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) code[j] = c0 + j < C_in ? (uint32_t)w9[(int64_t)co * C_in + c0 + j] : 0x8000u;
        if (codebook) {
            // a sub-bit layer: the entries are indices into the layer's subset (Sec. 4.2)
#pragma unroll
            for (int j = 0; j < 32; ++j)
                if (c0 + j < C_in) code[j] = codebook[min(code[j], (uint32_t)K - 1u)];     // (an index >= K is the caller's error: no fault)
        }
#pragma unroll
        for (int j = 0; j < 32; ++j) code[j] &= 0x81ffu;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            have |= (code[j] >> 15 ^ 1u) << j;
#pragma unroll
            for (int t = 0; t < 9; ++t) bits[t] |= ((code[j] >> (8 - t)) & 1u) << j;
        }
    }
    const v8i keep = expand_signs(have, 0xFFF00F00u);       // nibble j = 0xF where channel c0 + j exists
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const v8i e = expand_signs(bits[t], FP4_PAIR_TABLE);
        u32x4 out;
#pragma unroll
        for (int q = 0; q < 4; ++q) out[q] = (uint32_t)(e[q] & keep[q]);
        wq[(bs * 9 + t) * 64 + lane] = out;
    }
}

// Workgroup = four waves on one tile of CB output-channel blocks and four neighbouring pixel tiles (one
// per wave, PB blocks of 32 pixels each).  The weights of one channel block (nine taps x CB x 1 KB) are
// fetched by the four waves together, a quarter each, into one of two LDS buffers while the previous
// block is being multiplied: every wave then reads its operands from LDS, and the only loads whose
// round trip a wave waits for directly were issued a whole channel block (9 PB CB matrix
// instructions) earlier.
constexpr int CHUNK_ENTRIES = 9 * 64;                       // 16-byte entries per co block and channel block

template <int PB, int CB, bool SIGN>
__global__ __launch_bounds__(256)
void dense_fp4_kernel(DenseParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];   // [2][CB][9][64] x 16 bytes of weights, then [2][CB * 32] floats
    const Geom &g = p.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    DENSE_TRACE(0);
    const int cotile = (int)blockIdx.x / p.n_pxgroups;
    const int pxgroup = (int)blockIdx.x - cotile * p.n_pxgroups;
    // alpha (and beta) of the tile's channels, one per thread: channels past the end read 0
    const __amdgpu_buffer_rsrc_t ares = make_rsrc(p.alpha, (uint32_t)g.C_out * 4u);
    const __amdgpu_buffer_rsrc_t bres = make_rsrc(SIGN ? p.beta : p.alpha, (uint32_t)g.C_out * 4u);
    const uint32_t scale_off = tid < CB * 32 ? (uint32_t)(cotile * CB * 32 + tid) * 4u : OFF_BIT;
    const float early_alpha = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(ares, (int)scale_off, 0, 0));
    const float early_beta = SIGN ? __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(bres, (int)scale_off, 0, 0)) : 0.0f;
    const int pxtile = pxgroup * 4 + wave;                  // past the last tile: a wave without pixels, still loading weights

    const uint32_t cb_stride = (uint32_t)p.ncb64 * 9u * 1024u;      // bytes between the co blocks of the tile
    const __amdgpu_buffer_rsrc_t wres = make_rsrc(p.wq, (uint32_t)p.n_cotiles * CB * cb_stride);
    const uint32_t w_tile = (uint32_t)cotile * CB * cb_stride;
    // this thread's share of a weight chunk: entries tid, tid + 256, ... of the CB x 576
    constexpr int TOTAL = CB * CHUNK_ENTRIES;
    constexpr int NW = (TOTAL + 255) / 256;
    uint32_t w_src[NW];                                     // byte offset inside the tile's weights, channel block 0
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const int e = tid + 256 * i;
        const int cb = e / CHUNK_ENTRIES, rest = e - cb * CHUNK_ENTRIES;
        w_src[i] = e < TOTAL ? w_tile + (uint32_t)cb * cb_stride + (uint32_t)rest * 16u : OFF_BIT;
    }
    u32x4 wreg[NW];
    auto fetch_w = [&](int s) {
#pragma unroll
        for (int i = 0; i < NW; ++i)
            wreg[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, (int)w_src[i], (int)((uint32_t)s * 9216u), 0);
    };
    fetch_w(0);

    // (the first weights are on their way while the lanes work out their geometry)
    // the lane's output pixel in each pixel block, its input corner and the taps inside the image
    uint32_t base[PB];                                      // byte offset of the window's corner word (mod 2^32)
    uint32_t inside[PB];
    int64_t y_off[PB];                                      // of channel 0 (sign epilogue: word 0) at the lane's pixel; -1: no pixel
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
        const int64_t q = ((int64_t)pxtile * PB + pb) * 32 + (lane & 31);
        const bool ok = q < g.P;
        const int qq = ok ? (int)q : 0;                     // P < 2^31
        const int n = qq / g.HoWo;
        const int r = qq - n * g.HoWo;
        y_off[pb] = !ok ? -1 : SIGN ? (int64_t)qq * ((g.C_out + 31) / 32) : (int64_t)n * g.C_out * g.HoWo + r;
        const int ho = r / g.Wo, wo = r - ho * g.Wo;
        const int hi0 = ho * g.stride - 1, wi0 = wo * g.stride - 1;
        base[pb] = (uint32_t)(((n * g.H + hi0) * g.W + wi0) * g.CW + h) * 4u;
        // bit 3 dy + dx: row hi0 + dy and column wi0 + dx are inside the image
        const uint32_t cols = (wi0 >= 0 ? 1u : 0u) | 2u | (wi0 + 2 < g.W ? 4u : 0u);     // wi0 + 1 = wo * stride is inside
        const uint32_t m = (hi0 >= 0 ? cols : 0u) | (cols << 3) | (hi0 + 2 < g.H ? cols << 6 : 0u);
        inside[pb] = ok ? m : 0u;
    }

    v16f acc[CB][PB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0.0f;

    const __amdgpu_buffer_rsrc_t xres = make_rsrc(p.x, (uint32_t)g.N * (uint32_t)(g.H * g.W) * (uint32_t)g.CW * 4u);
    const int cw_h = g.CW - h;

    uint32_t xn[9][PB], xc[9][PB];

    // 1 where the lane half has a word of channels in block s (2 s + h < CW) and tap t of pixel block pb
    // lies inside the image; plain bit arithmetic throughout, so that the loads stay unconditional
    auto tap_mask = [&](int s, int t, int pb) -> uint32_t {
        const uint32_t have_word = (uint32_t)(2 * s - cw_h) >> 31;
        return 0u - ((inside[pb] >> t) & have_word);
    };
    auto fetch_x = [&](int s) {
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const uint32_t toff = (uint32_t)(((t / 3) * g.W + (t % 3)) * g.CW + 2 * s) * 4u;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb)
                xn[t][pb] = __builtin_amdgcn_raw_buffer_load_b32(xres, (int)((base[pb] + toff) | (~tap_mask(s, t, pb) & OFF_BIT)), 0, 0);
        }
    };

    DENSE_TRACE(1);
    fetch_x(0);
    // the tile's scales (and offsets) wait in LDS for the epilogue: requested first of all, stored now
    float *const scale_lds = (float *)(smem + 2 * TOTAL * 16);              // [2][CB * 32]
    if (tid < CB * 32) {
        scale_lds[tid] = early_alpha;
        if constexpr (SIGN) scale_lds[CB * 32 + tid] = early_beta;
    }
    for (int s = 0; s < p.ncb64; ++s) {
        unsigned char *buf = smem + (s & 1) * (TOTAL * 16);
#pragma unroll
        for (int i = 0; i < NW; ++i)
            if (tid + 256 * i < TOTAL) *(u32x4 *)(buf + (tid + 256 * i) * 16) = wreg[i];
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) xc[t][pb] = xn[t][pb];
        // One barrier per channel block: a wave that writes buffer (s + 1) & 1 in the next round has passed
        // this barrier, hence every wave has finished reading that buffer in round s - 1.
        __syncthreads();
        if (s + 1 < p.ncb64) {
            fetch_w(s + 1);
            fetch_x(s + 1);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            v8i B[PB];
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) B[pb] = expand_signs(xc[t][pb], FP4_PAIR_TABLE & tap_mask(s, t, pb));
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const u32x4 a = *(const u32x4 *)(buf + ((cb * 9 + t) * 64 + lane) * 16);
                const v8i A = {(int)a[0], (int)a[1], (int)a[2], (int)a[3], 0, 0, 0, 0};
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
                    acc[cb][pb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B[pb], acc[cb][pb], 4, 4, 0, 0, 0, 0);
            }
        }
    }

    DENSE_TRACE(2);
    // y = alpha * S; lanes 0..31 of a register are 32 consecutive pixels of one channel
    float al[CB][16];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) al[cb][r] = scale_lds[cb * 32 + 8 * (r / 4) + (r % 4) + 4 * h];
    if constexpr (SIGN) {
        // The next layer's sign: bit = (fl(fl(S alpha) + beta) >= 0).  A lane holds 16 of the 32 channels
        // of a block for its pixel (rows 8 j + i + 4 h, i < 4); the other lane half holds the rest: one
        // exchange across the halves, and lane half 0 stores the word of 32 channels.
        float be[CB][16];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) be[cb][r] = scale_lds[CB * 32 + cb * 32 + 8 * (r / 4) + (r % 4) + 4 * h];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const int co0 = (cotile * CB + cb) * 32;
            if (co0 >= g.C_out) continue;                                    // (wave-uniform)
            const uint32_t real = g.C_out - co0 >= 32 ? 0xffffffffu : (1u << (g.C_out - co0)) - 1u;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                uint32_t m = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    m |= (mul_then_add(acc[cb][pb][r], al[cb][r], be[cb][r]) >= 0.0f ? 1u : 0u) << (8 * (r / 4) + (r % 4));
                m <<= 4 * h;
                m |= (uint32_t)__shfl_xor((int)m, 32);
                if (h == 0 && y_off[pb] >= 0) p.sign_out[y_off[pb] + (cotile * CB + cb)] = m & real;
            }
        }
        DENSE_TRACE(4);
        return;
    }
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = (cotile * CB + cb) * 32 + 8 * (r / 4) + (r % 4) + 4 * h;
            if (co >= g.C_out) continue;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb)
                if (y_off[pb] >= 0) store_output(p.y + y_off[pb] + (int64_t)co * g.HoWo, acc[cb][pb][r] * al[cb][r]);
            if (cb == 0 && r == 0) DENSE_TRACE(3);
        }
    DENSE_TRACE(4);
}

struct DensePlan {
    int PB, CB;
    int ncb64, n_coblocks, n_cotiles, n_pxtiles, n_pxgroups;
    int64_t n_wgs;
    size_t bytes;
};

DensePlan dense_plan(const Geom &g)
{
    DensePlan pl;
    pl.ncb64 = (g.C_in + 63) / 64;
    const int coblocks = (g.C_out + 31) / 32;
    const int64_t pxblocks = (g.P + 31) / 32;
    // Measured on the layers of a ResNet-18 at batch 64: one pixel block per wave (more waves per SIMD,
    // whose store and compute phases then overlap) and four output-channel blocks while that still
    // leaves a few hundred workgroups, else two.  The two-pixel-block shapes remain selectable
    // (knob SNN_TUNE_DENSE_TILE = 0 / 1) for tuning on larger batches.
    static const int shapes[5][2] = {{2, 4}, {2, 2}, {1, 2}, {1, 1}, {1, 4}};
    const int64_t groups = (pxblocks + 3) / 4;
    int pick = coblocks >= 4 && groups * ((coblocks + 3) / 4) >= 300 ? 4 : coblocks >= 2 ? 2 : 3;
    if (const int v = tuning(SNN_TUNE_DENSE_TILE); v >= 0) pick = v;
    pl.PB = shapes[pick][0];
    pl.CB = shapes[pick][1];
    pl.n_cotiles = (coblocks + pl.CB - 1) / pl.CB;
    pl.n_coblocks = pl.n_cotiles * pl.CB;
    pl.n_pxtiles = (int)((pxblocks + pl.PB - 1) / pl.PB);
    pl.n_pxgroups = (pl.n_pxtiles + 3) / 4;
    pl.n_wgs = (int64_t)pl.n_cotiles * pl.n_pxgroups;
    pl.bytes = align_up((size_t)pl.n_coblocks * pl.ncb64 * 9 * 64 * sizeof(u32x4), 256);
    return pl;
}

template <int PB, int CB, bool SIGN>
int launch_dense_cfg(const DenseParams &prm, int64_t wgs, hipStream_t s)
{
    auto kern = dense_fp4_kernel<PB, CB, SIGN>;
    const size_t lds = (size_t)2 * CB * CHUNK_ENTRIES * 16 + 2 * CB * 32 * sizeof(float);
    static LdsGrant grant;
    if (grant_dynamic_lds((const void *)kern, lds, grant) != SNN_OK) return SNN_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(256), lds, s, prm);
    return check_launch();
}

template <int PB, int CB>
int launch_dense_one(const DenseParams &prm, int64_t wgs, hipStream_t s)
{
    return prm.sign_out ? launch_dense_cfg<PB, CB, true>(prm, wgs, s) : launch_dense_cfg<PB, CB, false>(prm, wgs, s);
}

}  // namespace

bool dense_fp4_supported(const Geom &g)
{
    // 32-bit byte offsets into the packed input and the expanded weights; whole-tile counts that fit the grid
    const int64_t x_words = (int64_t)g.N * g.H * g.W * g.CW;
    const int64_t w_bytes = (int64_t)(((g.C_out + 31) / 32 + 3) / 4 * 4) * ((g.C_in + 63) / 64) * 9 * 1024;
    return x_words < ((int64_t)1 << 29) && w_bytes < ((int64_t)1 << 31) && g.P < ((int64_t)1 << 31) - 64 &&
           ((g.P + 31) / 32) * ((g.C_out + 31) / 32) < ((int64_t)1 << 31);
}

size_t dense_fp4_workspace_bytes(const Geom &g)
{
    const int ncb64 = (g.C_in + 63) / 64;
    // room for the co blocks rounded up to the largest tile
    size_t bytes = align_up((size_t)(((g.C_out + 31) / 32 + 3) / 4 * 4) * ncb64 * 9 * 64 * sizeof(u32x4), 256);
#ifdef SNN_DENSE_TRACE
    bytes += 4096;
#endif
    return bytes;
}

int launch_dense_fp4(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *w9, const float *alpha,
                     float *y, void *ws, hipStream_t s, int phases, const float *beta, uint32_t *sign_out)
{
    const DensePlan pl = dense_plan(g);
    if (phases & SNN_PHASE_PREPARE) {
        // all co blocks the workspace has room for (the largest tile's rounding), whatever tile runs later
        const int n_coblocks = ((g.C_out + 31) / 32 + 3) / 4 * 4;
        const int64_t prep_threads = (int64_t)n_coblocks * pl.ncb64 * 64;
        hipLaunchKernelGGL(dense_fp4_prep_kernel, dim3((unsigned)((prep_threads + 255) / 256)), dim3(256), 0, s, codebook,
                           g.K, w9, g.C_in, g.C_out, pl.ncb64, n_coblocks, (u32x4 *)ws);
        const int rc = check_launch();
        if (rc != SNN_OK) return rc;
    }
    if (!(phases & SNN_PHASE_CONVOLVE)) return SNN_OK;
    DenseParams prm;
    prm.x = (const uint32_t *)x;
    prm.wq = (const u32x4 *)ws;
    prm.alpha = alpha;
    prm.beta = beta;
    prm.y = y;
    prm.sign_out = sign_out;
    prm.g = g;
    prm.ncb64 = pl.ncb64;
    prm.n_cotiles = pl.n_cotiles;
    prm.n_pxtiles = pl.n_pxtiles;
    prm.n_pxgroups = pl.n_pxgroups;
#ifdef SNN_DENSE_TRACE
    prm.trace = (unsigned long long *)((char *)ws + dense_fp4_workspace_bytes(g) - 4096);
#endif
    if (pl.PB == 2 && pl.CB == 4) return launch_dense_one<2, 4>(prm, pl.n_wgs, s);
    if (pl.PB == 2 && pl.CB == 2) return launch_dense_one<2, 2>(prm, pl.n_wgs, s);
    if (pl.PB == 1 && pl.CB == 2) return launch_dense_one<1, 2>(prm, pl.n_wgs, s);
    if (pl.PB == 1 && pl.CB == 4) return launch_dense_one<1, 4>(prm, pl.n_wgs, s);
    return launch_dense_one<1, 1>(prm, pl.n_wgs, s);
}

}  // namespace snn
