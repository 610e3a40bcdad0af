// The 1-bit convolution of Sec. 3: a = lambda * (w_bar o a_bar), "o" = XNOR + bit count over
// words of 32 input channels.  It is the denominator of every speed-up the sub-bit kernel
// reports, so it is written to the same standard.
//
// Packed activations (SNN_ACT_BIN_CHANNELS), two kernels.  Up to 512 input channels: one lane owns
// one output pixel and keeps its window in registers; a block walks a chunk of output channels
// whose weight words wait in LDS (bnn_regs_kernel).  More channels: one lane owns PXL output
// pixels and keeps the mismatch counts of a block of COG output channels in registers; the loop
// runs over the 9 * C_in/32 words of the window, the lane loads its pixel's word and the COG
// weight words that meet it are wave-uniform scalar loads from a [channel block][tap][word][COG]
// table (bnn_bin_kernel).  Either way the body is v_xor + v_bcnt_u32_b32: 2 lane-ops per 32
// multiply-adds.  Taps outside the image are loaded as 0 and the mismatches they fake are taken
// out again with a per-(channel, border type) table.
//
// fp32 activations (SNN_ACT_F32, the W/A = 1/32 rows): the same direct loop with add/subtract.
#include <cstdlib>

#include "snn_internal.h"

namespace snn {

namespace {

constexpr int BNN_THREADS = 256;
// output channels per block of the register-window kernel, by words per tap
__host__ __device__ constexpr int bnn_regs_chunk(int cwt) { return cwt >= 16 ? 16 : cwt >= 8 ? 32 : 64; }

// workspace layout (packed activations):  wplanes [C_out][9][CWT] u32 | corr [C_out][16] i32
// workspace layout (fp32 activations):    flips   [C_out][C_in]    u32 (bit t = tap t is -1)

// One wave per output channel: 64 kernels' codes at a time, one ballot per tap gives two words of
// that tap's bit-plane; the population counts of the planes give the border corrections.
// Layout written: wq[(co / COG)][tap][word][co % COG]; channels past C_out are zero.
__global__ __launch_bounds__(256)
void bnn_prep_bin_kernel(const uint16_t *__restrict__ w9, int C_out, int COP, int C_in, int CW, int COG,
                         uint32_t *__restrict__ wq, int32_t *__restrict__ corr)   // COG = 1: plain [co][tap][word]
{
    const int co = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (co >= COP) return;
    uint32_t *wp = wq + (int64_t)(co / COG) * 9 * CW * COG + (co % COG);
    int ones[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) ones[t] = 0;
    for (int b = 0; 2 * b < CW; ++b) {
        const int ci = 64 * b + lane;
        const uint32_t code = (co < C_out && ci < C_in) ? (w9[(int64_t)co * C_in + ci] & 511u) : 0u;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const unsigned long long m = __ballot((code >> (8 - t)) & 1u);
            ones[t] += __popcll(m);
            if (lane == 0) {
                wp[(t * CW + 2 * b) * COG] = (uint32_t)m;
                if (2 * b + 1 < CW) wp[(t * CW + 2 * b + 1) * COG] = (uint32_t)(m >> 32);
            }
        }
    }
    if (lane < 16) {
        const uint32_t inv = border_invalid_window(lane);
        int s = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t)
            if ((inv >> t) & 1u) s += ones[t];
        corr[co * 16 + lane] = s;
    }
}

__global__ void bnn_prep_f32_kernel(const uint16_t *__restrict__ w9, int64_t n, uint32_t *__restrict__ flips)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        flips[i] = (~code_to_window_order(w9[i] & 511u)) & 511u;
}

// popcount(v) + acc as the one instruction it is (written out: the compiler otherwise counts into fresh
// registers and adds them up three at a time, half an instruction more per word)
__device__ inline int count_add(uint32_t v, int acc)
{
    int r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(v), "v"(acc));
    return r;
}

// Variant for C_in <= 512: a block is 256 output pixels (one per lane) x a chunk of CH output channels.
// The chunk's weight words, border corrections and scales are staged in LDS once; a lane keeps its
// 3x3 window of up to 8 words per tap (256 input channels) in registers and walks the chunk's
// channels, reading the weight words back as wave-wide broadcasts: v_xor + v_bcnt with accumulate,
// 2 lane-ops per 32 multiply-adds.  Wider layers take two passes over the channel halves, with the
// partial counts parked in LDS in between.  The window is loaded through a buffer resource, whose range
// check turns taps outside the image (and padding words) into zeros without a branch.
// (Earlier forms kept the whole window of 144 words in registers and read the weights with scalar
// loads or LDS reads issued right before their use: one wave per SIMD and a wait per read, 24 % of the
// xor / bit-count rate.)
template <int CWT>
__global__ __launch_bounds__(BNN_THREADS)
void bnn_regs_kernel(const uint32_t *__restrict__ x, const uint32_t *__restrict__ wplanes,
                     const int32_t *__restrict__ corr, const float *__restrict__ alpha, float *__restrict__ y,
                     Geom g, int ch)
{
    constexpr int WPC = 9 * CWT;                           // weight words of one output channel
    constexpr int WPCP = (WPC + 3) & ~3;                   //   padded to 16 bytes in LDS
    constexpr int CH = bnn_regs_chunk(CWT);                // most channels per block (about 9 KB of weights); `ch` <= CH are used
    constexpr int WPP = CWT < 8 ? CWT : 8;                 // words per tap and pass
    constexpr int NP = CWT / WPP;                          // passes: 1, or 2 for 16 words per tap
    constexpr int NWL = (CH * WPC + BNN_THREADS - 1) / BNN_THREADS;
    __shared__ __align__(16) uint32_t wl[CH * WPCP];
    __shared__ int32_t cl[CH * 16];
    __shared__ float al[CH];
    __shared__ int part[NP > 1 ? CH * BNN_THREADS : 1];    // partial counts between the passes
    const int tid = threadIdx.x;
    const int co0 = blockIdx.y * ch;
    const int cnt = min(ch, g.C_out - co0);

    // stage the chunk (words of channels past C_out: zero)
#pragma unroll
    for (int i = 0; i < NWL; ++i) {
        const int e = tid + BNN_THREADS * i;               // word e % WPC of channel co0 + e / WPC
        const int j = e / WPC;
        if (j < CH) wl[j * WPCP + (e - j * WPC)] = j < cnt ? wplanes[(int64_t)co0 * WPC + e] : 0u;
    }
    for (int e = tid; e < CH * 16; e += BNN_THREADS) cl[e] = e / 16 < cnt ? corr[(int64_t)co0 * 16 + e] : 0;
    if (tid < CH) al[tid] = tid < cnt ? alpha[co0 + tid] : 0.0f;

    const int64_t p_raw = (int64_t)blockIdx.x * BNN_THREADS + tid;
    const bool active = p_raw < g.P;
    const int64_t p = active ? p_raw : g.P - 1;
    const int n = (int)(p / g.HoWo);
    const int r = (int)(p - (int64_t)n * g.HoWo);
    const int ho = r / g.Wo, wo = r - ho * g.Wo;
    const int hc = ho * g.stride, wc = wo * g.stride;
    const int type = border_type(ho, wo, g.H, g.W, g.stride);
    const int base = border_valid_taps(type) * g.C_in;
    float *yp = y + ((int64_t)n * g.C_out + co0) * g.HoWo + r;

    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(x), 0, (int)((uint32_t)g.N * (uint32_t)(g.H * g.W) * (uint32_t)g.CW * 4u), 0x00020000);
    uint32_t toff[9];                                      // byte offset of the tap's first word; beyond the buffer: outside the image
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int h = hc + t / 3 - 1, w = wc + t % 3 - 1;
        const bool valid = (h >= 0) && (h < g.H) && (w >= 0) && (w < g.W);
        toff[t] = valid ? (uint32_t)(((n * g.H + h) * g.W + w) * g.CW) * 4u : 0x80000000u;
    }
    __syncthreads();

#pragma unroll
    for (int pass = 0; pass < NP; ++pass) {
        uint32_t xr[9][WPP];
        if (WPP % 4 == 0 && g.CW % 4 == 0) {
            // 16-byte loads (a pixel's words start at a multiple of 16 bytes): lanes are a pixel apart, so
            // every lane touches a cache line of its own and the load unit's time goes with the
            // number of instructions, not of bytes
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int q = 0; q < WPP / 4; ++q) {
                    const int word = pass * WPP + 4 * q;   // whole groups past CW pad the power of two: zero
                    const auto v = __builtin_amdgcn_raw_buffer_load_b128(xres, (int)(word < g.CW ? toff[t] + 4u * (uint32_t)word : 0x80000000u), 0, 0);
                    xr[t][4 * q] = v[0];
                    xr[t][4 * q + 1] = v[1];
                    xr[t][4 * q + 2] = v[2];
                    xr[t][4 * q + 3] = v[3];
                }
        } else {
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int cw = 0; cw < WPP; ++cw) {
                    const int word = pass * WPP + cw;      // words past CW pad the power of two: zero
                    xr[t][cw] = __builtin_amdgcn_raw_buffer_load_b32(xres, (int)(word < g.CW ? toff[t] + 4u * (uint32_t)word : 0x80000000u), 0, 0);
                }
        }
        for (int j = 0; j < cnt; ++j) {
            // two chains of bit counts that add as they count (v_bcnt_u32_b32 with its addend)
            int m0 = 0, m1 = 0;
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                // the same address in every lane: broadcast reads
                const uint32_t *wt = &wl[j * WPCP + t * CWT + pass * WPP];
                if constexpr (WPP % 4 == 0) {
#pragma unroll
                    for (int q = 0; q < WPP / 4; ++q) {
                        const uint4 v = *(const uint4 *)(wt + 4 * q);
                        m0 = count_add(xr[t][4 * q] ^ v.x, m0);
                        m1 = count_add(xr[t][4 * q + 1] ^ v.y, m1);
                        m0 = count_add(xr[t][4 * q + 2] ^ v.z, m0);
                        m1 = count_add(xr[t][4 * q + 3] ^ v.w, m1);
                    }
                } else {
#pragma unroll
                    for (int cw = 0; cw < WPP; ++cw) {
                        if (cw & 1) m1 = count_add(xr[t][cw] ^ wt[cw], m1);
                        else m0 = count_add(xr[t][cw] ^ wt[cw], m0);
                    }
                }
            }
            int mm = m0 + m1;
            if (NP > 1 && pass == 0) {
                part[j * BNN_THREADS + tid] = mm;
            } else {
                if (NP > 1) mm += part[j * BNN_THREADS + tid];
                const int S = base - 2 * (mm - cl[j * 16 + type]);
                if (active) store_output(yp + (int64_t)j * g.HoWo, (float)S * al[j]);
            }
        }
    }
}

template <int PXL, int COG>
__global__ __launch_bounds__(BNN_THREADS)
void bnn_bin_kernel(const uint32_t *__restrict__ x, const uint32_t *__restrict__ wq,
                    const int32_t *__restrict__ corr, const float *__restrict__ alpha, float *__restrict__ y,
                    Geom g)
{
    const int cog = blockIdx.y;
    int off[PXL][9];                // word offset of each tap's first word; -1 if the tap is outside
    int type[PXL], base[PXL], nn[PXL], rr[PXL];
    bool active[PXL];
#pragma unroll
    for (int q = 0; q < PXL; ++q) {
        const int64_t p_raw = ((int64_t)blockIdx.x * PXL + q) * BNN_THREADS + threadIdx.x;
        active[q] = p_raw < g.P;
        const int64_t p = active[q] ? p_raw : g.P - 1;
        const int n = (int)(p / g.HoWo);
        const int r = (int)(p - (int64_t)n * g.HoWo);
        const int ho = r / g.Wo, wo = r - ho * g.Wo;
        const int hc = ho * g.stride, wc = wo * g.stride;
        nn[q] = n;
        rr[q] = r;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int h = hc + t / 3 - 1, w = wc + t % 3 - 1;
            const bool valid = (h >= 0) && (h < g.H) && (w >= 0) && (w < g.W);
            off[q][t] = valid ? ((n * g.H + h) * g.W + w) * g.CW : -1;
        }
        type[q] = border_type(ho, wo, g.H, g.W, g.stride);
        base[q] = border_valid_taps(type[q]) * g.C_in;
    }

    int mm[PXL][COG];
#pragma unroll
    for (int q = 0; q < PXL; ++q)
#pragma unroll
        for (int c = 0; c < COG; ++c) mm[q][c] = 0;

    const uint32_t *wt = wq + (int64_t)cog * 9 * g.CW * COG;        // wave-uniform
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        for (int cw = 0; cw < g.CW; ++cw) {
            uint32_t xw[PXL];
#pragma unroll
            for (int q = 0; q < PXL; ++q) xw[q] = off[q][t] >= 0 ? x[off[q][t] + cw] : 0u;
            const uint32_t *wv = wt + (t * g.CW + cw) * COG;
#pragma unroll
            for (int c = 0; c < COG; ++c) {
                const uint32_t w = wv[c];
#pragma unroll
                for (int q = 0; q < PXL; ++q) mm[q][c] += __popc(xw[q] ^ w);
            }
        }
    }

#pragma unroll
    for (int c = 0; c < COG; ++c) {
        const int co = cog * COG + c;
        if (co >= g.C_out) break;
        const float a = alpha[co];
#pragma unroll
        for (int q = 0; q < PXL; ++q) {
            const int cr = type[q] ? corr[co * 16 + type[q]] : 0;
            const int S = base[q] - 2 * (mm[q][c] - cr);
            if (active[q]) store_output(y + ((int64_t)nn[q] * g.C_out + co) * g.HoWo + rr[q], (float)S * a);
        }
    }
}

constexpr int F32_CO = 8;    // output channels accumulated per lane
constexpr int F32_CI = 4;    // input channels whose windows are held in registers

__global__ __launch_bounds__(BNN_THREADS)
void bnn_f32_kernel(const float *__restrict__ x, const uint32_t *__restrict__ flips,
                    const float *__restrict__ alpha, float *__restrict__ y, Geom g)
{
    const int64_t p_raw = (int64_t)blockIdx.x * BNN_THREADS + threadIdx.x;
    const bool active = p_raw < g.P;
    const int64_t p = active ? p_raw : g.P - 1;
    const int n = (int)(p / g.HoWo);
    const int r = (int)(p - (int64_t)n * g.HoWo);
    const int ho = r / g.Wo, wo = r - ho * g.Wo;
    const int hc = ho * g.stride, wc = wo * g.stride;
    const int co0 = blockIdx.y * F32_CO;

    int off[9];
    bool valid[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int h = hc + t / 3 - 1, w = wc + t % 3 - 1;
        valid[t] = (h >= 0) && (h < g.H) && (w >= 0) && (w < g.W);
        off[t] = valid[t] ? h * g.W + w : 0;
    }
    float acc[F32_CO];
#pragma unroll
    for (int j = 0; j < F32_CO; ++j) acc[j] = 0.0f;

    const int64_t plane = (int64_t)g.H * g.W;
    for (int ci0 = 0; ci0 < g.C_in; ci0 += F32_CI) {
        float xv[F32_CI][9];
#pragma unroll
        for (int c = 0; c < F32_CI; ++c) {
            const bool cok = ci0 + c < g.C_in;
            const float *src = x + ((int64_t)n * g.C_in + (cok ? ci0 + c : 0)) * plane;
#pragma unroll
            for (int t = 0; t < 9; ++t)
                xv[c][t] = (cok && valid[t]) ? src[off[t]] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < F32_CO; ++j) {
            const int co = min(co0 + j, g.C_out - 1);
#pragma unroll
            for (int c = 0; c < F32_CI; ++c) {
                const int ci = min(ci0 + c, g.C_in - 1);
                const uint32_t fl = flips[(int64_t)co * g.C_in + ci];   // wave-uniform
#pragma unroll
                for (int t = 0; t < 9; ++t)
                    acc[j] += __uint_as_float(__float_as_uint(xv[c][t]) ^ (((fl >> t) & 1u) << 31));
            }
        }
    }
    if (active) {
#pragma unroll
        for (int j = 0; j < F32_CO; ++j)
            if (co0 + j < g.C_out)
                store_output(y + ((int64_t)n * g.C_out + co0 + j) * g.HoWo + r, alpha[co0 + j] * acc[j]);
    }
}

}  // namespace

// Channel block and pixels per lane: aim for several waves per SIMD (>= 4096 waves).
struct BnnCfg {
    int PXL, COG;
};

BnnCfg bnn_cfg(const Geom &g)
{
    static const BnnCfg cands[] = {{2, 32}, {1, 32}, {1, 16}, {1, 8}};
    for (const BnnCfg &c : cands) {
        const int64_t waves = (g.P + 64 * c.PXL - 1) / (64 * c.PXL) * ((g.C_out + c.COG - 1) / c.COG);
        if (waves >= 4096) return c;
    }
    return cands[3];
}

size_t bnn_workspace_bytes(const Geom &g, int act)
{
    if (act == SNN_ACT_F32) return align_up((size_t)g.C_out * g.C_in * sizeof(uint32_t), 256);
    // room for either kernel's tables (channels rounded up to the largest channel block, words to a power of two)
    int CWT = 1;
    while (CWT < g.CW) CWT <<= 1;
    const int CWmax = g.CW <= 16 ? CWT : g.CW;
    const int COP = (g.C_out + 31) / 32 * 32;
    return align_up((size_t)COP * 9 * CWmax * sizeof(uint32_t), 256) + align_up((size_t)COP * 16 * sizeof(int32_t), 256);
}

int launch_bnn(const Geom &g, int act, const void *x, const uint16_t *w9, const float *alpha, float *y,
               void *ws, hipStream_t s, int phases)
{
    const bool prepare = (phases & SNN_PHASE_PREPARE) != 0, convolve = (phases & SNN_PHASE_CONVOLVE) != 0;
    const int64_t pblocks = (g.P + BNN_THREADS - 1) / BNN_THREADS;
    if (pblocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;

    if (act == SNN_ACT_F32) {
        uint32_t *flips = (uint32_t *)ws;
        const int64_t nk = (int64_t)g.C_out * g.C_in;
        const int cgroups = (g.C_out + F32_CO - 1) / F32_CO;
        if (cgroups > 65535) return SNN_ERR_UNSUPPORTED;
        if (prepare) hipLaunchKernelGGL(bnn_prep_f32_kernel, dim3((unsigned)((nk + 255) / 256)), dim3(256), 0, s, w9, nk, flips);
        if (convolve)
            hipLaunchKernelGGL(bnn_f32_kernel, dim3((unsigned)pblocks, (unsigned)cgroups), dim3(BNN_THREADS), 0, s,
                               (const float *)x, flips, alpha, y, g);
        return check_launch();
    }

    // (its window loads use 32-bit byte offsets whose top bit means "outside": packed inputs below 2 GiB)
    if (g.CW <= 16 && (int64_t)g.N * g.H * g.W * g.CW < ((int64_t)1 << 29) &&
        tuning(SNN_TUNE_BNN_REGS) != 0) {
        // register-resident windows (C_in <= 512)
        int CWT = 1;
        while (CWT < g.CW) CWT <<= 1;
        uint32_t *wplanes = (uint32_t *)ws;
        int32_t *corr = (int32_t *)((char *)ws + align_up((size_t)g.C_out * 9 * CWT * sizeof(uint32_t), 256));
        // channels per block: fewer than the kernel's chunk where the layer would not fill the chip otherwise
        int ch = bnn_regs_chunk(CWT);
        while (ch > 8 && pblocks * ((g.C_out + ch - 1) / ch) < 2048) ch /= 2;
        const int cgroups = (g.C_out + ch - 1) / ch;
        if (cgroups > 65535) return SNN_ERR_UNSUPPORTED;
        if (prepare)
            hipLaunchKernelGGL(bnn_prep_bin_kernel, dim3((unsigned)((g.C_out + 3) / 4)), dim3(256), 0, s, w9, g.C_out,
                               g.C_out, g.C_in, CWT, 1, wplanes, corr);
        if (!convolve) return check_launch();
        const dim3 grid((unsigned)pblocks, (unsigned)cgroups), block(BNN_THREADS);
        const uint32_t *xp = (const uint32_t *)x;
#define SNN_BNN_CASE(CWT_)                                                                                   \
    case CWT_:                                                                                               \
        hipLaunchKernelGGL(bnn_regs_kernel<CWT_>, grid, block, 0, s, xp, wplanes, corr, alpha, y, g, ch);     \
        break;
        switch (CWT) {
            SNN_BNN_CASE(1)
            SNN_BNN_CASE(2)
            SNN_BNN_CASE(4)
            SNN_BNN_CASE(8)
            SNN_BNN_CASE(16)
        }
#undef SNN_BNN_CASE
        return check_launch();
    }

    const BnnCfg c = bnn_cfg(g);
    const int COP = (g.C_out + c.COG - 1) / c.COG * c.COG;
    uint32_t *wq = (uint32_t *)ws;
    int32_t *corr = (int32_t *)((char *)ws + align_up((size_t)COP * 9 * g.CW * sizeof(uint32_t), 256));
    const int64_t pb = (g.P + (int64_t)BNN_THREADS * c.PXL - 1) / ((int64_t)BNN_THREADS * c.PXL);
    const int cgroups = COP / c.COG;
    if (pb > 0x7fffffffLL || cgroups > 65535) return SNN_ERR_UNSUPPORTED;
    // the kernel addresses the packed input with 32-bit word offsets
    if ((int64_t)g.N * g.H * g.W * g.CW >= ((int64_t)1 << 31)) return SNN_ERR_UNSUPPORTED;

    if (prepare)
        hipLaunchKernelGGL(bnn_prep_bin_kernel, dim3((unsigned)((COP + 3) / 4)), dim3(256), 0, s, w9, g.C_out, COP, g.C_in,
                           g.CW, c.COG, wq, corr);
    if (!convolve) return check_launch();

    const dim3 grid((unsigned)pb, (unsigned)cgroups), block(BNN_THREADS);
    const uint32_t *xp = (const uint32_t *)x;
    if (c.PXL == 2)
        hipLaunchKernelGGL((bnn_bin_kernel<2, 32>), grid, block, 0, s, xp, wq, corr, alpha, y, g);
    else if (c.COG == 32)
        hipLaunchKernelGGL((bnn_bin_kernel<1, 32>), grid, block, 0, s, xp, wq, corr, alpha, y, g);
    else if (c.COG == 16)
        hipLaunchKernelGGL((bnn_bin_kernel<1, 16>), grid, block, 0, s, xp, wq, corr, alpha, y, g);
    else
        hipLaunchKernelGGL((bnn_bin_kernel<1, 8>), grid, block, 0, s, xp, wq, corr, alpha, y, g);
    return check_launch();
}

}  // namespace snn
