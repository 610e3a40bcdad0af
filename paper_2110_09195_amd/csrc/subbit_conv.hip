// The sub-bit convolution of Sec. 4.5 / Fig. 6 on gfx950, +-1 activations (SNN_ACT_BIN_ROWS):
// dispatch, and the fallback kernel for what the matrix-core kernel does not take (more than 64
// subset members, notably the full set of 512 that cross-checks the 1-bit kernel; a single input
// channel with K <= 32; tensors beyond its 32-bit offsets).
//
// Fallback: stage 1 and stage 2 fused in one kernel, the K x c_in response maps never leave the
// chip.  A workgroup owns a tile of 64 consecutive output pixels and a block of output channels.
// Per chunk of input channels it builds, in LDS, the table T[ci][k][pixel] of MATCH COUNTS
// (9 - popcount(window ^ code_k), one byte per pixel, four pixels per 32-bit word); every lane
// then gathers 16-byte rows T[ci][idx[co][ci]][16 pixels] and adds them with plain 32-bit adds.
// Bytes are widened into 16-bit pairs every <= 28 input channels (28 * 9 = 252 < 256).  The
// response of a kernel is 2 * matches - taps, so
//     S = 2 * (M - corr[co][type]) - C_in * valid_taps(type)
// where M is the accumulated match count and corr removes the matches that taps outside the
// image (read as bit 0) fake; it depends only on the output channel and the pixel's border type.
#include <stdlib.h>

#include "subbit_common.h"

namespace snn {

namespace {

constexpr int SB_WIDEN = 28;         // input channels a byte accumulator can take (28 * 9 <= 255)

struct SbParams {
    const uint32_t *x;
    const uint32_t *codes;    // [512] window-order codes
    const uint16_t *offs;     // [chunks of 8][COP][8] row byte offsets (idx * 64)
    const int32_t *corr;      // [COP][16]
    const float *alpha;
    float *y;
    Geom g;
    int COP;
};

// ---- index preparation -------------------------------------------------------------------------
// One launch, two jobs (by block range):
//   offs[cc][co][cl] = min(idx[co][8 cc + cl], K - 1) * 64      (0 for padding)
//   corr[co][type]   = sum over c_in of the zero bits of the selected code at the taps that
//                      border type `type` puts outside the image
//   codes[k]         = code k in window order (tap t at bit t)
__global__ __launch_bounds__(256)
void subbit_prep_kernel(const uint16_t *__restrict__ codebook, const uint16_t *__restrict__ idx, int C_in,
                        int C_out, int COP, int K, int nchunks, int offs_blocks, uint32_t *__restrict__ codes,
                        uint16_t *__restrict__ offs, int32_t *__restrict__ corr)
{
    const int tid = threadIdx.x;
    if ((int)blockIdx.x < offs_blocks) {
        const int64_t gid = (int64_t)blockIdx.x * 256 + tid;
        const int64_t n_offs = (int64_t)nchunks * COP * 8;
        if (gid < n_offs) {
            const int cl = (int)(gid % 8);
            const int co = (int)((gid / 8) % COP);
            const int cc = (int)(gid / ((int64_t)8 * COP));
            const int ci = cc * 8 + cl;
            int k = 0;
            if (co < C_out && ci < C_in) k = min((int)idx[(int64_t)co * C_in + ci], K - 1);
            offs[gid] = (uint16_t)(k * 64);
        }
        return;
    }
    const int b = blockIdx.x - offs_blocks;
    const int co = b * 4 + (tid >> 6);          // one wave per output channel
    const int lane = tid & 63;
    if (b == 0)
        for (int k = tid; k < 512; k += 256) codes[k] = k < K ? code_to_window_order(codebook[k] & 511u) : 0u;
    if (co >= COP) return;
    int zeros[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) zeros[t] = 0;
    if (co < C_out)
        for (int c0 = 0; c0 < C_in; c0 += 64) {
            const int ci = c0 + lane;
            uint32_t z = 0;
            if (ci < C_in) {
                const int k = min((int)idx[(int64_t)co * C_in + ci], K - 1);
                z = ~code_to_window_order(codebook[k] & 511u) & 511u;
            }
#pragma unroll
            for (int t = 0; t < 9; ++t) zeros[t] += __popcll(__ballot((z >> t) & 1u));
        }
    if (lane < 16) {
        const uint32_t inv = border_invalid_window(lane);
        int s = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t)
            if ((inv >> t) & 1u) s += zeros[t];
        corr[co * 16 + lane] = s;
    }
}

// ---- the kernel: lanes = 16 output channels x 4 groups of 16 pixels, J channel sets per lane, NW waves -----

template <int J, int NW>
__global__ __launch_bounds__(NW * 64)
void subbit_direct_kernel(const SbParams p, int CIC)
{
    constexpr int NT = NW * 64;
    constexpr int G = 4, TP = 64, CL = 16;
    constexpr int COW = CL * J;
    const Geom &g = p.g;
    const int K = g.K;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *T = smem;                                              // [CIC][K][TP]
    uint16_t *wins = (uint16_t *)(smem + (size_t)CIC * K * TP);           // [CIC][TP]
    uint32_t *lcodes = (uint32_t *)(wins + CIC * TP);                     // [K]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t p_tile = (int64_t)blockIdx.x * TP;
    const int gq = lane % G, cl = lane / G;
    const int lane_co = blockIdx.y * (COW * NW) + wave * COW + cl * J;

    for (int i = tid; i < K; i += NT) lcodes[i] = p.codes[i];
    const PixGeom geo = pix_geom(p_tile + (tid & 63), g);

    uint32_t acc[J][4], wide_e[J][4], wide_o[J][4];
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[j][w] = wide_e[j][w] = wide_o[j][w] = 0;
    int since_widen = 0;
    __syncthreads();

    // offsets are laid out for chunks of 8: [chunk8][COP][8]
    for (int c0 = 0; c0 < g.C_in; c0 += CIC) {
        const int nci = min(CIC, g.C_in - c0);
        for (int ci_l = tid >> 6; ci_l < nci; ci_l += NW)
            wins[ci_l * TP + (tid & 63)] = (uint16_t)window9(p.x, geo, c0 + ci_l, g);
        __syncthreads();
        const int items = nci * K * (TP / 4);
        for (int i = tid; i < items; i += NT) {
            const int wd = i & 15;
            const int k = (i >> 4) % K;
            const int ci_l = (i >> 4) / K;
            const uint2 w4 = *(const uint2 *)(wins + ci_l * TP + 4 * wd);
            const uint32_t code = lcodes[k];
            const uint32_t m0 = 9u - __popc((w4.x & 0xffffu) ^ code);
            const uint32_t m1 = 9u - __popc((w4.x >> 16) ^ code);
            const uint32_t m2 = 9u - __popc((w4.y & 0xffffu) ^ code);
            const uint32_t m3 = 9u - __popc((w4.y >> 16) ^ code);
            ((uint32_t *)T)[i] = m0 | (m1 << 8) | (m2 << 16) | (m3 << 24);
        }
        __syncthreads();
        if (since_widen + nci > SB_WIDEN) {
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
                    wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
                    acc[j][w] = 0;
                }
            since_widen = 0;
        }
        since_widen += nci;
        const unsigned char *Tl = T + gq * 16;
        for (int ci_l = 0; ci_l < nci; ++ci_l) {
            const int ci = c0 + ci_l;
            const uint16_t *op = p.offs + ((int64_t)(ci >> 3) * p.COP + lane_co) * 8 + (ci & 7);
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint4 v = *(const uint4 *)(Tl + op[j * 8]);
                acc[j][0] += v.x;
                acc[j][1] += v.y;
                acc[j][2] += v.z;
                acc[j][3] += v.w;
            }
            Tl += (size_t)K * TP;
        }
        __syncthreads();
    }

#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
            wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
        }
    const int64_t pl = p_tile + gq * 16;
    if (pl >= g.P) return;
    int n = (int)(pl / g.HoWo);
    int r = (int)(pl - (int64_t)n * g.HoWo);
    int ho = r / g.Wo, wo = r - ho * g.Wo;
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const bool ok = pl + 4 * w + b < g.P;
            const int type = border_type(ho, wo, g.H, g.W, g.stride);
            const int base = border_valid_taps(type) * g.C_in;
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int co = lane_co + j;
                if (ok && co < g.C_out) {
                    const uint32_t pair = (b & 1) ? wide_o[j][w] : wide_e[j][w];
                    const int M = (int)((pair >> (16 * (b >> 1))) & 0xffffu);
                    const int S = 2 * (M - p.corr[co * 16 + type]) - base;
                    store_output(p.y + ((int64_t)n * g.C_out + co) * g.HoWo + r, (float)S * p.alpha[co]);
                }
            }
            if (++wo == g.Wo) {
                wo = 0;
                if (++ho == g.Ho) ho = 0;
            }
            if (++r == g.HoWo) {
                r = 0;
                ++n;
            }
        }
}

// ---- configuration ------------------------------------------------------------------------------------

struct SbCfg {
    int J, NW;
    int cob() const { return 16 * J * NW; }     // output channels per workgroup
};

struct SbPlan {
    SbCfg cfg;
    int CIC;          // input channels per chunk
    int COP;          // C_out padded to whole channel blocks
    int nchunks;      // chunks of 8 channels of the offsets table
    size_t lds;
    size_t off_codes, off_offs, off_corr, bytes;    // workspace carve-up
};

SbPlan make_plan(const Geom &g)
{
    static const SbCfg cfgs[] = {{1, 1}, {1, 2}, {1, 4}, {2, 4}, {4, 4}};
    SbPlan pl;
    pl.cfg = cfgs[4];                            // several channel blocks of the largest one beyond 256 channels
    for (const SbCfg &c : cfgs)
        if (g.C_out <= c.cob()) {
            pl.cfg = c;
            break;
        }
    int CIC = 8;
    while (CIC > 1 && (size_t)CIC * g.K * 64 > 32 * 1024) CIC >>= 1;
    pl.CIC = CIC;
    pl.lds = (size_t)CIC * g.K * 64 + (size_t)CIC * 64 * sizeof(uint16_t) + (size_t)g.K * sizeof(uint32_t);
    pl.nchunks = (g.C_in + 7) / 8;
    pl.COP = (g.C_out + pl.cfg.cob() - 1) / pl.cfg.cob() * pl.cfg.cob();
    size_t o = 0;
    pl.off_codes = o;
    o += align_up(512 * sizeof(uint32_t), 256);
    pl.off_offs = o;
    o += align_up((size_t)pl.nchunks * pl.COP * 8 * sizeof(uint16_t), 256);
    pl.off_corr = o;
    o += align_up((size_t)pl.COP * 16 * sizeof(int32_t), 256);
    pl.bytes = o;
    return pl;
}

template <int J, int NW>
int launch_direct(const SbPlan &pl, const SbParams &prm, dim3 grid, hipStream_t s)
{
    auto kern = subbit_direct_kernel<J, NW>;
    static LdsGrant grant;
    if (grant_dynamic_lds((const void *)kern, pl.lds, grant) != SNN_OK) return SNN_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), pl.lds, s, prm, pl.CIC);
    return check_launch();
}

// The matrix-core kernel takes every layer it supports; the knob SNN_TUNE_SUBBIT_MFMA = 0 (tuning and tests)
// sends those layers to the fallback kernel instead.
bool use_mfma(const Geom &g)
{
    return subbit_mfma_supported(g) && tuning(SNN_TUNE_SUBBIT_MFMA) != 0;
}

}  // namespace

int launch_subbit_f32(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *idx,
                      const float *alpha, float *y, void *ws, hipStream_t s, int phases);
size_t subbit_f32_workspace_bytes(const Geom &g);

int subbit_slots_per_channel(const Geom &g, int act)
{
    if (act == SNN_ACT_F32 || !use_mfma(g)) return 0;
    return subbit_mfma_slots_per_channel(g);
}

size_t subbit_workspace_bytes(const Geom &g, int act)
{
    if (act == SNN_ACT_F32) return subbit_f32_workspace_bytes(g);
    // sized for either kernel, so that the override cannot outgrow a workspace
    const size_t a = make_plan(g).bytes;
    const size_t b = subbit_mfma_supported(g) ? subbit_mfma_workspace_bytes(g) : 0;
    return a > b ? a : b;
}

int launch_subbit(const Geom &g, int act, const void *x, const uint16_t *codebook, const uint16_t *idx,
                  const float *alpha, float *y, void *ws, hipStream_t s, int phases)
{
    if (act == SNN_ACT_F32) return launch_subbit_f32(g, x, codebook, idx, alpha, y, ws, s, phases);
    if (use_mfma(g)) return launch_subbit_mfma(g, x, codebook, idx, alpha, y, ws, s, nullptr, phases);

    const SbPlan pl = make_plan(g);
    const SbCfg &c = pl.cfg;
    const int64_t tiles = (g.P + 63) / 64;
    const int cblocks = pl.COP / c.cob();
    if (tiles > 0x7fffffffLL || cblocks > 65535 || pl.lds > 160 * 1024) return SNN_ERR_UNSUPPORTED;
    // the kernel addresses the packed input with 32-bit word offsets
    if ((int64_t)g.N * g.C_in * g.H * g.WW >= ((int64_t)1 << 31)) return SNN_ERR_UNSUPPORTED;

    SbParams prm;
    prm.x = (const uint32_t *)x;
    prm.codes = (const uint32_t *)((char *)ws + pl.off_codes);
    prm.offs = (const uint16_t *)((char *)ws + pl.off_offs);
    prm.corr = (const int32_t *)((char *)ws + pl.off_corr);
    prm.alpha = alpha;
    prm.y = y;
    prm.g = g;
    prm.COP = pl.COP;

    const int64_t n_offs = (int64_t)pl.nchunks * pl.COP * 8;
    const int offs_blocks = (int)((n_offs + 255) / 256);
    const int corr_blocks = (pl.COP + 3) / 4;
    if (phases & SNN_PHASE_PREPARE)
        hipLaunchKernelGGL(subbit_prep_kernel, dim3((unsigned)(offs_blocks + corr_blocks)), dim3(256), 0, s, codebook, idx,
                           g.C_in, g.C_out, pl.COP, g.K, pl.nchunks, offs_blocks, (uint32_t *)prm.codes,
                           (uint16_t *)prm.offs, (int32_t *)prm.corr);
    if (!(phases & SNN_PHASE_CONVOLVE)) return check_launch();

    const dim3 grid((unsigned)tiles, (unsigned)cblocks);
    if (c.J == 1 && c.NW == 1) return launch_direct<1, 1>(pl, prm, grid, s);
    if (c.J == 1 && c.NW == 2) return launch_direct<1, 2>(pl, prm, grid, s);
    if (c.J == 1 && c.NW == 4) return launch_direct<1, 4>(pl, prm, grid, s);
    if (c.J == 2 && c.NW == 4) return launch_direct<2, 4>(pl, prm, grid, s);
    return launch_direct<4, 4>(pl, prm, grid, s);
}

// ---- one layer's forward pass in one call -----------------------------------------------------------
// Workspace: [the convolution's own workspace][packed rows of sign(x)].
size_t subbit_forward_workspace_bytes(const Geom &g)
{
    return align_up(subbit_workspace_bytes(g, SNN_ACT_BIN_ROWS), 256) +
           align_up((size_t)g.N * g.C_in * g.H * g.WW * sizeof(uint32_t), 256);
}

int launch_subbit_forward(const Geom &g, const float *x, const float *w, const uint16_t *codebook,
                          const float *alpha, uint16_t *idx_out, float *y, void *ws, hipStream_t s)
{
    uint32_t *xr = (uint32_t *)((char *)ws + align_up(subbit_workspace_bytes(g, SNN_ACT_BIN_ROWS), 256));
    if (use_mfma(g)) return launch_subbit_forward_mfma(g, x, w, codebook, alpha, idx_out, y, xr, ws, s);
    // layers the matrix-core kernel does not take: the three operations one after the other
    int rc = launch_pack_rows(x, xr, (int64_t)g.N * g.C_in * g.H, g.W, s);
    if (rc != SNN_OK) return rc;
    rc = launch_project(w, (int64_t)g.C_out * g.C_in, codebook, g.K, idx_out, s);
    if (rc != SNN_OK) return rc;
    return launch_subbit(g, SNN_ACT_BIN_ROWS, xr, codebook, idx_out, alpha, y, ws, s);
}

// ---- convolution + the next layer's binarisation --------------------------------------------------------
int launch_subbit_sign(const Geom &g, const void *x_packed, const uint16_t *codebook, const uint16_t *idx,
                       const float *alpha, const float *beta, uint32_t *out_packed, void *ws, hipStream_t s, int phases)
{
    if (!use_mfma(g)) return SNN_ERR_UNSUPPORTED;
    // the convolution alone needs only the output pointer; a non-null epilogue selects the sign form either way
    const SignEpilogue sign = {beta, out_packed};
    return launch_subbit_mfma(g, x_packed, codebook, idx, alpha, nullptr, ws, s, &sign, phases);
}

int launch_subbit_forward_sign(const Geom &g, const void *x_packed, const float *w, const uint16_t *codebook,
                               const float *alpha, const float *beta, uint16_t *idx_out, uint32_t *out_packed, void *ws,
                               hipStream_t s)
{
    if (!use_mfma(g)) return SNN_ERR_UNSUPPORTED;
    const SignEpilogue sign = {beta, out_packed};
    return launch_subbit_forward_mfma(g, nullptr, w, codebook, alpha, idx_out, nullptr, (uint32_t *)x_packed, ws, s, &sign);
}

}  // namespace snn
