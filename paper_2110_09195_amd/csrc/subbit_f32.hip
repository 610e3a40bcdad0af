// The sub-bit convolution of Sec. 4.5 / Fig. 6 with real-valued activations (SNN_ACT_F32; the
// W/A = x/32 models of Tables 1-2 and the deployment test of Table 4).
//
// Same two stages as the +-1 kernel: per chunk of input channels the workgroup builds
// T[ci][k][pixel] in LDS (nine add/subtracts of the window's values per response, as
// fma(x, +-1, acc)), then every lane gathers float4 rows T[ci][idx[co][ci]][4 pixels] and adds
// them in fp32.  y = alpha * S.
#include "subbit_common.h"

namespace snn {

namespace {

constexpr int SF_TP = 64;    // pixels per tile; a row of T is 64 floats
constexpr int SF_G = 16;     // float4 groups per row
constexpr int SF_CL = 4;     // output channels per wave instruction

// Largest chunk of input channels a workgroup stages at once: one channel per wave and chunk where the registers
// for the chunk's gather offsets allow it.
template <int J, int NW>
struct SfChunk { static constexpr int max = (NW >= 16 && J <= 4) ? 16 : 8; };

template <int J, int NW>
__global__ __launch_bounds__(NW * 64)
void subbit_f32_kernel(const float *__restrict__ x, const float *__restrict__ coef,
                       const uint16_t *__restrict__ offs, const float *__restrict__ alpha,
                       float *__restrict__ y, Geom g, int COP, int CIC)
{
    constexpr int COW = SF_CL * J;
    extern __shared__ __align__(16) unsigned char smem[];
    const int K = g.K;
    float *T = (float *)smem;                               // [CIC][K][TP]
    // coef[K][9] (+-1.0f, window order) stays in memory: its index is wave-uniform, so the nine coefficients of a
    // member arrive through the scalar cache and are scalar operands of the multiply-adds (read from LDS they were
    // 288 broadcast reads per input channel and thread, and the loop waited for every one of them)

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t p_tile = (int64_t)blockIdx.x * SF_TP;

    // stage-1 geometry: this thread always evaluates pixel (tid & 63) of the tile
    int off9[9];
    bool ok9[9];
    int n1;
    {
        int64_t p = p_tile + (tid & 63);
        if (p >= g.P) p = g.P - 1;
        n1 = (int)(p / g.HoWo);
        const int r = (int)(p - (int64_t)n1 * g.HoWo);
        const int ho = r / g.Wo, wo = r - ho * g.Wo;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int h = ho * g.stride + t / 3 - 1, w = wo * g.stride + t % 3 - 1;
            ok9[t] = h >= 0 && h < g.H && w >= 0 && w < g.W;
            off9[t] = ok9[t] ? h * g.W + w : 0;
        }
    }

    float acc[J][4];
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[j][w] = 0.0f;

    const int g16 = lane & (SF_G - 1);
    const int cl = lane / SF_G;
    const int lane_co = blockIdx.y * (COW * NW) + wave * COW + cl * J;
    const int64_t plane = (int64_t)g.H * g.W;

    __syncthreads();

    // window of the wave's first channel of the first chunk (every later one is requested a chunk ahead)
    float xnext[9];
    {
        const float *src0 = x + ((int64_t)n1 * g.C_in + min(tid >> 6, g.C_in - 1)) * plane;
#pragma unroll
        for (int t = 0; t < 9; ++t) xnext[t] = ok9[t] ? src0[off9[t]] : 0.0f;
    }

    for (int c0 = 0; c0 < g.C_in; c0 += CIC) {
        const int nci = min(CIC, g.C_in - c0);
        // the gather offsets of this chunk are requested before stage 1 and used after it (a dependent global load
        // per gather in stage 2 was most of the kernel's time at one wave per SIMD)
        constexpr int CIC_MAX = SfChunk<J, NW>::max;
        uint16_t ofs[CIC_MAX][J];
        {
            const uint16_t *op = offs + (int64_t)c0 * COP + lane_co;
#pragma unroll
            for (int ci_l = 0; ci_l < CIC_MAX; ++ci_l)
#pragma unroll
                for (int j = 0; j < J; ++j) ofs[ci_l][j] = ci_l < nci ? op[(int64_t)ci_l * COP + j] : (uint16_t)0;
        }
        // stage 1: nine add/subtracts per (pixel, ci, k)
        for (int ci_l = tid >> 6; ci_l < nci; ci_l += NW) {
            float xv[9];
            if (ci_l == (tid >> 6)) {
                // the wave's first channel of the chunk was requested a chunk ahead; now the next chunk's
#pragma unroll
                for (int t = 0; t < 9; ++t) xv[t] = xnext[t];
                const int cn = c0 + CIC + (tid >> 6);
                const float *srcn = x + ((int64_t)n1 * g.C_in + min(cn, g.C_in - 1)) * plane;
#pragma unroll
                for (int t = 0; t < 9; ++t) xnext[t] = ok9[t] ? srcn[off9[t]] : 0.0f;
            } else {
                const float *src = x + ((int64_t)n1 * g.C_in + c0 + ci_l) * plane;
#pragma unroll
                for (int t = 0; t < 9; ++t) xv[t] = ok9[t] ? src[off9[t]] : 0.0f;
            }
            float *Tw = T + (size_t)ci_l * K * SF_TP + (tid & 63);
#pragma unroll 4
            for (int k = 0; k < K; ++k) {
                const float *ck = coef + k * 9;
                float s = 0.0f;
#pragma unroll
                for (int t = 0; t < 9; ++t) s = __builtin_fmaf(xv[t], ck[t], s);
                Tw[k * SF_TP] = s;
            }
        }
        __syncthreads();
        // stage 2
        {
            const float *Tl = T + g16 * 4;
#pragma unroll
            for (int ci_l = 0; ci_l < CIC_MAX; ++ci_l) {
                if (ci_l < nci) {
#pragma unroll
                    for (int j = 0; j < J; ++j) {
                        // offs holds idx * 64 (row bytes of the packed kernel); a row here is 64 floats
                        const float4 v = *(const float4 *)(Tl + ofs[ci_l][j]);
                        acc[j][0] += v.x;
                        acc[j][1] += v.y;
                        acc[j][2] += v.z;
                        acc[j][3] += v.w;
                    }
                }
                Tl += (size_t)K * SF_TP;
            }
        }
        __syncthreads();
    }

    const int64_t p0 = p_tile + g16 * 4;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int64_t p = p0 + b;
        if (p >= g.P) break;
        const int n = (int)(p / g.HoWo);
        const int r = (int)(p - (int64_t)n * g.HoWo);
#pragma unroll
        for (int j = 0; j < J; ++j)
            if (lane_co + j < g.C_out)
                store_output(y + ((int64_t)n * g.C_out + lane_co + j) * g.HoWo + r, alpha[lane_co + j] * acc[j][b]);
    }
}

struct F32Cfg { int J, NW, COB, CIC; size_t lds; };

// J output channels per lane, NW waves: a workgroup covers COB = 4 * J * NW output channels, and stage 1 is
// repeated once per group of COB, so COB should reach C_out.  Few pixel tiles (a small image or batch) want many
// waves per workgroup, since a tile is then all a compute unit has to hide its latencies with; many tiles want
// several small workgroups per unit, which overlap each other's barriers.
F32Cfg pick_f32_cfg(const Geom &g)
{
    const int64_t tiles = (g.P + SF_TP - 1) / SF_TP;
    int NW = tiles <= 512 ? 16 : tiles <= 2048 ? 8 : 4;
    const int forced = tuning(SNN_TUNE_F32_WAVES);
    if (forced == 4 || forced == 8 || forced == 16) NW = forced;
    int J = 1;
    while (J < 8 && 4 * J * NW < g.C_out) J <<= 1;
    while (NW > 4 && J == 1 && 4 * (NW / 2) >= g.C_out) NW >>= 1;     // no wave without output channels
    F32Cfg c;
    c.J = J;
    c.NW = NW;
    c.COB = 4 * J * NW;
    const size_t budget = NW >= 16 ? 128 * 1024 : NW >= 8 ? 64 * 1024 : 48 * 1024;
    c.CIC = (NW >= 16 && J <= 4) ? 16 : 8;
    while (c.CIC > 1 && (size_t)c.CIC * g.K * SF_TP * sizeof(float) > budget) c.CIC >>= 1;
    c.lds = (size_t)c.CIC * g.K * SF_TP * sizeof(float);
    return c;
}

// offs[ci][co] = min(idx[co][ci], K-1) * 64 (floats per row of T); codes[k] in window order.
__global__ __launch_bounds__(256)
void subbit_f32_prep_kernel(const uint16_t *__restrict__ codebook, const uint16_t *__restrict__ idx, int C_in,
                            int C_out, int COP, int K, uint32_t *__restrict__ codes, float *__restrict__ coef,
                            uint16_t *__restrict__ offs)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n_offs = (int64_t)C_in * COP;
    if (gid < n_offs) {
        const int ci = (int)(gid / COP), co = (int)(gid - (int64_t)ci * COP);
        const int k = co < C_out ? min((int)idx[(int64_t)co * C_in + ci], K - 1) : 0;
        offs[gid] = (uint16_t)(k * SF_TP);
    } else if (gid < n_offs + 512) {
        const int k = (int)(gid - n_offs);
        const uint32_t c = k < K ? code_to_window_order(codebook[k] & 511u) : 0u;
        codes[k] = c;
        for (int t = 0; t < 9; ++t) coef[k * 9 + t] = ((c >> t) & 1u) ? 1.0f : -1.0f;    // window order: tap t is bit t
    }
}

}  // namespace

size_t subbit_f32_workspace_bytes(const Geom &g)
{
    // the widest padding of C_out any launch shape uses (the shape may change with the tuning knob between the
    // size query and the call)
    const int COP = (g.C_out + 511) / 512 * 512;
    return align_up(512 * sizeof(uint32_t), 256) + align_up(512 * 9 * sizeof(float), 256) + align_up((size_t)g.C_in * COP * sizeof(uint16_t), 256);
}

int launch_subbit_f32(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *idx,
                      const float *alpha, float *y, void *ws, hipStream_t s, int phases)
{
    const F32Cfg c = pick_f32_cfg(g);
    const int COP = (g.C_out + c.COB - 1) / c.COB * c.COB;
    uint32_t *codes = (uint32_t *)ws;
    float *coef = (float *)((char *)ws + align_up(512 * sizeof(uint32_t), 256));
    uint16_t *offs = (uint16_t *)((char *)coef + align_up(512 * 9 * sizeof(float), 256));
    const int64_t tiles = (g.P + SF_TP - 1) / SF_TP;
    const int cblocks = COP / c.COB;
    if (tiles > 0x7fffffffLL || cblocks > 65535) return SNN_ERR_UNSUPPORTED;
    const int CIC = c.CIC;
    const size_t lds = c.lds;
    if (lds > 160 * 1024) return SNN_ERR_UNSUPPORTED;
    const int64_t nprep = (int64_t)g.C_in * COP + 512;
    if (phases & SNN_PHASE_PREPARE)
        hipLaunchKernelGGL(subbit_f32_prep_kernel, dim3((unsigned)((nprep + 255) / 256)), dim3(256), 0, s, codebook, idx,
                           g.C_in, g.C_out, COP, g.K, codes, coef, offs);
    if (!(phases & SNN_PHASE_CONVOLVE)) return check_launch();
    const dim3 grid((unsigned)tiles, (unsigned)cblocks);
#define SNN_F32_CASE(J_, NW_)                                                                                  \
    case J_ * 100 + NW_: {                                                                                     \
        auto kern = subbit_f32_kernel<J_, NW_>;                                                                \
        static LdsGrant grant;                                                                                 \
        if (grant_dynamic_lds((const void *)kern, lds, grant) != SNN_OK) return SNN_ERR_LAUNCH;                \
        hipLaunchKernelGGL(kern, grid, dim3(NW_ * 64), lds, s, (const float *)x, coef, offs, alpha, y, g, COP, \
                           CIC);                                                                               \
    } break;
    switch (c.J * 100 + c.NW) {
        SNN_F32_CASE(1, 4)
        SNN_F32_CASE(2, 4)
        SNN_F32_CASE(4, 4)
        SNN_F32_CASE(8, 4)
        SNN_F32_CASE(1, 8)
        SNN_F32_CASE(2, 8)
        SNN_F32_CASE(4, 8)
        SNN_F32_CASE(8, 8)
        SNN_F32_CASE(1, 16)
        SNN_F32_CASE(2, 16)
        SNN_F32_CASE(4, 16)
        SNN_F32_CASE(8, 16)
    default:
        return SNN_ERR_UNSUPPORTED;
    }
#undef SNN_F32_CASE
    return check_launch();
}

}  // namespace snn
