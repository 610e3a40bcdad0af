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

template <int J, int NW>
__global__ __launch_bounds__(NW * 64)
void subbit_f32_kernel(const float *__restrict__ x, const uint32_t *__restrict__ codes,
                       const uint16_t *__restrict__ offs, const float *__restrict__ alpha,
                       float *__restrict__ y, Geom g, int COP, int CIC)
{
    constexpr int NT = NW * 64;
    constexpr int COW = SF_CL * J;
    extern __shared__ __align__(16) unsigned char smem[];
    const int K = g.K;
    float *T = (float *)smem;                               // [CIC][K][TP]
    float *coef = T + (size_t)CIC * K * SF_TP;              // [K][9] +-1

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t p_tile = (int64_t)blockIdx.x * SF_TP;

    for (int i = tid; i < K * 9; i += NT) {
        const int k = i / 9, t = i - 9 * k;
        coef[i] = ((codes[k] >> t) & 1u) ? 1.0f : -1.0f;    // window order: tap t is bit t
    }

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

    for (int c0 = 0; c0 < g.C_in; c0 += CIC) {
        const int nci = min(CIC, g.C_in - c0);
        // stage 1: nine add/subtracts per (pixel, ci, k)
        for (int ci_l = tid >> 6; ci_l < nci; ci_l += NW) {
            const float *src = x + ((int64_t)n1 * g.C_in + c0 + ci_l) * plane;
            float xv[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) xv[t] = ok9[t] ? src[off9[t]] : 0.0f;
            float *Tw = T + (size_t)ci_l * K * SF_TP + (tid & 63);
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
            const uint16_t *op = offs + (int64_t)c0 * COP + lane_co;
            for (int ci_l = 0; ci_l < nci; ++ci_l) {
#pragma unroll
                for (int j = 0; j < J; ++j) {
                    // offs holds idx * 64 (row bytes of the packed kernel); a row here is 64 floats
                    const float4 v = *(const float4 *)(Tl + op[j]);
                    acc[j][0] += v.x;
                    acc[j][1] += v.y;
                    acc[j][2] += v.z;
                    acc[j][3] += v.w;
                }
                Tl += (size_t)K * SF_TP;
                op += COP;
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

struct F32Cfg { int J, NW, COB; };

F32Cfg pick_f32_cfg(int C_out)
{
    static const F32Cfg cfgs[] = {{1, 4, 16}, {2, 4, 32}, {4, 4, 64}, {8, 4, 128}};
    for (const F32Cfg &c : cfgs)
        if (C_out <= c.COB) return c;
    return cfgs[3];
}

// offs[ci][co] = min(idx[co][ci], K-1) * 64 (floats per row of T); codes[k] in window order.
__global__ __launch_bounds__(256)
void subbit_f32_prep_kernel(const uint16_t *__restrict__ codebook, const uint16_t *__restrict__ idx, int C_in,
                            int C_out, int COP, int K, uint32_t *__restrict__ codes, uint16_t *__restrict__ offs)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n_offs = (int64_t)C_in * COP;
    if (gid < n_offs) {
        const int ci = (int)(gid / COP), co = (int)(gid - (int64_t)ci * COP);
        const int k = co < C_out ? min((int)idx[(int64_t)co * C_in + ci], K - 1) : 0;
        offs[gid] = (uint16_t)(k * SF_TP);
    } else if (gid < n_offs + 512) {
        const int k = (int)(gid - n_offs);
        codes[k] = k < K ? code_to_window_order(codebook[k] & 511u) : 0u;
    }
}

}  // namespace

size_t subbit_f32_workspace_bytes(const Geom &g)
{
    const F32Cfg c = pick_f32_cfg(g.C_out);
    const int COP = (g.C_out + c.COB - 1) / c.COB * c.COB;
    return align_up(512 * sizeof(uint32_t), 256) + align_up((size_t)g.C_in * COP * sizeof(uint16_t), 256);
}

int launch_subbit_f32(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *idx,
                      const float *alpha, float *y, void *ws, hipStream_t s, int phases)
{
    const F32Cfg c = pick_f32_cfg(g.C_out);
    const int COP = (g.C_out + c.COB - 1) / c.COB * c.COB;
    uint32_t *codes = (uint32_t *)ws;
    uint16_t *offs = (uint16_t *)((char *)ws + align_up(512 * sizeof(uint32_t), 256));
    const int64_t tiles = (g.P + SF_TP - 1) / SF_TP;
    const int cblocks = COP / c.COB;
    if (tiles > 0x7fffffffLL || cblocks > 65535) return SNN_ERR_UNSUPPORTED;
    int CIC = 8;
    while (CIC > 1 && (size_t)CIC * g.K * SF_TP * sizeof(float) > 48 * 1024) CIC >>= 1;
    const size_t lds = (size_t)CIC * g.K * SF_TP * sizeof(float) + (size_t)g.K * 9 * sizeof(float);
    if (lds > 160 * 1024) return SNN_ERR_UNSUPPORTED;
    const int64_t nprep = (int64_t)g.C_in * COP + 512;
    if (phases & SNN_PHASE_PREPARE)
        hipLaunchKernelGGL(subbit_f32_prep_kernel, dim3((unsigned)((nprep + 255) / 256)), dim3(256), 0, s, codebook, idx,
                           g.C_in, g.C_out, COP, g.K, codes, offs);
    if (!(phases & SNN_PHASE_CONVOLVE)) return check_launch();
    const dim3 grid((unsigned)tiles, (unsigned)cblocks);
#define SNN_F32_CASE(J_)                                                                                       \
    case J_: {                                                                                                 \
        auto kern = subbit_f32_kernel<J_, 4>;                                                                  \
        static LdsGrant grant;                                                                                 \
        if (grant_dynamic_lds((const void *)kern, lds, grant) != SNN_OK) return SNN_ERR_LAUNCH;                \
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, (const float *)x, codes, offs, alpha, y, g, COP,     \
                           CIC);                                                                               \
    } break;
    switch (c.J) {
        SNN_F32_CASE(1)
        SNN_F32_CASE(2)
        SNN_F32_CASE(4)
        SNN_F32_CASE(8)
    default:
        return SNN_ERR_UNSUPPORTED;
    }
#undef SNN_F32_CASE
    return check_launch();
}

}  // namespace snn
