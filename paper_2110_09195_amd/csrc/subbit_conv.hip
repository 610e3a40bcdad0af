// The sub-bit convolution of Sec. 4.5 / Fig. 6 on gfx950.
//
// Stage 1 (each input channel x each of the K subset kernels) and stage 2 (per output channel,
// gather the responses its indices select and sum them along c_in) run fused in one kernel; the
// K x c_in response maps never leave the chip.
//
// +-1 activations (SNN_ACT_BIN_ROWS)
//   A workgroup owns a tile of TP = 64 consecutive output pixels and a block of output channels.
//   Per chunk of input channels it builds, in LDS, the table T[ci][k][pixel] of MATCH COUNTS
//   (0..9, one byte per pixel, so four pixels share a 32-bit word), then every lane gathers
//   16-byte rows T[ci][idx[co][ci]][16 pixels] and adds them with plain 32-bit adds: one
//   v_add_u32 accumulates four pixels.  Bytes are widened into 16-bit pairs every <= 28 input
//   channels (28 * 9 = 252 < 256).  The response of a kernel is 2 * matches - taps, so
//       S = 2 * (M - corr[co][type]) - C_in * valid_taps(type)
//   where M is the accumulated match count, and corr removes the matches that taps outside the
//   image (read as bit 0) fake; it depends only on the output channel and the pixel's border type.
//   Stage 1 is a 512-entry table lookup (window -> K match counts) for K <= 64, a direct
//   XOR + popcount otherwise.
//
// fp32 activations (SNN_ACT_F32): same structure, T holds fp32 responses (add/subtract of the nine
//   taps), stage 2 gathers float4 rows.
#include "snn_internal.h"

namespace snn {

namespace {

constexpr int SB_G = 4;              // 16-pixel groups per tile
constexpr int SB_TP = 16 * SB_G;     // pixels per tile
constexpr int SB_CL = 64 / SB_G;     // output channels served by one wave instruction
constexpr int SB_WIDEN = 28;         // input channels a byte accumulator can take (28 * 9 <= 255)
constexpr int SB_LUT_MAXK = 64;

// workspace: codes [512] u32 (window order) | offs [C_in][COP] u16 (idx * row bytes) |
//            corr [COP][16] i32
struct SubbitWs {
    uint32_t *codes;
    uint16_t *offs;
    int32_t *corr;
    int COP;          // C_out padded to the channel block of the kernel configuration
    size_t bytes;
};

struct SubbitCfg {
    int J, NW;        // accumulator sets per lane, waves per workgroup
    int COB;          // output channels per workgroup = SB_CL * J * NW
};

SubbitCfg pick_cfg(int C_out)
{
    static const SubbitCfg cfgs[] = {{1, 1, 16}, {1, 2, 32}, {1, 4, 64}, {2, 4, 128}, {4, 4, 256}};
    for (const SubbitCfg &c : cfgs)
        if (C_out <= c.COB) return c;
    return cfgs[4];
}

SubbitWs carve_ws(const Geom &g, void *ws)
{
    const SubbitCfg c = pick_cfg(g.C_out);
    SubbitWs w;
    w.COP = (g.C_out + c.COB - 1) / c.COB * c.COB;
    size_t o = 0;
    w.codes = (uint32_t *)((char *)ws + o);
    o += align_up(512 * sizeof(uint32_t), 256);
    w.offs = (uint16_t *)((char *)ws + o);
    o += align_up((size_t)g.C_in * w.COP * sizeof(uint16_t), 256);
    w.corr = (int32_t *)((char *)ws + o);
    o += align_up((size_t)w.COP * 16 * sizeof(int32_t), 256);
    w.bytes = o;
    return w;
}

// codes[k] in window order; offs[ci][co] = min(idx, K-1) * row_bytes (0 for padded channels);
// corr[co][type] = sum_ci popcount(~code[idx] & taps outside the image).
__global__ void subbit_prep_kernel(const uint16_t *__restrict__ codebook, const uint16_t *__restrict__ idx,
                                   int C_in, int C_out, int COP, int K, int row_bytes,
                                   uint32_t *__restrict__ codes, uint16_t *__restrict__ offs,
                                   int32_t *__restrict__ corr)
{
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n_offs = (int64_t)C_in * COP;
    if (gid < n_offs) {
        const int ci = (int)(gid / COP), co = (int)(gid - (int64_t)ci * COP);
        const int k = co < C_out ? min((int)idx[(int64_t)co * C_in + ci], K - 1) : 0;
        offs[gid] = (uint16_t)(k * row_bytes);
    } else if (gid < n_offs + (int64_t)COP * 16) {
        const int q = (int)(gid - n_offs);
        const int co = q >> 4, type = q & 15;
        const uint32_t inv = border_invalid_window(type);
        int32_t s = 0;
        if (inv && co < C_out)
            for (int ci = 0; ci < C_in; ++ci) {
                const int k = min((int)idx[(int64_t)co * C_in + ci], K - 1);
                s += __popc(~code_to_window_order(codebook[k] & 511u) & inv);
            }
        corr[q] = s;
    } else if (gid < n_offs + (int64_t)COP * 16 + 512) {
        const int k = (int)(gid - n_offs - (int64_t)COP * 16);
        codes[k] = k < K ? code_to_window_order(codebook[k] & 511u) : 0u;
    }
}

// Where one output pixel's 3x3 window sits in the row-packed input.
struct PixGeom {
    int n;             // image
    int rowoff[3];     // h * WW of the three window rows (0 if the row is outside)
    uint32_t rowmask;  // bit dy set if window row dy is inside the image
    int j;             // word holding column wc - 1 (0 if wc == 0)
    int sh;            // bit of column wc - 1 in that word, or -1 if wc == 0
    bool need_hi;      // the three columns straddle two words
    uint32_t colmask;  // 3-bit mask of the window columns inside the image
};

__device__ inline PixGeom pix_geom(int64_t p, const Geom &g)
{
    PixGeom q;
    if (p >= g.P) p = g.P - 1;
    q.n = (int)(p / g.HoWo);
    const int r = (int)(p - (int64_t)q.n * g.HoWo);
    const int ho = r / g.Wo, wo = r - ho * g.Wo;
    const int hc = ho * g.stride, wc = wo * g.stride;
    q.rowmask = 0;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const int h = hc + dy - 1;
        const bool ok = h >= 0 && h < g.H;
        q.rowoff[dy] = ok ? h * g.WW : 0;
        q.rowmask |= ok ? (1u << dy) : 0u;
    }
    const int c = wc - 1;
    q.j = c >= 0 ? (c >> 5) : 0;
    q.sh = c >= 0 ? (c & 31) : -1;
    q.need_hi = q.sh > 29 && q.j + 1 < g.WW;
    q.colmask = (wc > 0 ? 1u : 0u) | 2u | (wc + 1 < g.W ? 4u : 0u);
    return q;
}

// 9-bit window of one (pixel, input channel): bit (3*dy + dx) = sign bit of x[h+dy-1][w+dx-1],
// 0 outside the image.
__device__ inline uint32_t window9(const uint32_t *__restrict__ x, const PixGeom &q, int ci, const Geom &g)
{
    const uint32_t *plane = x + ((int64_t)q.n * g.C_in + ci) * ((int64_t)g.H * g.WW);
    uint32_t win = 0;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const uint32_t *row = plane + q.rowoff[dy];
        const uint32_t lo = row[q.j];
        const uint32_t hi = q.need_hi ? row[q.j + 1] : 0u;
        const unsigned long long v = ((unsigned long long)hi << 32) | lo;
        uint32_t b3 = q.sh >= 0 ? (uint32_t)(v >> q.sh) : (lo << 1);
        b3 &= q.colmask;
        if (!((q.rowmask >> dy) & 1u)) b3 = 0;
        win |= b3 << (3 * dy);
    }
    return win;
}

// 4x4 byte transpose: in[i] byte b  ->  out[b] byte i.
__device__ inline void transpose4x4(const uint32_t in[4], uint32_t out[4])
{
    const uint32_t a_lo = __builtin_amdgcn_perm(in[1], in[0], 0x05010400u);
    const uint32_t a_hi = __builtin_amdgcn_perm(in[1], in[0], 0x07030602u);
    const uint32_t b_lo = __builtin_amdgcn_perm(in[3], in[2], 0x05010400u);
    const uint32_t b_hi = __builtin_amdgcn_perm(in[3], in[2], 0x07030602u);
    out[0] = __builtin_amdgcn_perm(b_lo, a_lo, 0x05040100u);
    out[1] = __builtin_amdgcn_perm(b_lo, a_lo, 0x07060302u);
    out[2] = __builtin_amdgcn_perm(b_hi, a_hi, 0x05040100u);
    out[3] = __builtin_amdgcn_perm(b_hi, a_hi, 0x07060302u);
}

template <int J, int NW, bool LUT>
__global__ __launch_bounds__(NW * 64)
void subbit_bin_kernel(const uint32_t *__restrict__ x, const uint32_t *__restrict__ codes,
                       const uint16_t *__restrict__ offs, const int32_t *__restrict__ corr,
                       const float *__restrict__ alpha, float *__restrict__ y, Geom g, int COP, int CIC)
{
    constexpr int NT = NW * 64;
    constexpr int COW = SB_CL * J;                 // output channels per wave
    extern __shared__ __align__(16) unsigned char smem[];
    const int K = g.K;
    const int KP = (K + 15) & ~15;                 // LUT row bytes
    // LDS: T [CIC][K][TP] bytes | (LUT ? lut [512][KP] bytes : win [CIC][TP] u16 + codes [K] u32)
    unsigned char *T = smem;
    unsigned char *aux = smem + (size_t)CIC * K * SB_TP;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t p_tile = (int64_t)blockIdx.x * SB_TP;
    const int co_wave = blockIdx.y * (COW * NW) + wave * COW;   // first channel of this wave

    // ---- set-up -----------------------------------------------------------------------------
    PixGeom geo[LUT ? 4 : 1];
    if (LUT) {
        unsigned char *lut = aux;
        // lut[window][k] = 9 - popcount(window ^ code_k); four k per word
        const int words_per_row = KP / 4;
        for (int i = tid; i < 512 * words_per_row; i += NT) {
            const int win = i / words_per_row, kq = i - win * words_per_row;
            uint32_t word = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int k = 4 * kq + b;
                const uint32_t m = k < K ? 9u - __popc((uint32_t)win ^ codes[k]) : 0u;
                word |= m << (8 * b);
            }
            ((uint32_t *)lut)[i] = word;
        }
        const int wd = tid & 15;
#pragma unroll
        for (int b = 0; b < 4; ++b) geo[b] = pix_geom(p_tile + 4 * wd + b, g);
    } else {
        uint32_t *lcodes = (uint32_t *)(aux + (size_t)CIC * SB_TP * sizeof(uint16_t));
        for (int i = tid; i < K; i += NT) lcodes[i] = codes[i];
        geo[0] = pix_geom(p_tile + (tid & 63), g);
    }

    uint32_t acc[J][4];
    uint32_t wide_e[J][4], wide_o[J][4];     // even / odd bytes of acc, as 16-bit pairs
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[j][w] = wide_e[j][w] = wide_o[j][w] = 0;

    const int g4 = lane & (SB_G - 1);
    const int cl = lane / SB_G;
    const int lane_co = co_wave + cl * J;          // first of this lane's J channels
    int since_widen = 0;

    __syncthreads();

    for (int c0 = 0; c0 < g.C_in; c0 += CIC) {
        const int nci = min(CIC, g.C_in - c0);

        // ---- stage 1: T[ci_l][k][pixel] for the chunk ------------------------------------------
        if (LUT) {
            const unsigned char *lut = aux;
            const int wd = tid & 15;
            for (int ci_l = tid >> 4; ci_l < nci; ci_l += NT / 16) {
                const uint4 *e[4];
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    e[b] = (const uint4 *)(lut + (size_t)window9(x, geo[b], c0 + ci_l, g) * KP);
                uint32_t *Tw = (uint32_t *)(T + (size_t)ci_l * K * SB_TP) + wd;
                for (int kv = 0; kv < KP / 16; ++kv) {
                    uint4 v[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) v[b] = e[b][kv];
                    const uint32_t in0[4] = {v[0].x, v[1].x, v[2].x, v[3].x};
                    const uint32_t in1[4] = {v[0].y, v[1].y, v[2].y, v[3].y};
                    const uint32_t in2[4] = {v[0].z, v[1].z, v[2].z, v[3].z};
                    const uint32_t in3[4] = {v[0].w, v[1].w, v[2].w, v[3].w};
                    uint32_t o[16];
                    transpose4x4(in0, o + 0);
                    transpose4x4(in1, o + 4);
                    transpose4x4(in2, o + 8);
                    transpose4x4(in3, o + 12);
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int k = 16 * kv + i;
                        if (k < K) Tw[k * (SB_TP / 4)] = o[i];
                    }
                }
            }
        } else {
            uint16_t *wins = (uint16_t *)aux;
            const uint32_t *lcodes = (const uint32_t *)(aux + (size_t)CIC * SB_TP * sizeof(uint16_t));
            for (int ci_l = tid >> 6; ci_l < nci; ci_l += NW)
                wins[ci_l * SB_TP + (tid & 63)] = (uint16_t)window9(x, geo[0], c0 + ci_l, g);
            __syncthreads();
            const int items = nci * K * (SB_TP / 4);
            for (int i = tid; i < items; i += NT) {
                const int wd = i & 15;
                const int k = (i >> 4) % K;
                const int ci_l = (i >> 4) / K;
                const uint2 w4 = *(const uint2 *)(wins + ci_l * SB_TP + 4 * wd);
                const uint32_t code = lcodes[k];
                const uint32_t m0 = 9u - __popc((w4.x & 0xffffu) ^ code);
                const uint32_t m1 = 9u - __popc((w4.x >> 16) ^ code);
                const uint32_t m2 = 9u - __popc((w4.y & 0xffffu) ^ code);
                const uint32_t m3 = 9u - __popc((w4.y >> 16) ^ code);
                ((uint32_t *)T)[i] = m0 | (m1 << 8) | (m2 << 16) | (m3 << 24);
            }
        }
        __syncthreads();

        // ---- stage 2: gather-accumulate ----------------------------------------------------------
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
        {
            const unsigned char *Tl = T + g4 * 16;
            const uint16_t *op = offs + (int64_t)c0 * COP + lane_co;
            for (int ci_l = 0; ci_l < nci; ++ci_l) {
                uint16_t o[J];
#pragma unroll
                for (int j = 0; j < J; ++j) o[j] = op[j];
#pragma unroll
                for (int j = 0; j < J; ++j) {
                    const uint4 v = *(const uint4 *)(Tl + o[j]);
                    acc[j][0] += v.x;
                    acc[j][1] += v.y;
                    acc[j][2] += v.z;
                    acc[j][3] += v.w;
                }
                Tl += (size_t)K * SB_TP;
                op += COP;
            }
        }
        __syncthreads();
    }

    // ---- epilogue: S = 2 * (M - corr) - C_in * valid_taps, y = float(S) * alpha ------------------
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
            wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
        }
    const int64_t p0 = p_tile + g4 * 16;
    if (p0 >= g.P) return;
    int n = (int)(p0 / g.HoWo);
    int r = (int)(p0 - (int64_t)n * g.HoWo);
    int ho = r / g.Wo, wo = r - ho * g.Wo;
    const bool vec4 = (g.HoWo & 3) == 0;
    float a[J];
#pragma unroll
    for (int j = 0; j < J; ++j) a[j] = lane_co + j < g.C_out ? alpha[lane_co + j] : 0.0f;

#pragma unroll
    for (int w = 0; w < 4; ++w) {
        float out[J][4];
        int rr[4], nn[4];
        bool ok[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            ok[b] = p0 + 4 * w + b < g.P;
            rr[b] = r;
            nn[b] = n;
            const int type = border_type(ho, wo, g.H, g.W, g.stride);
            const int base = border_valid_taps(type) * g.C_in;
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint32_t pair = (b & 1) ? wide_o[j][w] : wide_e[j][w];
                const int M = (int)((pair >> (16 * (b >> 1))) & 0xffffu);
                const int co = lane_co + j;
                const int cr = co < g.C_out ? corr[co * 16 + type] : 0;
                out[j][b] = (float)(2 * (M - cr) - base) * a[j];
            }
            // next pixel
            if (++wo == g.Wo) {
                wo = 0;
                if (++ho == g.Ho) { ho = 0; }
            }
            if (++r == g.HoWo) { r = 0; ++n; }
        }
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int co = lane_co + j;
            if (co >= g.C_out) continue;
            if (vec4 && ok[3]) {
                float4 *dst = (float4 *)(y + ((int64_t)nn[0] * g.C_out + co) * g.HoWo + rr[0]);
                *dst = make_float4(out[j][0], out[j][1], out[j][2], out[j][3]);
            } else {
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    if (ok[b]) y[((int64_t)nn[b] * g.C_out + co) * g.HoWo + rr[b]] = out[j][b];
            }
        }
    }
}

// ---- fp32 activations ---------------------------------------------------------------------------

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
                y[((int64_t)n * g.C_out + lane_co + j) * g.HoWo + r] = alpha[lane_co + j] * acc[j][b];
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

}  // namespace

size_t subbit_workspace_bytes(const Geom &g, int act)
{
    if (act == SNN_ACT_F32) {
        const F32Cfg c = pick_f32_cfg(g.C_out);
        const int COP = (g.C_out + c.COB - 1) / c.COB * c.COB;
        return align_up(512 * sizeof(uint32_t), 256) + align_up((size_t)g.C_in * COP * sizeof(uint16_t), 256) +
               align_up((size_t)COP * 16 * sizeof(int32_t), 256);
    }
    return carve_ws(g, nullptr).bytes;
}

int launch_subbit(const Geom &g, int act, const void *x, const uint16_t *codebook, const uint16_t *idx,
                  const float *alpha, float *y, void *ws, hipStream_t s)
{
    if (act == SNN_ACT_F32) {
        const F32Cfg c = pick_f32_cfg(g.C_out);
        const int COP = (g.C_out + c.COB - 1) / c.COB * c.COB;
        uint32_t *codes = (uint32_t *)ws;
        uint16_t *offs = (uint16_t *)((char *)ws + align_up(512 * sizeof(uint32_t), 256));
        int32_t *corr = (int32_t *)((char *)offs + align_up((size_t)g.C_in * COP * sizeof(uint16_t), 256));
        // T rows are 64 floats; offs counts floats (idx * 64), so K * 64 must fit 16 bits
        const int64_t tiles = (g.P + SF_TP - 1) / SF_TP;
        const int cblocks = COP / c.COB;
        if (tiles > 0x7fffffffLL || cblocks > 65535) return SNN_ERR_UNSUPPORTED;
        int CIC = 8;
        while (CIC > 1 && (size_t)CIC * g.K * SF_TP * sizeof(float) > 48 * 1024) CIC >>= 1;
        const size_t lds = (size_t)CIC * g.K * SF_TP * sizeof(float) + (size_t)g.K * 9 * sizeof(float);
        if (lds > 160 * 1024) return SNN_ERR_UNSUPPORTED;
        const int64_t nprep = (int64_t)g.C_in * COP + (int64_t)COP * 16 + 512;
        hipLaunchKernelGGL(subbit_prep_kernel, dim3((unsigned)((nprep + 255) / 256)), dim3(256), 0, s, codebook, idx,
                           g.C_in, g.C_out, COP, g.K, SF_TP, codes, offs, corr);
        const dim3 grid((unsigned)tiles, (unsigned)cblocks);
#define SNN_F32_CASE(J_)                                                                                       \
    case J_: {                                                                                                 \
        auto kern = subbit_f32_kernel<J_, 4>;                                                                  \
        if (lds > 64 * 1024 &&                                                                                 \
            hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=   \
                hipSuccess)                                                                                    \
            return SNN_ERR_LAUNCH;                                                                             \
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

    const SubbitCfg c = pick_cfg(g.C_out);
    const SubbitWs w = carve_ws(g, ws);
    const bool lut = g.K <= SB_LUT_MAXK;
    const int KP = (g.K + 15) & ~15;
    const int64_t tiles = (g.P + SB_TP - 1) / SB_TP;
    const int cblocks = w.COP / c.COB;
    if (tiles > 0x7fffffffLL || cblocks > 65535) return SNN_ERR_UNSUPPORTED;

    // input channels per chunk: a few KB of T per chunk, at most 8 so that three chunks fit
    // between two widenings
    int CIC = 8;
    while (CIC > 1 && (size_t)CIC * g.K * SB_TP > 32 * 1024) CIC >>= 1;
    const size_t lds = (size_t)CIC * g.K * SB_TP +
                       (lut ? (size_t)512 * KP : (size_t)CIC * SB_TP * sizeof(uint16_t) + (size_t)g.K * sizeof(uint32_t));
    if (lds > 160 * 1024) return SNN_ERR_UNSUPPORTED;

    const int64_t nprep = (int64_t)g.C_in * w.COP + (int64_t)w.COP * 16 + 512;
    hipLaunchKernelGGL(subbit_prep_kernel, dim3((unsigned)((nprep + 255) / 256)), dim3(256), 0, s, codebook, idx,
                       g.C_in, g.C_out, w.COP, g.K, SB_TP, w.codes, w.offs, w.corr);

    const dim3 grid((unsigned)tiles, (unsigned)cblocks);
    const uint32_t *xp = (const uint32_t *)x;
#define SNN_SB_LAUNCH(J_, NW_, LUT_)                                                                           \
    {                                                                                                          \
        auto kern = subbit_bin_kernel<J_, NW_, LUT_>;                                                          \
        if (lds > 64 * 1024 &&                                                                                 \
            hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=   \
                hipSuccess)                                                                                    \
            return SNN_ERR_LAUNCH;                                                                             \
        hipLaunchKernelGGL(kern, grid, dim3(NW_ * 64), lds, s, xp, w.codes, w.offs, w.corr, alpha, y, g,       \
                           w.COP, CIC);                                                                        \
    }
#define SNN_SB_CASE(J_, NW_)                                                                                   \
    if (c.J == J_ && c.NW == NW_) {                                                                            \
        if (lut) SNN_SB_LAUNCH(J_, NW_, true) else SNN_SB_LAUNCH(J_, NW_, false)                               \
    } else
    SNN_SB_CASE(1, 1)
    SNN_SB_CASE(1, 2)
    SNN_SB_CASE(1, 4)
    SNN_SB_CASE(2, 4)
    SNN_SB_CASE(4, 4)
    return SNN_ERR_UNSUPPORTED;
#undef SNN_SB_CASE
#undef SNN_SB_LAUNCH
    return check_launch();
}

}  // namespace snn
